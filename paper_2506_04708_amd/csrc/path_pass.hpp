// path_pass.hpp -- path_exact_kernel, path_finish_kernel, commit_scan_kernel: the accepted path, exact
// normalisers of its rows, observations, replay of the stop node and the resampled token (paper Sec. 3.2, 4.1).
#pragma once
#include "row_pass.hpp"
#include "table_merge.hpp"

namespace stand {

// ---------------------------------------------------------------------------------------------
// Path pass.  The accepted path of trajectory b follows `outcome` from the root (verify), or is
// given as commit rows (update).  For each path row the exact normaliser is needed (its
// observation is stored in the table), for the last one also the resampled token.
//   path_exact_kernel   block (seg, j, b): exact partial sum of a segment of path row j, stored in
//                       seg_part; the segments spread a handful of rows over all compute units
//   path_finish_kernel  block (j, b): adds the partial sums, writes the observation of the row;
//                       at the stop row it replays the node with exact probabilities and draws the
//                       resampled token by inverting the residual's cumulative integer mass.
//                       Further blocks of the same launch claim the table slots of the merge,
//                       which depends on the tokens of the path only.
// Kernel boundaries are the only synchronisation between blocks.
// ---------------------------------------------------------------------------------------------
constexpr int kSegMax = 32;  // most segments per path row
constexpr int kFinishThreads = 1024;  // path_finish_kernel: many waves, so that locating a token is one short round

struct PathArgs {
    const void *logits;
    int B, N, V, K, W, mode;   // mode 0: verify (path from outcome), 1: update (rows given)
    int R;                     // row slots per trajectory: W (slot j = path position j), or N when
    bool all_nodes;            // every drafted node's row is observed (slot j = node j)
    int nseg;                  // segments per path row (grid.x of path_exact_kernel)
    float c;
    uint64_t seed, step;
    TreeDev tree;
    const int32_t *draft_tok, *draft_has, *draft_qid;
    const float *draft_qmu;
    const float *src_m;        // mode 0: [B*N] by row; mode 1: [B*W] by (b, j)
    const int32_t *src_top_idx;
    const float *src_top_l;
    const int32_t *outcome;
    const int32_t *commit_row, *commit_len;  // mode 1
    int32_t *out_tok, *out_node, *out_len;   // mode 0
    unsigned long long *seg_part;  // [B][W][kSegMax] exact fixed-point partial sums
    // record of the stop node of each trajectory, gathered by path_exact_kernel so that
    // path_finish_kernel starts its replay after one round trip to memory
    int32_t *stop_i;           // [B][4] node, path length, drafted children, first child
    float *stop_m;             // [B] maximum of the stop row
    int32_t *stop_qid;         // [B][kMaxK] stored ids of the stop node's proposal (-1: none)
    float *stop_qmu;           // [B][kMaxK] their means
    float *stop_ql;            // [B][kMaxK] the stop row's logits at these ids
    int32_t *stop_child;       // [B][kMaxK] tokens of the drafted children (-1: none)
    int32_t *obs_idx;          // [B][W][K]
    float *obs_p;              // [B][W][K]
    unsigned long long *stats;
    unsigned long long *node_count;  // [N] verifications in which a node lay on the accepted path (mode 0)
    bool onehot;                     // deterministic drafting: one-hot proposals in the accept tests
    int late_len;                    // paths longer than this count as late (kStatLatePaths)
    int fx_shift;                    // the exact normaliser counts in units of 2^-(40 - fx_shift)
    // one-launch step: the rows' top-K as self-validating words of the same launch (RowPub), else NULL
    const unsigned long long *top_pub;
};

// Walks the accepted path of trajectory b and leaves it in path[0..len) (shared memory).  Must be
// called by the whole workgroup (verify mode only: src_m is indexed by row); returns len.
// Per-node data of one trajectory staged in shared memory by resolve_path: everything the walk
// and the code after it reads by node, fetched in one round trip.
struct PathStage {
    int oc[kMaxNodes];     // outcome: accepted child rank or -1
    int fc[kMaxNodes];     // first child
    int has[kMaxNodes];    // drafted children
    float m[kMaxNodes];    // row maximum
};
__device__ __forceinline__ int resolve_path(const PathArgs &a, int b, int *path, PathStage *st, int *len_sh)
{
    for (int u = threadIdx.x; u < a.N; u += blockDim.x) {
        st->oc[u] = a.outcome[(size_t)b * a.N + u];
        st->fc[u] = a.tree.first_child[u];
        st->has[u] = a.draft_has[(size_t)b * a.N + u];
        st->m[u] = a.src_m[(size_t)b * a.N + u];
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int cur = 0, len = 0;
        for (;;) {
            path[len++] = cur;
            const int acc = st->oc[cur];
            if (acc < 0 || len > a.tree.D) break;
            cur = st->fc[cur] + acc;
        }
        *len_sh = len;
    }
    __syncthreads();
    return *len_sh;
}

// tree node of path position j in update mode, or -1 if there is none
__device__ __forceinline__ int commit_row_of(const PathArgs &a, int b, int j)
{
    int cl = a.commit_len[b];
    cl = cl < 0 ? 0 : (cl > a.W ? a.W : cl);
    if (j >= cl) return -1;
    const int node = a.commit_row[(size_t)b * a.W + j];
    return (node < 0 || node >= a.N) ? -1 : node;
}

// Inclusive prefix sum over the 64 lanes of a wave, by data-parallel-primitive moves inside
// rows of 16 lanes and two row broadcasts (no LDS traffic).  A lane without a source adds 0.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ unsigned long long dpp_fetch_u64(unsigned long long x)
{
    const uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)x, CTRL, ROW_MASK, 0xF, false);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)(x >> 32), CTRL, ROW_MASK, 0xF, false);
    return ((unsigned long long)hi << 32) | lo;
}
__device__ __forceinline__ unsigned long long wave_inclusive_scan_u64(unsigned long long x)
{
    x += dpp_fetch_u64<0x111, 0xF>(x);  // row_shr:1
    x += dpp_fetch_u64<0x112, 0xF>(x);  // row_shr:2
    x += dpp_fetch_u64<0x114, 0xF>(x);  // row_shr:4
    x += dpp_fetch_u64<0x118, 0xF>(x);  // row_shr:8
    x += dpp_fetch_u64<0x142, 0xA>(x);  // row_bcast:15 into rows 1 and 3
    x += dpp_fetch_u64<0x143, 0xC>(x);  // row_bcast:31 into rows 2 and 3
    return x;
}
__device__ __forceinline__ unsigned long long wave_sum_u64(unsigned long long x)
{
    return readlane_u64(wave_inclusive_scan_u64(x), 63);
}
__device__ __forceinline__ unsigned long long fixed_mass(float e, int shift)
{
    uint32_t hi, lo;
    fixed_split(e, hi, lo);
    return ((unsigned long long)hi << (20 - shift)) + (lo >> shift);
}

template <int DT>
__global__ __launch_bounds__(kPathThreads) void path_exact_kernel(PathArgs a)
{
    constexpr int ES = VecTraits<DT>::ES;
    __shared__ int path[32];
    __shared__ PathStage stage;
    __shared__ int s_len;
    __shared__ unsigned long long s_part[kPathThreads / 64];
    // row slots are the slowest grid dimension: the workgroups of slot 0 (every trajectory has that
    // row) are dispatched before those of the later slots, most of which find no row
    const int seg = blockIdx.x, nseg = a.nseg, j = blockIdx.z, b = blockIdx.y, tid = threadIdx.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // scalar: the same in every lane
    if (seg == nseg) {
        // ---- the extra block of a trajectory (verify only): outputs and the stop record
        if (a.mode != 0 || j != 0) return;
        const int len = resolve_path(a, b, path, &stage, &s_len);
        // accepted tokens are the tokens of the path nodes after the root; the last emitted
        // token (position len - 1) is written by path_finish_kernel
        if (tid < a.W) {
            a.out_node[(size_t)b * a.W + tid] = tid < len ? path[tid] : -1;
            if (tid + 1 < len) a.out_tok[(size_t)b * a.W + tid] = a.draft_tok[(size_t)b * a.N + path[tid + 1]];
            else if (tid >= len) a.out_tok[(size_t)b * a.W + tid] = -1;
        }
        if (tid < len) atomicAdd(&a.node_count[path[tid]], 1ull);  // paper Sec. 4.3: acceptance statistics per node
        if (wave != 1) return;
        const int node = path[len - 1];
        const int row = b * a.N + node;
        const char *rowp = (const char *)a.logits + (size_t)row * (size_t)a.V * ES;
        const int fc = stage.fc[node];
        const int nch = stage.has[node];
        const float m = stage.m[node];
        int32_t qid = -1, ch = -1;
        float qmu = 0.0f, ql = 0.0f;
        if (lane < a.K) { qid = a.draft_qid[(size_t)row * a.K + lane]; qmu = a.draft_qmu[(size_t)row * a.K + lane]; }
        if (lane < nch && lane < kMaxK && fc >= 0 && fc + lane < a.N) ch = a.draft_tok[(size_t)b * a.N + fc + lane];
        if ((uint32_t)qid >= (uint32_t)a.V) { qid = -1; qmu = 0.0f; }  // never index outside the row
        else ql = load_scalar<DT>(rowp, qid);
        if (lane < kMaxK) {
            a.stop_qid[(size_t)b * kMaxK + lane] = qid; a.stop_qmu[(size_t)b * kMaxK + lane] = qmu;
            a.stop_ql[(size_t)b * kMaxK + lane] = ql; a.stop_child[(size_t)b * kMaxK + lane] = ch;
        }
        if (lane == 0) {
            a.stop_i[(size_t)b * 4 + 0] = node; a.stop_i[(size_t)b * 4 + 1] = len;
            a.stop_i[(size_t)b * 4 + 2] = nch; a.stop_i[(size_t)b * 4 + 3] = fc;
            a.stop_m[b] = m;
            a.out_len[b] = len;
            // accept tests along the path: rank + 1 at every accepted node, all children at the stop node
            unsigned long long tests = (unsigned long long)nch;
            for (int q = 0; q + 1 < len; ++q) tests += (unsigned long long)(stage.oc[path[q]] + 1);
            atomicAdd(&a.stats[kStatTokens], (unsigned long long)len);
            atomicAdd(&a.stats[kStatTests], tests);
            if (len > a.late_len) atomicAdd(&a.stats[kStatLatePaths], 1ull);
        }
        return;
    }
    // ---- partial sums of segment seg of the rows j, j + gridDim.z, ...; the root row needs no walk.
    // In verify mode the grid has only a few row slots: most paths are short, and a workgroup that
    // finds no row costs a launch slot; longer paths loop.
    int len = -1;  // path length once the walk has been done (verify mode, rows below the root)
    for (int jj = j; jj < a.R; jj += gridDim.z) {
        int node;
        bool staged = false;
        // (in verify mode the root row is always on the path, also when the trajectory has no context yet
        // and its root carries no token)
        if (a.all_nodes) node = (a.draft_tok[(size_t)b * a.N + jj] >= 0 || (a.mode == 0 && jj == 0)) ? jj : -1;
        else if (a.mode != 0) node = commit_row_of(a, b, jj);
        else if (jj == 0) node = 0;
        else {
            if (len < 0) {
                // (no separate look at the root's outcome first: that would be one more dependent round
                // trip to memory in front of the staging for every path that does go on)
                len = resolve_path(a, b, path, &stage, &s_len);
            }
            if (jj >= len) return;  // block-uniform; later rows do not exist either
            node = path[jj];
            staged = true;
        }
        if (node < 0) continue;  // block-uniform: no such row
        const int row = b * a.N + node;
        const char *rowp = (const char *)a.logits + (size_t)row * (size_t)a.V * ES;
        const float m = staged ? stage.m[node] : a.src_m[a.mode == 0 ? row : b * a.R + jj];
        const RowGeom g = row_geom<DT>(rowp, a.V);
        const int per = (g.nvec + nseg - 1) / nseg;
        const int v0 = seg * per < g.nvec ? seg * per : g.nvec;
        const int v1 = (v0 + per < g.nvec) ? v0 + per : g.nvec;
        unsigned long long S = thread_exact_partial<DT>(rowp, g, v0, v1, seg == 0, m, a.c, tid, kPathThreads, a.fx_shift);
        S = wave_sum_u64(S);
        __syncthreads();  // s_part of the previous row has been read
        if (lane == 0) s_part[wave] = S;
        __syncthreads();
        if (tid == 0) {
            unsigned long long t = 0ull;
            for (int q = 0; q < kPathThreads / 64; ++q) t += s_part[q];
            a.seg_part[((size_t)b * a.R + jj) * kSegMax + seg] = t;
        }
    }
}

struct FinishShared {
    unsigned long long P[kSegMax + 2];  // masked mass of: head elements, vector segments, tail elements
    unsigned long long wave_tot[kFinishThreads / 64];
    unsigned long long rem;             // position inside the chosen segment
    int32_t sup_id[kMaxK];              // stored ids that lie inside the chosen segment
    int nsup, seg, found;
    int32_t top0;                       // the row's best token
};

// masked integer masses of the EPV elements of vector idx (elements e0 .. e0 + EPV - 1 of the row)
template <int DT>
__device__ __forceinline__ void vector_masses(const uint4 &w, int e0, float m, float c, int shift, const FinishShared &sh,
                                              unsigned long long *f)
{
    constexpr int EPV = VecTraits<DT>::EPV;
    float x[EPV];
    unpack<DT>(w, x);
    uint32_t bits = 0u;
    for (int q = 0; q < sh.nsup; ++q) {
        const uint32_t d = (uint32_t)(sh.sup_id[q] - e0);
        if (d < (uint32_t)EPV) bits |= 1u << d;
    }
#pragma unroll
    for (int q = 0; q < EPV; ++q) f[q] = ((bits >> q) & 1u) ? 0ull : fixed_mass(exact_exp2(scaled_offset(x[q], m, c)), shift);
}
// Update mode: maximum and top-K of the given commit rows (one workgroup of 4 waves per row).
struct CommitScanArgs {
    const void *logits;
    int B, N, V, K, W, R;
    bool all_nodes;            // rows = the drafted nodes (slot j = node j) instead of the commit rows
    const int32_t *draft_tok;
    float c;
    const int32_t *commit_row, *commit_len;
    float *pr_m;          // [B*W]
    int32_t *pr_top_idx;  // [B*W][K]
    float *pr_top_l;      // [B*W][K]
};

template <int DT>
__global__ __launch_bounds__(256) void commit_scan_kernel(CommitScanArgs a)
{
    constexpr int ES = VecTraits<DT>::ES;
    __shared__ WaveScan wsh[4];
    __shared__ unsigned long long ebuf[kElemCap + 8];
    __shared__ int part_cnt[4];
    const int j = blockIdx.x, b = blockIdx.y, lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    int node;
    if (a.all_nodes) {
        if (a.draft_tok[(size_t)b * a.N + j] < 0) return;
        node = j;
    } else {
        int cl = a.commit_len[b];
        cl = cl < 0 ? 0 : (cl > a.W ? a.W : cl);
        if (j >= cl) return;
        node = a.commit_row[(size_t)b * a.W + j];
        if (node < 0 || node >= a.N) return;
    }
    const char *rowp = (const char *)a.logits + ((size_t)b * a.N + node) * (size_t)a.V * ES;
    WaveScan *ws = &wsh[wave];
    const WavePartial wp = wave_row_stream<DT>(rowp, a.V, a.c, a.K, ws, lane, wave, 4);
    if (lane == 0) part_cnt[wave] = wp.cnt;
    __syncthreads();
    if (wave != 0) return;
    int cnt = part_cnt[0];
    for (int q = 1; q < 4; ++q) {
        const int cq = part_cnt[q];
        if (lane < cq) ws->buf[cnt + lane] = wsh[q].buf[lane];
        cnt += cq;
    }
    __builtin_amdgcn_wave_barrier();
    wave_row_finish<DT>(rowp, a.V, a.K, ws, ebuf, lane, cnt);
    const size_t src = (size_t)b * a.R + j;
    if (lane < a.K) {
        a.pr_top_idx[src * a.K + lane] = (int32_t)rank_key_id(ws->top[lane]);
        a.pr_top_l[src * a.K + lane] = rank_key_value(ws->top[lane]);
    }
    if (lane == 0) a.pr_m[src] = rank_key_value(ws->top[0]);
}


// Finishes row slot j of trajectory b, whose row is tree node `node`: its observation (paper Sec. 4.1:
// top-k ids and probabilities with the exact normaliser) and, at the stop row of a verification, the
// replay of the node's accept tests with exact probabilities and the resampled token.  A row that is
// not a stop row is finished by ONE wave (wave = 0, tid = lane); the stop row by all NT threads of the
// workgroup, which all call this with their wave and thread numbers.  m: the row's maximum.  Wave 0's
// lanes hold the stop node's proposal (my_id, my_mu), the row's logits at those ids (my_l) and the
// tokens of the drafted children (ch); nch / fc / len as in the stop record.  `walked`: the node's outcome as
// the caller followed it (a path node that is not the stop node is replayed against it), or -2: read it from
// the row pass's results.
template <int DT, int NT>
__device__ __forceinline__ void finish_row(const PathArgs &a, FinishShared &sh, int b, int j, int node, bool stop, float m,
                                           int nch, int fc, int len, int32_t my_id, float my_mu, float my_l, int32_t ch,
                                           unsigned long long part, int tid, int wave, int walked = -2)
{
    constexpr int ES = VecTraits<DT>::ES, EPV = VecTraits<DT>::EPV;
    const int lane = tid & 63;
    const int nseg = a.nseg;
    const int row = b * a.N + node;
    const int src = a.mode == 0 ? row : b * a.R + j;
    const char *rowp = (const char *)a.logits + (size_t)row * (size_t)a.V * ES;
    const RowGeom g = row_geom<DT>(rowp, a.V);
    const int per = (g.nvec + nseg - 1) / nseg;

    if (wave == 0) {
        int32_t o_idx = 0;
        float o_l = 0.0f;
        if (lane < a.K) {
            if (a.top_pub) {
                // (the caller has seen these words carry this launch's mark)
                const unsigned long long tw = ld_agent(&a.top_pub[(size_t)src * a.K + lane]);
                o_idx = top_pub_id(tw); o_l = top_pub_logit(tw);
            } else {
                o_idx = a.src_top_idx[(size_t)src * a.K + lane]; o_l = a.src_top_l[(size_t)src * a.K + lane];
            }
        }
        if (stop && lane == 0) sh.top0 = o_idx;
        if (!stop || nch <= 0 || lane >= a.K) { my_id = -1; my_mu = 0.0f; }
        const float my_e = my_id >= 0 ? exact_exp2(scaled_offset(my_l, m, a.c)) : 0.0f;
        int edge_id = -1;
        if (stop) {
            if (lane < g.head) edge_id = lane;
            else if (lane < g.head + g.ntail) edge_id = g.tail0 + (lane - g.head);
        }
        const unsigned long long edge_f =
            edge_id >= 0 ? fixed_mass(exact_exp2(scaled_offset(load_scalar<DT>(rowp, edge_id), m, a.c)), a.fx_shift) : 0ull;

        const unsigned long long S = wave_sum_u64(part);
        const float s = normaliser_from_fixed(S, a.fx_shift);
        if (!stop) {
            // observation of this row (paper Sec. 4.1: top-k ids and probabilities)
            if (lane < a.K) {
                st_agent(&a.obs_idx[((size_t)b * a.R + j) * a.K + lane], o_idx);
                st_agent(&a.obs_p[((size_t)b * a.R + j) * a.K + lane], exact_exp2(scaled_offset(o_l, m, a.c)) / s);
            }
            if (a.mode == 0 && a.draft_has[row] > 0) {
                // self-check of the row pass's decision at this node (taken with the fast normaliser and its
                // error bound): the accept tests again with exact probabilities must name the same child
                const int c_n = a.draft_has[row], c_fc = a.tree.first_child[node];
                int32_t c_id = -1, c_ch = -1;
                float c_mu = 0.0f, c_l = 0.0f;
                if (lane < a.K) { c_id = a.draft_qid[(size_t)row * a.K + lane]; c_mu = a.draft_qmu[(size_t)row * a.K + lane]; }
                if (lane < c_n && lane < kMaxK && c_fc >= 0 && c_fc + lane < a.N) c_ch = a.draft_tok[(size_t)b * a.N + c_fc + lane];
                if ((uint32_t)c_id >= (uint32_t)a.V) { c_id = -1; c_mu = 0.0f; }  // never index outside the row
                else c_l = load_scalar<DT>(rowp, c_id);
                const float c_e = c_id >= 0 ? exact_exp2(scaled_offset(c_l, m, a.c)) : 0.0f;
                const NodeResult nr = wave_node_outcome(lane, a.K, c_id, c_mu, c_e / s, c_n, c_ch, a.seed, (uint32_t)b, a.step, c_fc,
                                                        false, 0.0f, a.onehot);
                if (lane == 0 && nr.accepted != (walked != -2 ? walked : a.outcome[row])) atomicAdd(&a.stats[kStatMismatch], 1ull);
            }
            return;
        }

        // ---- residual at the stop node: replay its accept sequence with exact probabilities
        bool support = nch > 0;
        float my_r = 0.0f, rho = 1.0f;
        if (support) {
            const NodeResult nr = wave_node_outcome(lane, a.K, my_id, my_mu, my_e / s, nch, ch, a.seed, (uint32_t)b, a.step,
                                                    fc, false, 0.0f, a.onehot);
            my_r = (lane < a.K && my_id >= 0) ? nr.r : 0.0f;
            rho = nr.rho;
            if (lane == 0 && nr.accepted != -1) atomicAdd(&a.stats[kStatMismatch], 1ull);  // the stop node rejects all
            // a residual that is not a distribution any more (the normalising mass underflowed)
            // is not used
            const float rs = wave_tree_sum(my_r);
            if (!(rs <= 2.0f) || !(rho < __builtin_inff())) support = false;
        }
        // the stop row's observation (its loads have had the replay to arrive)
        if (lane < a.K) {
            st_agent(&a.obs_idx[((size_t)b * a.R + j) * a.K + lane], o_idx);
            st_agent(&a.obs_p[((size_t)b * a.R + j) * a.K + lane], exact_exp2(scaled_offset(o_l, m, a.c)) / s);
        }
        // ---- integer masses (unit 2^-(40 - fx_shift) / s * rho): support token i weighs floor(r_i * (S / rho)),
        // a token outside the support the term it contributes to S
        const bool has_edge = g.head + g.ntail > 0;  // rows that start on a 16-byte boundary have none
        const unsigned long long edge_all = has_edge ? wave_sum_u64(edge_f) : 0ull;
        unsigned long long my_g = 0ull, g_inc = 0ull, gsum = 0ull, T = 0ull, edge_m = 0ull;
        for (int attempt = 0; attempt < 2; ++attempt) {
            unsigned long long my_f = 0ull;
            int my_ps = -1;  // 0: head elements, 1 + q: vector segment q, nseg + 1: tail elements
            my_g = 0ull;
            if (support && lane < a.K && my_id >= 0) {
                const double ratio = (double)S / (double)rho;  // skipped by the whole wave without a support
                my_g = (unsigned long long)((double)my_r * ratio);
                my_f = fixed_mass(my_e, a.fx_shift);
                my_ps = my_id < g.head ? 0 : (my_id >= g.tail0 ? nseg + 1 : 1 + ((my_id - g.head) / EPV) / per);
            }
            unsigned long long head_m = 0ull, tail_m = 0ull;
            if (has_edge) {
                bool edge_in_support = false;
                if (support)
                    for (int q = 0; q < a.K; ++q) edge_in_support |= __builtin_amdgcn_readlane(my_id, q) == edge_id;
                edge_m = (edge_id >= 0 && !edge_in_support) ? edge_f : 0ull;
                head_m = wave_sum_u64(lane < g.head ? edge_m : 0ull);
                tail_m = wave_sum_u64(lane >= g.head ? edge_m : 0ull);
            }
            if (lane < nseg) sh.P[1 + lane] = part - (lane == 0 ? edge_all : 0ull);
            if (lane == 0) { sh.P[0] = head_m; sh.P[nseg + 1] = tail_m; }
            __builtin_amdgcn_wave_barrier();
            if (my_ps >= 1 && my_ps <= nseg) atomicAdd(&sh.P[my_ps], 0ull - my_f);
            __builtin_amdgcn_wave_barrier();
            // every support token lies in exactly one part, so the masked parts add up to S - sum my_f
            g_inc = wave_inclusive_scan_u64(my_g);
            gsum = readlane_u64(g_inc, 63);
            T = S + gsum - wave_sum_u64(my_f);
            if (!support || T != 0ull) break;
            support = false;  // the residual vanished: draw from the target itself
        }
        const Philox4 ph = philox_group(a.seed, (uint32_t)b, a.step, (uint32_t)node, 0u, kStreamBonus);
        const unsigned long long u = ((unsigned long long)ph.x << 32) | ph.y;
        unsigned long long t = __umul64hi(u, T);
        int32_t token = -1;
        int seg = -1;
        if (t < gsum) {
            const int win = __ffsll((long long)__ballot(t < g_inc)) - 1;
            token = __builtin_amdgcn_readlane(my_id, win);
        } else {
            t -= gsum;
            const unsigned long long pv = lane < nseg + 2 ? sh.P[lane] : 0ull;
            const unsigned long long inc = wave_inclusive_scan_u64(pv);
            int win = __ffsll((long long)__ballot(lane < nseg + 2 && t < inc)) - 1;
            if (win < 0) win = 1;  // not reachable: t is below the total mass
            const unsigned long long rem = t - (readlane_u64(inc, win) - readlane_u64(pv, win));
            if (win == 0 || win == nseg + 1) {
                // inside the head or the tail elements: lanes hold them in id order
                const unsigned long long em = ((win == 0) == (lane < g.head)) ? edge_m : 0ull;
                const unsigned long long einc = wave_inclusive_scan_u64(em);
                const int ew = __ffsll((long long)__ballot(rem < einc)) - 1;
                token = ew >= 0 ? __builtin_amdgcn_readlane(edge_id, ew) : __builtin_amdgcn_readlane(o_idx, 0);
            } else {
                seg = win - 1;
                // stored ids inside the chosen segment
                const int e_lo = g.head + seg * per * EPV, e_hi = e_lo + per * EPV;
                const bool in_seg = support && lane < a.K && my_id >= e_lo && my_id < e_hi && my_id < g.tail0;
                const unsigned long long mk = __ballot(in_seg);
                if (in_seg) sh.sup_id[lane_prefix_count(mk)] = my_id;
                if (lane == 0) { sh.nsup = __popcll(mk); sh.rem = rem; }
            }
        }
        if (lane == 0) {
            sh.seg = seg;
            sh.found = 0;
            if (seg < 0) a.out_tok[(size_t)b * a.W + (len - 1)] = token;
        }
    }
    __syncthreads();
    const int seg = sh.seg;
    if (seg < 0) return;

    // ---- locate the token inside vector segment seg: every thread owns a contiguous run of
    // vectors, so thread order is id order
    const int vs = seg * per, ve = (vs + per < g.nvec) ? vs + per : g.nvec;
    const int cpt = (ve - vs + NT - 1) / NT;
    const int r0 = vs + tid * cpt < ve ? vs + tid * cpt : ve;
    const int r1 = r0 + cpt < ve ? r0 + cpt : ve;
    // four independent loads per round (indices clamped, unused vectors skipped)
    const int rlast = r1 > r0 ? r1 - 1 : r0;
    unsigned long long mine = 0ull;
    auto vec_sum = [&](const uint4 &w, int idx) {
        if (idx < r1) {
            unsigned long long f[EPV];
            vector_masses<DT>(w, g.head + idx * EPV, m, a.c, a.fx_shift, sh, f);
#pragma unroll
            for (int q = 0; q < EPV; ++q) mine += f[q];
        }
    };
    uint4 w0 = make_uint4(0, 0, 0, 0), w1 = w0, w2 = w0, w3 = w0;  // the last round's vectors are kept
    unsigned long long f1[EPV];  // cpt == 1 (the usual case): the masses of this thread's only vector are kept
#pragma unroll
    for (int q = 0; q < EPV; ++q) f1[q] = 0ull;
    if (cpt == 1) {
        if (r0 < r1) {
            vector_masses<DT>(g.vp[r0], g.head + r0 * EPV, m, a.c, a.fx_shift, sh, f1);
#pragma unroll
            for (int q = 0; q < EPV; ++q) mine += f1[q];
        }
    } else if (r0 < r1)
        for (int base = r0; base < r1; base += 4) {
            w0 = g.vp[base < rlast ? base : rlast];
            w1 = g.vp[base + 1 < rlast ? base + 1 : rlast];
            w2 = g.vp[base + 2 < rlast ? base + 2 : rlast];
            w3 = g.vp[base + 3 < rlast ? base + 3 : rlast];
            vec_sum(w0, base); vec_sum(w1, base + 1); vec_sum(w2, base + 2); vec_sum(w3, base + 3);
        }
    const unsigned long long inc = wave_inclusive_scan_u64(mine);
    if (lane == 63) sh.wave_tot[wave] = inc;
    __syncthreads();
    unsigned long long before = inc - mine;
    for (int q = 0; q < wave; ++q) before += sh.wave_tot[q];
    const unsigned long long rem = sh.rem;
    if (rem >= before && rem - before < mine) {
        unsigned long long left = rem - before;
        int32_t token = -1;
        auto vec_find = [&](const uint4 &w, int idx) {
            if (idx < r1 && token < 0) {
                unsigned long long f[EPV];
                vector_masses<DT>(w, g.head + idx * EPV, m, a.c, a.fx_shift, sh, f);
#pragma unroll
                for (int q = 0; q < EPV; ++q) {
                    if (token < 0) {
                        if (left < f[q]) token = g.head + idx * EPV + q;
                        else left -= f[q];
                    }
                }
            }
        };
        const bool single_round = r1 - r0 <= 4;  // then w0..w3 still hold this thread's whole run
        if (cpt == 1) {
#pragma unroll
            for (int q = 0; q < EPV; ++q) {
                if (token < 0) {
                    if (left < f1[q]) token = g.head + r0 * EPV + q;
                    else left -= f1[q];
                }
            }
        } else
        for (int base = r0; base < r1 && token < 0; base += 4) {
            if (!single_round) {
                w0 = g.vp[base < rlast ? base : rlast];
                w1 = g.vp[base + 1 < rlast ? base + 1 : rlast];
                w2 = g.vp[base + 2 < rlast ? base + 2 : rlast];
                w3 = g.vp[base + 3 < rlast ? base + 3 : rlast];
            }
            vec_find(w0, base); vec_find(w1, base + 1); vec_find(w2, base + 2); vec_find(w3, base + 3);
        }
        a.out_tok[(size_t)b * a.W + (len - 1)] = token;
        sh.found = 1;
    }
    __syncthreads();
    if (tid == 0 && !sh.found) {
        // not reachable while the partial sums describe this row; keep the output a valid token
        a.out_tok[(size_t)b * a.W + (len - 1)] = sh.top0;
        atomicAdd(&a.stats[kStatMismatch], 1ull);
    }
}

// See the comment above PathArgs.  Blocks [0, finish_blocks) finish row slot j of trajectory b with
// (j, b) = (block / B, block % B); the blocks after them claim merge records, kFinishThreads per block.
template <int DT>
__global__ __launch_bounds__(kFinishThreads) void path_finish_kernel(PathArgs a, MergeArgs mg, int finish_blocks)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    if ((int)blockIdx.x >= finish_blocks) {
        merge_claim_record(mg, ((int)blockIdx.x - finish_blocks) * kFinishThreads + tid);
        return;
    }
    __shared__ FinishShared sh;
    const int j = (int)blockIdx.x / a.B, b = (int)blockIdx.x % a.B;  // slot-major, as in path_exact_kernel
    // Everything whose address depends on (b, j) only is requested at once: the partial sums and,
    // in verify mode, the stop record of the trajectory (used if this turns out to be its stop row).
    const unsigned long long part = (wave == 0 && lane < a.nseg) ? ld_agent(&a.seg_part[((size_t)b * a.R + j) * kSegMax + lane]) : 0ull;
    int len = 0, node, nch = 0, fc = -1;
    bool stop = false;
    int32_t my_id = -1, ch = -1;
    float my_mu = 0.0f, my_l = 0.0f, m;
    if (a.mode == 0) {
        const int stop_node = a.stop_i[(size_t)b * 4 + 0];
        len = a.stop_i[(size_t)b * 4 + 1];
        nch = a.stop_i[(size_t)b * 4 + 2];
        fc = a.stop_i[(size_t)b * 4 + 3];
        m = a.stop_m[b];
        if (wave == 0 && lane < kMaxK) {
            my_id = a.stop_qid[(size_t)b * kMaxK + lane]; my_mu = a.stop_qmu[(size_t)b * kMaxK + lane];
            my_l = a.stop_ql[(size_t)b * kMaxK + lane]; ch = a.stop_child[(size_t)b * kMaxK + lane];
        }
        // all-nodes mode: slot j = node j; an undrafted root (empty context) is still the stop row
        if (a.all_nodes) node = (a.draft_tok[(size_t)b * a.N + j] >= 0 || j == 0) ? j : -1;
        else node = j < len ? (j == len - 1 ? stop_node : a.out_node[(size_t)b * a.W + j]) : -1;
        stop = node >= 0 && node == stop_node;
    } else {
        node = a.all_nodes ? (a.draft_tok[(size_t)b * a.N + j] >= 0 ? j : -1) : commit_row_of(a, b, j);
        m = 0.0f;
    }
    if (node < 0) return;  // block-uniform
    if (!stop && wave != 0) return;
    if (!stop) m = a.src_m[a.mode == 0 ? b * a.N + node : b * a.R + j];
    finish_row<DT, kFinishThreads>(a, sh, b, j, node, stop, m, nch, fc, len, my_id, my_mu, my_l, ch, part, tid, wave);
}

}  // namespace stand
