// kernels.hpp -- HIP kernels of the STAND speculation step for gfx950 (wave64).
//
//   row_pass_kernel   softmax statistics + top-K of every logits row in one streaming pass, and
//                     the accept/reject outcome of the row's tree node        (paper Sec. 4.1, 3.2)
//   path_pass_kernel  exact normaliser + observation of the rows on the accepted path, and the
//                     resampled token at the stop node                        (paper Sec. 3.2, 4.1)
//   merge_*           running-mean merge into the open-addressing table       (paper Sec. 4.1)
//   draft_kernel      multi-level lookup + Gumbel-Top-K along the static tree (paper Sec. 4.2)
//
// The row pass is the only kernel that touches all of the logits; it is bound by HBM bandwidth.
// Its softmax normaliser uses the hardware exp2 and float accumulation (relative error far
// below the 5e-5 bound used here); every accept test whose margin is inside that bound, and
// every probability that is stored in the table or used for resampling, is recomputed with
// the exact integer normaliser of numeric.hpp, so all decisions are those of exact arithmetic.
#pragma once
#include "numeric.hpp"

namespace stand {

constexpr int kDtBf16 = 0, kDtF32 = 1;
constexpr int kCap = 2048;      // candidate buffer entries per workgroup (>= kRefresh + largest block)
constexpr int kRefresh = 256;   // prune the buffer when it holds more than this
constexpr int kRowThreads = 256;
constexpr int kPathThreads = 1024;
constexpr float kFastEps = 5e-5f;  // bound on the relative error of the fast normaliser

enum StatSlot {
    kStatHits = 0,  // kStatHits + n, n = 1..8
    kStatMisses = 9, kStatInserts, kStatMerges, kStatDrops, kStatNear, kStatTokens, kStatTests, kStatMismatch,
    kStatCount
};

struct TreeDev {
    const int32_t *parent, *depth, *nchild, *first_child, *level_start;  // level_start[D+2]
    int N, D;
};

// One table slot = 16-byte header + K ids + K probabilities.
struct SlotHeader { unsigned long long fp; uint32_t count; uint32_t order; };

__device__ __forceinline__ SlotHeader *slot_header(char *table, uint64_t slot, int slot_bytes)
{
    return (SlotHeader *)(table + slot * (uint64_t)slot_bytes);
}
__device__ __forceinline__ int32_t *slot_ids(char *table, uint64_t slot, int slot_bytes)
{
    return (int32_t *)(table + slot * (uint64_t)slot_bytes + 16);
}
__device__ __forceinline__ float *slot_mu(char *table, uint64_t slot, int slot_bytes, int K)
{
    return (float *)(table + slot * (uint64_t)slot_bytes + 16 + 4 * K);
}

// ---------------------------------------------------------------------------------------------
// Workgroup-level streaming scan of one row: running max / sum (fast) and exact top-K.
// ---------------------------------------------------------------------------------------------
struct ScanShared {
    unsigned long long buf[kCap];
    unsigned long long top[kMaxK];
    unsigned long long theta_key;
    unsigned long long acc64;
    uint32_t cnt;
    int flag;
    float red[32];
    float tmp[kMaxK];
};

// Keeps the K best of the n candidates in sh.buf (sorted into sh.top and copied back) and sets
// sh.theta_key to the K-th best (0 if n < K).  Precondition: a barrier has passed since the last
// push, every thread holds the same n == sh.cnt, and nobody touches sh until the call returns.
template <int BS>
__device__ __noinline__ uint32_t wg_select_topk(ScanShared &sh, int K, uint32_t n_in)
{
    const int tid = threadIdx.x;
    const int n = (int)n_in;
    for (int i = tid; i < n; i += BS) {
        unsigned long long a = sh.buf[i];
        int r = 0;
        for (int j = 0; j < n; ++j) r += (sh.buf[j] > a) ? 1 : 0;
        if (r < K) sh.top[r] = a;
    }
    __syncthreads();
    const int keep = n < K ? n : K;
    if (tid < keep) sh.buf[tid] = sh.top[tid];
    if (tid == 0) {
        sh.cnt = (uint32_t)keep;
        sh.theta_key = (n >= K) ? sh.top[K - 1] : 0ull;
    }
    __syncthreads();
    return (uint32_t)keep;
}

__device__ __forceinline__ void push_candidate(ScanShared &sh, float val, uint32_t id, unsigned long long thr)
{
    unsigned long long key = rank_key(val, id);
    if (key > thr) {
        uint32_t pos = atomicAdd(&sh.cnt, 1u);
        if (pos < (uint32_t)kCap) sh.buf[pos] = key;
    }
}

template <int DT> struct VecTraits;
template <> struct VecTraits<kDtBf16> { static constexpr int ES = 2, EPV = 8; };
template <> struct VecTraits<kDtF32> { static constexpr int ES = 4, EPV = 4; };

template <int DT>
__device__ __forceinline__ void unpack(const uint4 &w, float *x)
{
    if constexpr (DT == kDtBf16) {
        x[0] = u2f(w.x << 16); x[1] = u2f(w.x & 0xFFFF0000u);
        x[2] = u2f(w.y << 16); x[3] = u2f(w.y & 0xFFFF0000u);
        x[4] = u2f(w.z << 16); x[5] = u2f(w.z & 0xFFFF0000u);
        x[6] = u2f(w.w << 16); x[7] = u2f(w.w & 0xFFFF0000u);
    } else {
        x[0] = u2f(w.x); x[1] = u2f(w.y); x[2] = u2f(w.z); x[3] = u2f(w.w);
    }
}

template <int DT>
__device__ __forceinline__ float load_scalar(const void *rowp, int v)
{
    if constexpr (DT == kDtBf16) return u2f((uint32_t)((const uint16_t *)rowp)[v] << 16);
    else return ((const float *)rowp)[v];
}

// Geometry of a row in memory: scalar head up to 16-byte alignment, aligned vectors, scalar tail.
struct RowGeom {
    int head, nvec, tail0, ntail;
    const uint4 *vp;
};
template <int DT>
__device__ __forceinline__ RowGeom row_geom(const void *rowp, int V)
{
    constexpr int ES = VecTraits<DT>::ES, EPV = VecTraits<DT>::EPV;
    RowGeom g;
    uintptr_t addr = (uintptr_t)rowp;
    g.head = (int)(((16 - (addr & 15)) & 15) / ES);
    if (g.head > V) g.head = V;
    g.nvec = (V - g.head) / EPV;
    g.tail0 = g.head + g.nvec * EPV;
    g.ntail = V - g.tail0;
    g.vp = (const uint4 *)((const char *)rowp + (size_t)g.head * ES);
    return g;
}

__device__ __forceinline__ float fast_exp2(float y) { return __builtin_amdgcn_exp2f(y); }

// Returns through m_out the exact row maximum, through s_out the fast normaliser
// sum_v 2^((l_v - m) c); leaves the K best (value desc, id asc) keys sorted in sh.top[0..K).
template <int DT, int BS>
__device__ void wg_row_scan(const void *rowp, int V, float c, int K, ScanShared &sh, float &m_out, float &s_out)
{
    constexpr int EPV = VecTraits<DT>::EPV;
    constexpr int U = 4;
    const int tid = threadIdx.x;
    const RowGeom g = row_geom<DT>(rowp, V);

    if (tid == 0) { sh.cnt = 0; sh.theta_key = 0ull; }
    __syncthreads();

    float m_t = -3.402823466e38f, s_t = 0.0f, nb = 0.0f;  // nb = -m_t * c once a finite value was seen
    auto absorb_max = [&](float cm) {
        if (cm > m_t) {
            s_t *= fast_exp2((m_t - cm) * c);
            m_t = cm;
            nb = -cm * c;
        }
    };

    // the scalar edge element of this thread, if any (only threads < head + ntail have one)
    float edge_val = 0.0f;
    int edge_id = -1;
    if (tid < g.head) edge_id = tid;
    else if (tid < g.head + g.ntail) edge_id = g.tail0 + (tid - g.head);
    if (edge_id >= 0) {
        edge_val = load_scalar<DT>(rowp, edge_id);
        absorb_max(edge_val);
        s_t += fast_exp2(__builtin_fmaf(edge_val, c, nb));
    }

    // Shared state is only read between two barriers and only written (pushes aside) by
    // wg_select_topk or thread 0 between two barriers; `cnt` mirrors sh.cnt at those points.
    uint32_t cnt = 0;
    bool first = true;
    for (int base = 0; base < g.nvec || first; base += BS * U) {
        uint4 w[U];
        bool ok[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            int idx = base + u * BS + tid;
            ok[u] = idx < g.nvec;
            if (ok[u]) w[u] = g.vp[idx];
        }
        const uint32_t cnt0 = cnt;
        const unsigned long long theta = sh.theta_key;
        const float theta_val = theta ? rank_key_value(theta) : -__builtin_inff();

        // ---- softmax statistics + candidate filter
        unsigned long long best = 0ull;  // best key of this thread (seeding only)
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (!ok[u]) continue;
            float x[EPV];
            unpack<DT>(w[u], x);
            float cm = x[0];
#pragma unroll
            for (int j = 1; j < EPV; ++j) cm = fmaxf(cm, x[j]);
            absorb_max(cm);
#pragma unroll
            for (int j = 0; j < EPV; ++j) s_t += fast_exp2(__builtin_fmaf(x[j], c, nb));
            const uint32_t id0 = (uint32_t)(g.head + (base + u * BS + tid) * EPV);
            if (first) {
#pragma unroll
                for (int j = 0; j < EPV; ++j) {
                    unsigned long long k = rank_key(x[j], id0 + j);
                    best = k > best ? k : best;
                }
            } else if (cm >= theta_val) {
#pragma unroll
                for (int j = 0; j < EPV; ++j)
                    if (x[j] >= theta_val) push_candidate(sh, x[j], id0 + j, theta);
            }
        }

        unsigned long long thr = theta;  // strict threshold for a replay of this super-iteration
        if (first) {
            // seed: the K-th best of the per-thread maxima bounds the K-th best element from below
            if (edge_id >= 0) {
                unsigned long long k = rank_key(edge_val, (uint32_t)edge_id);
                best = k > best ? k : best;
            }
            if (best) { uint32_t pos = atomicAdd(&sh.cnt, 1u); sh.buf[pos] = best; }
            __syncthreads();
            const uint32_t nseed = sh.cnt;
            __syncthreads();
            wg_select_topk<BS>(sh, K, nseed);
            thr = sh.theta_key ? sh.theta_key - 1ull : 0ull;
            __syncthreads();
            if (tid == 0) sh.cnt = 0;
            __syncthreads();
            if (edge_id >= 0) push_candidate(sh, edge_val, (uint32_t)edge_id, thr);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (!ok[u]) continue;
                float x[EPV];
                unpack<DT>(w[u], x);
                const uint32_t id0 = (uint32_t)(g.head + (base + u * BS + tid) * EPV);
#pragma unroll
                for (int j = 0; j < EPV; ++j) push_candidate(sh, x[j], id0 + j, thr);
            }
        }
        __syncthreads();
        cnt = sh.cnt;
        __syncthreads();
        if (cnt > (uint32_t)kCap) {
            // More candidates than the buffer holds (e.g. an ascending run): replay this
            // super-iteration one element per thread at a time, pruning in between.
            cnt = first ? 0u : cnt0;
            if (tid == 0) sh.cnt = cnt;
            __syncthreads();
            if (first && edge_id >= 0) push_candidate(sh, edge_val, (uint32_t)edge_id, thr);
#pragma unroll
            for (int u = 0; u < U; ++u) {
#pragma unroll
                for (int j = 0; j < EPV; ++j) {
                    if (ok[u]) {
                        float x[EPV];
                        unpack<DT>(w[u], x);
                        push_candidate(sh, x[j], (uint32_t)(g.head + (base + u * BS + tid) * EPV + j), thr);
                    }
                    __syncthreads();
                    cnt = sh.cnt;
                    __syncthreads();
                    if (cnt > (uint32_t)kRefresh) {
                        cnt = wg_select_topk<BS>(sh, K, cnt);
                        if (sh.theta_key) thr = sh.theta_key;  // the K-th best is in the buffer now: strict
                        __syncthreads();
                    }
                }
            }
        }
        if (first || cnt > (uint32_t)kRefresh) cnt = wg_select_topk<BS>(sh, K, cnt);
        first = false;
    }
    wg_select_topk<BS>(sh, K, cnt);  // leaves sh.top[0..min(K, V)) sorted

    const float m = rank_key_value(sh.top[0]);
    float part = s_t * fast_exp2((m_t - m) * c);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) part += __shfl_xor(part, off);
    if ((tid & 63) == 0) sh.red[tid >> 6] = part;
    __syncthreads();
    float s = 0.0f;
    for (int wv = 0; wv < BS / 64; ++wv) s += sh.red[wv];
    __syncthreads();
    m_out = m;
    s_out = s;
}

// Exact normaliser of a row whose maximum is known: S = sum_v floor(E((l_v - m) c) * 2^F).
template <int DT, int BS>
__device__ unsigned long long wg_row_exact_sum(const void *rowp, int V, float m, float c, unsigned long long *acc /* LDS */)
{
    constexpr int EPV = VecTraits<DT>::EPV;
    const int tid = threadIdx.x;
    const int F = fixed_bits(V);
    const RowGeom g = row_geom<DT>(rowp, V);
    if (tid == 0) *acc = 0ull;
    __syncthreads();
    unsigned long long S = 0ull;
    int edge_id = -1;
    if (tid < g.head) edge_id = tid;
    else if (tid < g.head + g.ntail) edge_id = g.tail0 + (tid - g.head);
    if (edge_id >= 0) S += fixed_contrib(exact_exp2(scaled_offset(load_scalar<DT>(rowp, edge_id), m, c)), F);
    for (int idx = tid; idx < g.nvec; idx += BS) {
        float x[EPV];
        unpack<DT>(g.vp[idx], x);
#pragma unroll
        for (int j = 0; j < EPV; ++j) S += fixed_contrib(exact_exp2(scaled_offset(x[j], m, c)), F);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) S += __shfl_xor(S, off);
    if ((tid & 63) == 0) atomicAdd(acc, S);
    __syncthreads();
    unsigned long long total = *acc;
    __syncthreads();
    return total;
}

// ---------------------------------------------------------------------------------------------
// Accept/reject sequence at one tree node, executed by one wave (lane i = stored id i).
// Returns the rank of the accepted child or -1.  With track_err the values r are taken to
// carry a relative error of at most eps and `near` reports a test that the error could flip.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ float wave_ordered_sum(float x, int lane, int K, float *tmp)
{
    // LDS operations of one wave execute in order, so the reads below see the writes
    if (lane < K) tmp[lane] = x;
    __builtin_amdgcn_wave_barrier();
    float t = 0.0f;
    for (int i = 0; i < K; ++i) t = t + tmp[i];
    __builtin_amdgcn_wave_barrier();
    return t;
}

struct NodeResult { int accepted; int rounds; bool near; float r; float rho; };

__device__ __forceinline__ NodeResult wave_node_outcome(int lane, int K, int32_t my_id, float my_mu, float my_p, int nchild,
                                        const int32_t *child_tok, uint64_t seed, uint32_t b, uint64_t step,
                                        int first_child, float *tmp, bool track_err, float eps)
{
    NodeResult res;
    res.accepted = -1; res.rounds = 0; res.near = false;
    const bool act = lane < K;
    float w = (act && my_mu > 0.0f) ? my_mu : 0.0f;
    float zw = wave_ordered_sum(w, lane, K, tmp);
    w = zw > 0.0f ? w / zw : 0.0f;
    float r = act ? my_p : 0.0f;
    float rho = 1.0f;
    float err = track_err ? eps * r : 0.0f;
    for (int j = 0; j < nchild; ++j) {
        const int32_t x = child_tok[j];
        if (x < 0) break;
        const unsigned long long mask = __ballot(act && my_id == x);
        if (!mask) break;
        const int i = __ffsll((long long)mask) - 1;
        const float wi = __shfl(w, i), ri = __shfl(r, i), ei = __shfl(err, i);
        const float om = uniform(seed, b, step, (uint32_t)(first_child + j), 0u, kStreamAccept);
        const float lhs = om * wi;
        res.rounds++;
        if (track_err && fabsf(lhs - ri) <= ei + 4e-7f * ri) res.near = true;
        if (lhs < ri) { res.accepted = j; break; }
        const float mn = r < w ? r : w;
        const float M = wave_ordered_sum(mn, lane, K, tmp);
        float Z = 1.0f - M;
        if (!(Z > 1e-30f)) Z = 1e-30f;
        float d = r - w;
        if (!(d > 0.0f)) d = 0.0f;
        const float rn = d / Z;
        if (track_err) {
            float ez = (act && (r - err) < w) ? err : 0.0f;
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) ez += __shfl_xor(ez, off);
            if (ez > 0.25f * Z) res.near = true;
            err = ((err + rn * ez) / Z) * 1.001f + 4e-7f * rn;
        }
        r = rn;
        rho = rho / Z;
        if (lane == i) w = 0.0f;
        const float zw2 = wave_ordered_sum(w, lane, K, tmp);
        w = zw2 > 0.0f ? w / zw2 : 0.0f;
    }
    res.r = r;
    res.rho = rho;
    return res;
}

// ---------------------------------------------------------------------------------------------
// Row pass: one wave per logits row, no workgroup barriers.  The wave streams its row with
// kRowPF batches of kRowU 16-byte vectors per lane in flight, keeps a wave-uniform running
// maximum as the reference of the fast exponentials, and collects top-K candidates (elements
// not below the current K-th best) in a small per-wave list that is pruned by rank counting.
// ---------------------------------------------------------------------------------------------
#ifndef STAND_ROW_U
#define STAND_ROW_U 2
#endif
#ifndef STAND_ROW_PF
#define STAND_ROW_PF 2
#endif
constexpr int kRowU = STAND_ROW_U;     // vectors per lane per batch
constexpr int kRowPF = STAND_ROW_PF;   // batches in flight per wave
constexpr int kWaveCap = 128;          // vector records per wave (pruned when above 64)
#ifndef STAND_ROW_WPR
#define STAND_ROW_WPR 4
#endif
constexpr int kRowWPR = STAND_ROW_WPR;                 // waves that share one row (1, 2 or 4)
constexpr int kRowsPerBlock = kRowThreads / 64 / kRowWPR;

constexpr int kElemCap = 8 * kMaxK + 64;  // element candidates at the end of a row (<= 8 per kept vector + edges)

struct WaveScan {
    unsigned long long buf[kWaveCap + 8];   // vector records: (maximum of the vector, vector index)
    unsigned long long top[kMaxK];      // pruned / final keys, best first
    unsigned long long ebuf[kElemCap + 8];  // element keys offered to the final selection
    float tmp[kMaxK];
};

__device__ __forceinline__ int lane_prefix_count(unsigned long long mask)
{
    return (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

__device__ __forceinline__ float wave_max_f32(float x)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x = fmaxf(x, __shfl_xor(x, off));
    return x;
}

// Rank counting over n distinct non-zero keys in list[0..n): the K best are written, best
// first, to top[0..min(n,K)).  Returns the K-th best key (0 if n < K).  The list must have
// room for 7 padding entries behind n (they are zeroed here so that the scan can run in
// groups of 8 independent LDS reads).
__device__ __forceinline__ unsigned long long wave_select(unsigned long long *list, unsigned long long *top, int lane, int K,
                                                          int n)
{
    const int npad = (n + 7) & ~7;
    if (lane < npad - n) list[n + lane] = 0ull;
    __builtin_amdgcn_wave_barrier();
    for (int base = 0; base < n; base += 64) {
        const int i = base + lane;
        const unsigned long long c = i < n ? list[i] : ~0ull;
        int r = 0;
        for (int j = 0; j < npad; j += 8) {
            unsigned long long k8[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) k8[q] = list[j + q];
#pragma unroll
            for (int q = 0; q < 8; ++q) r += k8[q] > c ? 1 : 0;
        }
        if (i < n && r < K) top[r] = c;
    }
    __builtin_amdgcn_wave_barrier();
    return n >= K ? top[K - 1] : 0ull;
}

struct WaveScanState {
    unsigned long long theta_key;  // only records above it can enter the list
    float theta_val;               // value of theta_key (-inf if none): cheap pre-filter
    int cnt;                       // records in ws->buf (wave-uniform)
};

__device__ __forceinline__ void set_theta(WaveScanState &st, unsigned long long key)
{
    st.theta_key = key;
    st.theta_val = key ? rank_key_value(key) : -__builtin_inff();
}

// Prune the record list to its K best; they stay in ws->buf, the K-th best becomes the threshold.
__device__ __forceinline__ void wave_prune(WaveScan *ws, WaveScanState &st, int lane, int K)
{
    const unsigned long long th = wave_select(ws->buf, ws->top, lane, K, st.cnt);
    const int keep = st.cnt < K ? st.cnt : K;
    if (lane < keep) ws->buf[lane] = ws->top[lane];
    __builtin_amdgcn_wave_barrier();
    st.cnt = keep;
    if (th) set_theta(st, th);
}

// Lanes with `has` append the record (cm, vec) if it beats the threshold; prune above 64 records.
__device__ __forceinline__ void wave_offer(WaveScan *ws, WaveScanState &st, int lane, int K, bool has, float cm,
                                           uint32_t vec)
{
    const unsigned long long key = rank_key(cm, vec);
    const bool pred = has && key > st.theta_key;
    const unsigned long long bal = __ballot(pred);
    if (!bal) return;
    if (pred) ws->buf[st.cnt + lane_prefix_count(bal)] = key;
    st.cnt += __popcll(bal);
    __builtin_amdgcn_wave_barrier();
    if (st.cnt > 64) wave_prune(ws, st, lane, K);
}

// Leaves the row's K best element keys (value desc, id asc) sorted in ws->top[0..K), returns
// the row maximum and the fast normaliser sum_v 2^((l_v - m) c).
//
// While streaming, only one record per 16-byte vector is kept: its maximum.  The K vectors
// with the largest maxima (ties: lower index) contain the K best elements, so the elements
// are ranked only at the end, among those kept vectors.
struct WavePartial {
    float m_ref, s;   // reference maximum of this wave's part and its fast sum relative to it
    int cnt;          // vector records left in ws->buf (the wave's K best, sorted, also in ws->top)
};

// Streaming part: wave `wsub` of `wpr` cooperating waves takes every wpr-th batch of the row.
template <int DT>
__device__ __forceinline__ WavePartial wave_row_stream(const void *rowp, int V, float c, int K, WaveScan *ws, int lane,
                                                       int wsub, int wpr)
{
    constexpr int EPV = VecTraits<DT>::EPV;
    constexpr int U = kRowU, PF = kRowPF;
    const RowGeom g = row_geom<DT>(rowp, V);
    const int per_batch = 64 * U;
    const int nbatch_row = (g.nvec + per_batch - 1) / per_batch;
    const int nbatch = (nbatch_row - wsub + wpr - 1) / wpr;  // batches of this wave: wsub, wsub + wpr, ...

    WaveScanState st;
    st.cnt = 0;
    set_theta(st, 0ull);
    float m_ref = -3.402823466e38f, nb = 0.0f, s_t = 0.0f;  // m_ref, nb wave-uniform

    auto raise_reference = [&](float cm) {
        // some lane saw a value above the reference: move the reference to the wave's maximum
        const float nm = fmaxf(wave_max_f32(cm), m_ref);
        s_t *= fast_exp2((m_ref - nm) * c);
        m_ref = nm;
        nb = -nm * c;
    };
    // Loads are issued unconditionally (indices clamped to the last vector) so that the number of
    // loads in flight is the same on every path and only the oldest batch is waited for.
    const int last_vec = g.nvec > 0 ? g.nvec - 1 : 0;
    auto load_batch = [&](uint4 (&w)[U], int k) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int idx = ((k * wpr + wsub) * U + u) * 64 + lane;
            w[u] = g.vp[idx < last_vec ? idx : last_vec];
        }
    };

    uint4 ring[PF][U];
    if (g.nvec > 0) {
#pragma unroll
        for (int s = 0; s < PF; ++s) load_batch(ring[s], s);
    }

    // scalar edge elements (row start / end not on a 16-byte boundary): at most one per lane,
    // summed by the first wave of the row (they are ranked in wave_row_finish)
    int edge_id = -1;
    if (wsub == 0) {
        if (lane < g.head) edge_id = lane;
        else if (lane < g.head + g.ntail) edge_id = g.tail0 + (lane - g.head);
    }
    const float edge_val = edge_id >= 0 ? load_scalar<DT>(rowp, edge_id) : -__builtin_inff();
    if (__ballot(edge_val > m_ref)) raise_reference(edge_val);
    if (edge_id >= 0) s_t += fast_exp2(__builtin_fmaf(edge_val, c, nb));

    auto one_vector = [&](const uint4 &w, int idx, bool valid) {
        float x[EPV];
        unpack<DT>(w, x);
        float cm = x[0];
#pragma unroll
        for (int j = 1; j < EPV; ++j) cm = fmaxf(cm, x[j]);
        if (!valid) cm = -__builtin_inff();
        if (__ballot(cm > m_ref)) raise_reference(cm);
        float e = 0.0f;
#pragma unroll
        for (int j = 0; j < EPV; ++j) e += fast_exp2(__builtin_fmaf(x[j], c, nb));
        s_t += valid ? e : 0.0f;
#ifndef STAND_TUNE_NOTOPK
        if (__ballot(valid && cm >= st.theta_val)) wave_offer(ws, st, lane, K, valid && cm >= st.theta_val, cm, (uint32_t)idx);
#endif
    };
    auto do_batch = [&](uint4 (&w)[U], int k) {
        const int kb = k * wpr + wsub;        // batch of the row
        if ((kb + 1) * per_batch <= g.nvec) {  // wave-uniform: every lane has all its vectors
#pragma unroll
            for (int u = 0; u < U; ++u) one_vector(w[u], (kb * U + u) * 64 + lane, true);
        } else {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int idx = (kb * U + u) * 64 + lane;
                const bool valid = idx < g.nvec;
                one_vector(valid ? w[u] : make_uint4(0, 0, 0, 0), idx, valid);
            }
        }
    };

    // batches beyond the row (when nbatch is not a multiple of PF) have no valid lane and add nothing
    for (int k0 = 0; k0 < nbatch; k0 += PF) {
#pragma unroll
        for (int s = 0; s < PF; ++s) {
            do_batch(ring[s], k0 + s);
            load_batch(ring[s], k0 + s + PF);
        }
    }

    // leave this wave's K best records sorted in ws->buf / ws->top
    wave_prune(ws, st, lane, K);
    float s = s_t;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off);
    WavePartial out;
    out.m_ref = m_ref;
    out.s = s;
    out.cnt = st.cnt;
    return out;
}

// Finishing part (one wave per row): `cnt` vector records are in ws->buf.  The K vectors with
// the largest maxima contain the K best elements; their elements and the row's edge elements
// are ranked exactly.  Leaves the K best element keys sorted in ws->top[0..K).
template <int DT>
__device__ __forceinline__ void wave_row_finish(const void *rowp, int V, int K, WaveScan *ws, int lane, int cnt)
{
    constexpr int EPV = VecTraits<DT>::EPV;
    const RowGeom g = row_geom<DT>(rowp, V);
    int edge_id = -1;
    if (lane < g.head) edge_id = lane;
    else if (lane < g.head + g.ntail) edge_id = g.tail0 + (lane - g.head);
    const float edge_val = edge_id >= 0 ? load_scalar<DT>(rowp, edge_id) : -__builtin_inff();

    const unsigned long long th_vec = wave_select(ws->buf, ws->top, lane, K, cnt);
    const int kept = cnt < K ? cnt : K;
    const float th_val = th_vec ? rank_key_value(th_vec) : -__builtin_inff();
    int ne = 0;
    {
        const unsigned long long eb = __ballot(edge_id >= 0 && edge_val >= th_val);
        if (edge_id >= 0 && edge_val >= th_val) ws->ebuf[lane_prefix_count(eb)] = rank_key(edge_val, (uint32_t)edge_id);
        ne = __popcll(eb);
        float x[EPV];
        uint32_t vec = 0;
        const bool own = lane < kept;
        if (own) {
            vec = rank_key_id(ws->top[lane]);
            unpack<DT>(g.vp[vec], x);
        }
#pragma unroll
        for (int j = 0; j < EPV; ++j) {
            const bool pred = own && x[j] >= th_val;
            const unsigned long long bal = __ballot(pred);
            if (pred) ws->ebuf[ne + lane_prefix_count(bal)] = rank_key(x[j], (uint32_t)(g.head + (int)vec * EPV + j));
            ne += __popcll(bal);
        }
    }
    __builtin_amdgcn_wave_barrier();
    wave_select(ws->ebuf, ws->top, lane, K, ne);
}

// Exact normaliser of a row by one wave (rare path).
template <int DT>
__device__ unsigned long long wave_row_exact_sum(const void *rowp, int V, float m, float c, int lane)
{
    constexpr int EPV = VecTraits<DT>::EPV;
    const int F = fixed_bits(V);
    const RowGeom g = row_geom<DT>(rowp, V);
    unsigned long long S = 0ull;
    int edge_id = -1;
    if (lane < g.head) edge_id = lane;
    else if (lane < g.head + g.ntail) edge_id = g.tail0 + (lane - g.head);
    if (edge_id >= 0) S += fixed_contrib(exact_exp2(scaled_offset(load_scalar<DT>(rowp, edge_id), m, c)), F);
    for (int idx = lane; idx < g.nvec; idx += 64) {
        float x[EPV];
        unpack<DT>(g.vp[idx], x);
#pragma unroll
        for (int j = 0; j < EPV; ++j) S += fixed_contrib(exact_exp2(scaled_offset(x[j], m, c)), F);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) S += __shfl_xor(S, off);
    return S;
}

struct RowPassArgs {
    const void *logits;
    int B, N, V, K;
    float c;
    uint64_t seed, step;
    TreeDev tree;
    const int32_t *draft_tok;   // [B][N]
    const int32_t *draft_has;   // [B][N]
    const int32_t *draft_qid;   // [B][N][K]
    const float *draft_qmu;     // [B][N][K]
    float *row_m, *row_s;       // [B*N]
    int32_t *top_idx;           // [B*N][K]
    float *top_l, *top_p;       // [B*N][K]
    int32_t *outcome;           // [B*N] accepted child rank or -1
    unsigned long long *stats;
};

template <int DT>
__global__ __launch_bounds__(kRowThreads) void row_pass_kernel(RowPassArgs a)
{
    constexpr int ES = VecTraits<DT>::ES;
    __shared__ WaveScan wsh[kRowThreads / 64];
    __shared__ float part_m[kRowThreads / 64], part_s[kRowThreads / 64];
    __shared__ int part_cnt[kRowThreads / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wsub = wave % kRowWPR;
    const int row = blockIdx.x * kRowsPerBlock + wave / kRowWPR;
    const bool live = row < a.B * a.N;
    WaveScan *ws = &wsh[wave];
    const int b = live ? row / a.N : 0, u = live ? row % a.N : 0;
    const char *rowp = (const char *)a.logits + (size_t)(live ? row : 0) * (size_t)a.V * ES;
    float m, s;
    if constexpr (kRowWPR == 1) {
        if (!live) return;  // whole wave; no workgroup barrier in this configuration
        const WavePartial wp = wave_row_stream<DT>(rowp, a.V, a.c, a.K, ws, lane, 0, 1);
        wave_row_finish<DT>(rowp, a.V, a.K, ws, lane, wp.cnt);
        m = rank_key_value(ws->top[0]);
        s = wp.s * fast_exp2((wp.m_ref - m) * a.c);  // m_ref equals m: the factor is 1
    } else {
        if (live) {
            const WavePartial wp = wave_row_stream<DT>(rowp, a.V, a.c, a.K, ws, lane, wsub, kRowWPR);
            if (lane == 0) { part_m[wave] = wp.m_ref; part_s[wave] = wp.s; part_cnt[wave] = wp.cnt; }
        }
        __syncthreads();
        if (!live || wsub != 0) return;
        // gather the partner waves' records behind this wave's own (all lists hold at most K records)
        int cnt = part_cnt[wave];
        for (int q = 1; q < kRowWPR; ++q) {
            const int cq = part_cnt[wave + q];
            if (lane < cq) ws->buf[cnt + lane] = wsh[wave + q].buf[lane];
            cnt += cq;
        }
        __builtin_amdgcn_wave_barrier();
        wave_row_finish<DT>(rowp, a.V, a.K, ws, lane, cnt);
        m = rank_key_value(ws->top[0]);
        s = 0.0f;
        for (int q = 0; q < kRowWPR; ++q) s += part_s[wave + q] * fast_exp2((part_m[wave + q] - m) * a.c);
    }

    if (lane < a.K) {
        const unsigned long long key = ws->top[lane];
        const float l = rank_key_value(key);
        a.top_idx[(size_t)row * a.K + lane] = (int32_t)rank_key_id(key);
        a.top_l[(size_t)row * a.K + lane] = l;
        a.top_p[(size_t)row * a.K + lane] = exact_exp2(scaled_offset(l, m, a.c)) / s;
    }
    if (lane == 0) { a.row_m[row] = m; a.row_s[row] = s; }

    // ---- accept / reject outcome of this node's children (paper Sec. 3.2, applied recursively)
    const int nch_tree = a.tree.nchild[u];
    const int fc = a.tree.first_child[u];
    int nch = 0;
    if (a.draft_has[row] && a.draft_tok[row] >= 0)
        for (int j = 0; j < nch_tree; ++j) { if (a.draft_tok[(size_t)b * a.N + fc + j] < 0) break; ++nch; }
    if (nch == 0) {  // uniform over the wave
        if (lane == 0) a.outcome[row] = -1;
        return;
    }
    int32_t my_id = -1;
    float my_mu = 0.0f, my_l = 0.0f;
    if (lane < a.K) {
        my_id = a.draft_qid[(size_t)row * a.K + lane];
        my_mu = a.draft_qmu[(size_t)row * a.K + lane];
        if ((uint32_t)my_id >= (uint32_t)a.V) { my_id = -1; my_mu = 0.0f; }  // never index outside the row
        else my_l = load_scalar<DT>(rowp, my_id);
    }
    const int32_t *child_tok = a.draft_tok + (size_t)b * a.N + fc;
    const float e = (lane < a.K && my_id >= 0) ? exact_exp2(scaled_offset(my_l, m, a.c)) : 0.0f;
    NodeResult nr = wave_node_outcome(lane, a.K, my_id, my_mu, e / s, nch, child_tok, a.seed, (uint32_t)b, a.step, fc,
                                      ws->tmp, true, kFastEps);
    if (nr.near) {
        // a test fell inside the error bound of the fast normaliser: decide with the exact one
        const unsigned long long S = wave_row_exact_sum<DT>(rowp, a.V, m, a.c, lane);
        const float sx = normaliser_from_fixed(S, fixed_bits(a.V));
        nr = wave_node_outcome(lane, a.K, my_id, my_mu, e / sx, nch, child_tok, a.seed, (uint32_t)b, a.step, fc, ws->tmp,
                               false, 0.0f);
        if (lane == 0) atomicAdd(&a.stats[kStatNear], 1ull);
    }
    if (lane == 0) a.outcome[row] = nr.accepted;
}

// ---------------------------------------------------------------------------------------------
// Path pass: workgroup (j, b) handles the j-th row of trajectory b's accepted path.
// mode 0 (verify): the path follows `outcome`; writes out_tok / out_node / out_len and, for
//                  every path row, the exact observation (top-K ids, probabilities).
// mode 1 (update): rows are given (commit_row); statistics are computed here.
// ---------------------------------------------------------------------------------------------
struct PathPassArgs {
    const void *logits;
    int B, N, V, K, W, mode;
    float c;
    uint64_t seed, step;
    TreeDev tree;
    const int32_t *draft_tok, *draft_has, *draft_qid;
    const float *draft_qmu;
    const float *row_m;
    const int32_t *top_idx;
    const float *top_l;
    const int32_t *outcome;
    const int32_t *commit_row, *commit_len;  // mode 1
    int32_t *out_tok, *out_node, *out_len;   // mode 0
    int32_t *obs_idx;                         // [B][W][K]
    float *obs_p;                             // [B][W][K]
    unsigned long long *stats;
};

struct PathShared {
    ScanShared scan;
    int path[32];
    int len;
    int32_t sup_id[kMaxK];
    float sup_r[kMaxK];
    float rho;
    int nsup;
    unsigned long long best;
};

template <int DT>
__global__ __launch_bounds__(kPathThreads) void path_pass_kernel(PathPassArgs a)
{
    constexpr int ES = VecTraits<DT>::ES, EPV = VecTraits<DT>::EPV, BS = kPathThreads;
    __shared__ PathShared ps;
    const int j = blockIdx.x, b = blockIdx.y, tid = threadIdx.x, lane = tid & 63;
    int node;
    bool is_stop = false;
    if (a.mode == 0) {
        if (tid == 0) {
            int cur = 0, len = 0;
            for (;;) {
                ps.path[len++] = cur;
                const int acc = a.outcome[(size_t)b * a.N + cur];
                if (acc < 0 || len > a.tree.D) break;
                cur = a.tree.first_child[cur] + acc;
            }
            ps.len = len;
        }
        __syncthreads();
        const int len = ps.len;
        if (j == 0) {
            // accepted tokens are the tokens of the path nodes after the root
            if (tid < a.W) {
                a.out_node[(size_t)b * a.W + tid] = tid < len ? ps.path[tid] : -1;
                if (tid + 1 < len) a.out_tok[(size_t)b * a.W + tid] = a.draft_tok[(size_t)b * a.N + ps.path[tid + 1]];
                else if (tid >= len) a.out_tok[(size_t)b * a.W + tid] = -1;
            }
            if (tid == 0) { a.out_len[b] = len; atomicAdd(&a.stats[kStatTokens], (unsigned long long)len); }
        }
        if (j >= len) return;
        node = ps.path[j];
        is_stop = (j == len - 1);
    } else {
        int len = a.commit_len[b];
        len = len < 0 ? 0 : (len > a.W ? a.W : len);
        if (j >= len) return;
        node = a.commit_row[(size_t)b * a.W + j];
        if (node < 0 || node >= a.N) return;  // ignored record (the merge skips it too)
    }
    const int row = b * a.N + node;
    const char *rowp = (const char *)a.logits + (size_t)row * (size_t)a.V * ES;

    // ---- row maximum and top-K: from the row pass, or computed here
    float m;
    int32_t my_top = -1;
    float my_topl = 0.0f;
    if (a.mode == 0) {
        m = a.row_m[row];
        if (tid < a.K) { my_top = a.top_idx[(size_t)row * a.K + tid]; my_topl = a.top_l[(size_t)row * a.K + tid]; }
    } else {
        float s_unused;
        wg_row_scan<DT, BS>(rowp, a.V, a.c, a.K, ps.scan, m, s_unused);
        if (tid < a.K) { my_top = (int32_t)rank_key_id(ps.scan.top[tid]); my_topl = rank_key_value(ps.scan.top[tid]); }
    }

    // ---- exact normaliser and the observation (paper Sec. 4.1: top-k ids and probabilities)
    const unsigned long long S = wg_row_exact_sum<DT, BS>(rowp, a.V, m, a.c, &ps.scan.acc64);
    const float s = normaliser_from_fixed(S, fixed_bits(a.V));
    if (tid < a.K) {
        a.obs_idx[((size_t)b * a.W + j) * a.K + tid] = my_top;
        a.obs_p[((size_t)b * a.W + j) * a.K + tid] = exact_exp2(scaled_offset(my_topl, m, a.c)) / s;
    }
    if (a.mode != 0) return;

    // ---- replay the node's accept sequence with exact probabilities
    const int nch_tree = a.tree.nchild[node];
    const int fc = a.tree.first_child[node];
    int nch = 0;
    if (a.draft_has[row] && a.draft_tok[row] >= 0)
        for (int q = 0; q < nch_tree; ++q) { if (a.draft_tok[(size_t)b * a.N + fc + q] < 0) break; ++nch; }
    if (tid == 0) { ps.nsup = 0; ps.rho = 1.0f; ps.best = ~0ull; }
    __syncthreads();
    if (nch > 0 && tid < 64) {
        int32_t my_id = -1;
        float my_mu = 0.0f, my_p = 0.0f;
        if (tid < a.K) {
            my_id = a.draft_qid[(size_t)row * a.K + tid];
            my_mu = a.draft_qmu[(size_t)row * a.K + tid];
            if ((uint32_t)my_id >= (uint32_t)a.V) { my_id = -1; my_mu = 0.0f; }
            else my_p = exact_exp2(scaled_offset(load_scalar<DT>(rowp, my_id), m, a.c)) / s;
        }
        NodeResult nr = wave_node_outcome(lane, a.K, my_id, my_mu, my_p, nch, a.draft_tok + (size_t)b * a.N + fc, a.seed,
                                          (uint32_t)b, a.step, fc, ps.scan.tmp, false, 0.0f);
        if (tid < a.K) { ps.sup_id[tid] = my_id; ps.sup_r[tid] = nr.r; }
        if (tid == 0) {
            ps.nsup = a.K;
            ps.rho = nr.rho;
            atomicAdd(&a.stats[kStatTests], (unsigned long long)nr.rounds);
            if (nr.accepted != a.outcome[row]) atomicAdd(&a.stats[kStatMismatch], 1ull);
        }
    }
    __syncthreads();
    if (!is_stop) return;

    // ---- resample at the stop node: exponential race over the vocabulary (paper Sec. 3.2,
    //      "resampled from an adjusted distribution")
    const int nsup = ps.nsup;
    const float rho = ps.rho;
    const RowGeom g = row_geom<DT>(rowp, a.V);
    unsigned long long best = ~0ull;
    auto consider = [&](float l, uint32_t v, const Philox4 &ph, bool near_support) {
        float r = (exact_exp2(scaled_offset(l, m, a.c)) / s) * rho;
        if (near_support)
            for (int q = 0; q < nsup; ++q) if (ps.sup_id[q] == (int32_t)v) r = ps.sup_r[q];
        if (r > 0.0f) {
            const float xv = -exact_log(word_to_uniform(philox_word(ph, v & 3u)));
            const float t = xv / r;
            const unsigned long long key = ((unsigned long long)f2u(t) << 32) | (unsigned long long)v;
            best = key < best ? key : best;
        }
    };
    int edge_id = -1;
    if (tid < g.head) edge_id = tid;
    else if (tid < g.head + g.ntail) edge_id = g.tail0 + (tid - g.head);
    if (edge_id >= 0) {
        Philox4 ph = philox_group(a.seed, (uint32_t)b, a.step, (uint32_t)node, (uint32_t)edge_id >> 2, kStreamBonus);
        consider(load_scalar<DT>(rowp, edge_id), (uint32_t)edge_id, ph, true);
    }
    for (int idx = tid; idx < g.nvec; idx += BS) {
        float x[EPV];
        unpack<DT>(g.vp[idx], x);
        const uint32_t id0 = (uint32_t)(g.head + idx * EPV);
        bool near_support = false;  // does a stored id fall into this vector?
        for (int q = 0; q < nsup; ++q) near_support |= ((uint32_t)ps.sup_id[q] - id0) < (uint32_t)EPV;
        uint32_t grp = 0xFFFFFFFFu;
        Philox4 ph;
#pragma unroll
        for (int q = 0; q < EPV; ++q) {
            const uint32_t v = id0 + q;
            if ((v >> 2) != grp) { grp = v >> 2; ph = philox_group(a.seed, (uint32_t)b, a.step, (uint32_t)node, grp, kStreamBonus); }
            consider(x[q], v, ph, near_support);
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        unsigned long long o = __shfl_xor(best, off);
        best = o < best ? o : best;
    }
    if (lane == 0) atomicMin(&ps.best, best);
    __syncthreads();
    if (tid == 0) a.out_tok[(size_t)b * a.W + j] = (int32_t)(uint32_t)ps.best;
}

// ---------------------------------------------------------------------------------------------
// Table merge (paper Sec. 4.1): claim a slot per record, then apply the records of each slot in
// record order (b, then position, then order ascending).
// ---------------------------------------------------------------------------------------------
struct MergeArgs {
    char *table;
    uint64_t mask;
    int slot_bytes, K, max_probe;
    int B, W, omin, omax;
    const int32_t *ctx_tail;          // [B][kMaxOrder], newest token last
    const long long *ctx_len;         // [B]
    const int32_t *commit_tok;        // [B][W]
    const int32_t *commit_row;        // [B][W] or NULL (then every j < len is valid)
    const int32_t *commit_len;        // [B]
    int N;
    long long *rec_slot;              // [B*W*NO]
    const int32_t *obs_idx;
    const float *obs_p;
    unsigned long long *stats;
};

__device__ __forceinline__ int clamp_len(int len, int W) { return len < 0 ? 0 : (len > W ? W : len); }

__global__ void merge_claim_kernel(MergeArgs a)
{
    const int NO = a.omax - a.omin + 1;
    const int rec = blockIdx.x * blockDim.x + threadIdx.x;
    if (rec >= a.B * a.W * NO) return;
    const int n = a.omin + rec % NO;
    const int j = (rec / NO) % a.W;
    const int b = rec / (NO * a.W);
    long long slot_out = -1;
    const int len = clamp_len(a.commit_len[b], a.W);
    const long long base_len = a.ctx_len[b];
    bool valid = j < len && base_len + j >= n;
    if (valid && a.commit_row) {
        const int r = a.commit_row[(size_t)b * a.W + j];
        valid = r >= 0 && r < a.N;
    }
    if (valid) {
        int32_t key[kMaxOrder];
        for (int i = 0; i < n; ++i) {
            const int back = n - i;  // this token is `back` positions before token j
            // positions before j: commit tokens j-1, j-2, ... then the context tail
            key[i] = (back <= j) ? a.commit_tok[(size_t)b * a.W + (j - back)]
                                 : a.ctx_tail[(size_t)b * kMaxOrder + (kMaxOrder - (back - j))];
        }
        const unsigned long long fp = fingerprint(n, key);
        bool placed = false;
        for (int i = 0; i < a.max_probe; ++i) {
            const uint64_t slot = (fp + (uint64_t)i) & a.mask;
            SlotHeader *h = slot_header(a.table, slot, a.slot_bytes);
            const unsigned long long old = atomicCAS(&h->fp, 0ull, fp);
            if (old == 0ull) {
                h->order = (uint32_t)n;
                atomicAdd(&a.stats[kStatInserts], 1ull);
                slot_out = (long long)slot; placed = true; break;
            }
            if (old == fp) {
                atomicAdd(&a.stats[kStatMerges], 1ull);
                slot_out = (long long)slot; placed = true; break;
            }
        }
        if (!placed) atomicAdd(&a.stats[kStatDrops], 1ull);
    }
    a.rec_slot[rec] = slot_out;
}

// one wave per record; the first record of a slot applies all records of that slot in order
__global__ __launch_bounds__(64) void merge_apply_kernel(MergeArgs a)
{
    __shared__ int32_t l_id[2 * kMaxK];
    __shared__ float l_val[2 * kMaxK];
    const int NO = a.omax - a.omin + 1;
    const int nrec = a.B * a.W * NO;
    const int rec = blockIdx.x;
    const int lane = threadIdx.x;
    const int K = a.K;
    const long long slot = a.rec_slot[rec];
    if (slot < 0) return;
    // leader test: no earlier record on this slot
    for (int base = 0; base < rec; base += 64) {
        const int r = base + lane;
        const bool hit = r < rec && a.rec_slot[r] == slot;
        if (__ballot(hit)) return;
    }
    SlotHeader *h = slot_header(a.table, (uint64_t)slot, a.slot_bytes);
    int32_t *ids = slot_ids(a.table, (uint64_t)slot, a.slot_bytes);
    float *mus = slot_mu(a.table, (uint64_t)slot, a.slot_bytes, K);
    uint32_t count = h->count;
    // lanes 0..K-1: stored entry; lanes 32..32+K-1: observation
    int32_t e_id = -1;
    float e_mu = 0.0f;
    if (lane < K && count > 0) { e_id = ids[lane]; e_mu = mus[lane]; }
    for (int base = rec; base < nrec; base += 64) {
        const int r = base + lane;
        unsigned long long hits = __ballot(r < nrec && a.rec_slot[r] == slot);
        while (hits) {
            const int bit = __ffsll((long long)hits) - 1;
            hits &= hits - 1;
            const int rr = base + bit;
            const int jb = rr / NO;  // = b * W + j
            int32_t o_id = -1;
            float o_p = 0.0f;
            if (lane >= 32 && lane < 32 + K) { o_id = a.obs_idx[(size_t)jb * K + (lane - 32)]; o_p = a.obs_p[(size_t)jb * K + (lane - 32)]; }
            if (count == 0) {
                // first sight: the entry is the observation
                const int32_t id2 = __shfl(o_id, 32 + (lane & 31));
                const float p2 = __shfl(o_p, 32 + (lane & 31));
                if (lane < K) { e_id = id2; e_mu = p2; }
            } else {
                const float cf = (float)count;
                const float denom = cf + 1.0f;
                int32_t id = lane < 32 ? e_id : o_id;
                bool act = lane < 32 ? (lane < K) : (lane < 32 + K);
                float other = 0.0f;  // for stored lanes: the observation's value for the same id
                bool dup = false;    // for observation lanes: id already stored
                for (int q = 0; q < K; ++q) {
                    const int32_t sid = __shfl(e_id, q);
                    const int32_t oid = __shfl(o_id, 32 + q);
                    const float op = __shfl(o_p, 32 + q);
                    if (lane < 32 && act && oid == id) other = op;
                    if (lane >= 32 && act && sid == id) dup = true;
                }
                float val;
                if (lane < 32) { float t = cf * e_mu; t = t + other; val = t / denom; }
                else { float t = cf * 0.0f; t = t + o_p; val = t / denom; act = act && !dup; }
                const unsigned long long key = act ? rank_key(val, (uint32_t)id) : 0ull;
                int rank = 0;
                for (int q = 0; q < 64; ++q) {
                    const unsigned long long ok = __shfl(key, q);
                    rank += (ok > key) ? 1 : 0;
                }
                if (act && rank < K) { l_id[rank] = id; l_val[rank] = val; }
                __syncthreads();
                if (lane < K) { e_id = l_id[lane]; e_mu = l_val[lane]; }
                __syncthreads();
            }
            count++;
        }
    }
    if (lane < K) { ids[lane] = e_id; mus[lane] = e_mu; }
    if (lane == 0) h->count = count;
}

// append the committed tokens to the context tails
__global__ void ctx_append_kernel(int B, int W, int32_t *ctx_tail, long long *ctx_len, const int32_t *commit_tok,
                                  const int32_t *commit_len)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    const int len = clamp_len(commit_len[b], W);
    int32_t t[kMaxOrder];
    for (int i = 0; i < kMaxOrder; ++i) t[i] = ctx_tail[(size_t)b * kMaxOrder + i];
    for (int j = 0; j < len; ++j) {
        for (int i = 0; i + 1 < kMaxOrder; ++i) t[i] = t[i + 1];
        t[kMaxOrder - 1] = commit_tok[(size_t)b * W + j];
    }
    for (int i = 0; i < kMaxOrder; ++i) ctx_tail[(size_t)b * kMaxOrder + i] = t[i];
    ctx_len[b] += len;
}

// ---------------------------------------------------------------------------------------------
// Draft (paper Sec. 4.2): one workgroup per trajectory, tree levels in sequence, one wave per node.
// ---------------------------------------------------------------------------------------------
struct DraftArgs {
    char *table;
    uint64_t mask;
    int slot_bytes, K, max_probe;
    int B, omin, omax;
    uint64_t seed, step;
    TreeDev tree;
    const int32_t *ctx_tail;
    const long long *ctx_len;
    int32_t *draft_tok, *draft_has, *draft_qid;
    float *draft_qmu;
    int32_t *out_tok;  // caller's copy, may be NULL
    unsigned long long *stats;
};

constexpr int kDraftThreads = 256;
constexpr int kMaxNodes = 256;
constexpr int kMaxDepth = 31;

__global__ __launch_bounds__(kDraftThreads) void draft_kernel(DraftArgs a)
{
    __shared__ int32_t tok[kMaxNodes];
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int N = a.tree.N, K = a.K;
    const long long clen = a.ctx_len[b];
    for (int u = tid; u < N; u += kDraftThreads) {
        tok[u] = -1;
        a.draft_has[(size_t)b * N + u] = 0;
    }
    __syncthreads();
    if (tid == 0 && clen > 0) tok[0] = a.ctx_tail[(size_t)b * kMaxOrder + kMaxOrder - 1];
    __syncthreads();
    for (int d = 0; d < a.tree.D; ++d) {
        const int lo = a.tree.level_start[d], hi = a.tree.level_start[d + 1];
        for (int u = lo + wave; u < hi; u += kDraftThreads / 64) {
            const int nch = a.tree.nchild[u];
            if (nch == 0 || tok[u] < 0) continue;  // uniform per wave
            // lane q < NO looks up order n = omax - q
            const int NO = a.omax - a.omin + 1;
            long long hit_slot = -1;
            if (lane < NO) {
                const int n = a.omax - lane;
                if (clen + d >= n) {
                    int32_t key[kMaxOrder];
                    // newest token first while walking up: position n-1 is the node's own token
                    int x = u;
                    for (int i = n - 1; i >= 0; --i) {
                        const int back = n - 1 - i;  // tokens back from the node itself
                        if (back < d) { key[i] = tok[x]; x = a.tree.parent[x]; }
                        else key[i] = a.ctx_tail[(size_t)b * kMaxOrder + (kMaxOrder - 1 - (back - d))];
                    }
                    const unsigned long long fp = fingerprint(n, key);
                    for (int i = 0; i < a.max_probe; ++i) {
                        const uint64_t slot = (fp + (uint64_t)i) & a.mask;
                        const SlotHeader *h = slot_header(a.table, slot, a.slot_bytes);
                        const unsigned long long cur = h->fp;
                        if (cur == fp) { if (h->count > 0) hit_slot = (long long)slot; break; }
                        if (cur == 0ull) break;
                    }
                }
            }
            const unsigned long long hits = __ballot(hit_slot >= 0);
            if (!hits) {
                if (lane == 0) atomicAdd(&a.stats[kStatMisses], 1ull);
                continue;
            }
            const int win = __ffsll((long long)hits) - 1;  // lowest lane = longest order
            const long long slot = __shfl(hit_slot, win);
            if (lane == 0) atomicAdd(&a.stats[kStatHits + (a.omax - win)], 1ull);
            int32_t id = -1;
            float mu = 0.0f;
            if (lane < K) {
                id = slot_ids(a.table, (uint64_t)slot, a.slot_bytes)[lane];
                mu = slot_mu(a.table, (uint64_t)slot, a.slot_bytes, K)[lane];
                a.draft_qid[((size_t)b * N + u) * K + lane] = id;
                a.draft_qmu[((size_t)b * N + u) * K + lane] = mu;
            }
            if (lane == 0) a.draft_has[(size_t)b * N + u] = 1;
            // Gumbel-Top-K: score = ln mu - ln(-ln U); children get the largest scores in order
            const bool cand = lane < K && mu > 0.0f;
            unsigned long long key = 0ull;
            if (cand) {
                const float U = uniform(a.seed, (uint32_t)b, a.step, (uint32_t)u, (uint32_t)id, kStreamDraft);
                const float g = exact_log(-exact_log(U));
                key = rank_key(exact_log(mu) - g, (uint32_t)id);
            }
            int rank = 0;
            for (int q = 0; q < K; ++q) {
                const unsigned long long ok = __shfl(key, q);
                rank += (ok > key) ? 1 : 0;
            }
            if (cand && rank < nch) tok[a.tree.first_child[u] + rank] = id;
        }
        __syncthreads();
    }
    for (int u = tid; u < N; u += kDraftThreads) {
        a.draft_tok[(size_t)b * N + u] = tok[u];
        if (a.out_tok) a.out_tok[(size_t)b * N + u] = tok[u];
    }
}

// small helpers --------------------------------------------------------------------------------
__global__ void fill_i32_kernel(int32_t *p, int32_t v, size_t n)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

// top-K probabilities are produced by the row pass already; this copies the per-row results out
__global__ void copy_row_results_kernel(int rows, int K, const float *row_m, const float *row_s, const int32_t *top_idx,
                                        const float *top_p, float *o_m, float *o_s, int32_t *o_idx, float *o_p)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < (size_t)rows) {
        if (o_m) o_m[i] = row_m[i];
        if (o_s) o_s[i] = row_s[i];
    }
    if (i < (size_t)rows * K) {
        if (o_idx) o_idx[i] = top_idx[i];
        if (o_p) o_p[i] = top_p[i];
    }
}

// export support: count and compact the occupied slots
__global__ void table_compact_kernel(const char *table, uint64_t capacity, int slot_bytes, unsigned long long *counter,
                                     char *out, unsigned long long out_cap)
{
    uint64_t slot = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (slot >= capacity) return;
    const SlotHeader *h = (const SlotHeader *)(table + slot * (uint64_t)slot_bytes);
    if (h->fp == 0ull || h->count == 0) return;
    unsigned long long pos = atomicAdd(counter, 1ull);
    if (out && pos < out_cap) {
        const uint32_t *src = (const uint32_t *)(table + slot * (uint64_t)slot_bytes);
        uint32_t *dst = (uint32_t *)(out + pos * (unsigned long long)slot_bytes);
        for (int i = 0; i < slot_bytes / 4; ++i) dst[i] = src[i];
    }
}

}  // namespace stand
