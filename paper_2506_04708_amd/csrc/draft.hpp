// draft.hpp -- draft_kernel: multi-level lookup and Gumbel-Top-K along the static tree (paper Sec. 4.2).
#pragma once
#include "wave_ops.hpp"

namespace stand {

// ---------------------------------------------------------------------------------------------
// Draft (paper Sec. 4.2): one workgroup per trajectory, tree levels in sequence, one wave per node.
// ---------------------------------------------------------------------------------------------
struct DraftArgs {
    char *table;
    uint64_t mask;
    int slot_bytes, K, max_probe;
    int B, W, omin, omax;
    uint64_t seed, step;
    TreeDev tree;
    int32_t *ctx_tail;
    long long *ctx_len;
    const int32_t *append_tok;   // [B][W] tokens to append to the contexts first, or NULL
    const int32_t *append_len;   // [B]
    int32_t *draft_tok, *draft_has, *draft_qid;
    float *draft_qmu;
    int32_t *out_tok;  // caller's copy, may be NULL
    unsigned long long *stats;
    int mode;          // 0: Gumbel-Top-K, 1: sequential multinomial without replacement, 2: largest means
    int32_t *recent_out;  // [B][N][kMaxOrder] or NULL: the recent tokens of every drafted node (all-nodes update)
};

constexpr int kDraftThreads = 1024;  // 16 waves: the nodes of a tree level are looked up side by side

// Shared memory of one trajectory's draft, sized for a tree of N nodes and depth D.
struct DraftShared {
    int32_t *tok;                    // [N]
    int32_t (*recent)[kMaxOrder];    // [N][kMaxOrder] recent[u][i]: the token i positions before the end of the
                                     // sequence that ends at node u (recent[u][0] is the node's own token), so a
                                     // key is read without walking up the tree; 16-byte aligned
    int32_t *t_first, *t_nchild;     // [N]
    int32_t *t_level;                // [D + 2]
    long long *clen;
};
__host__ __device__ inline size_t draft_shared_bytes(int N, int D)
{
    return (size_t)N * kMaxOrder * 4 + 3 * (size_t)N * 4 + (((size_t)D + 2 + 3) & ~(size_t)3) * 4 + 16;
}
__device__ __forceinline__ DraftShared draft_shared_carve(char *base, int N, int D)
{
    DraftShared s;
    s.recent = (int32_t(*)[kMaxOrder])base;  base += (size_t)N * kMaxOrder * 4;
    s.tok = (int32_t *)base;                 base += (size_t)N * 4;
    s.t_first = (int32_t *)base;             base += (size_t)N * 4;
    s.t_nchild = (int32_t *)base;            base += (size_t)N * 4;
    s.t_level = (int32_t *)base;             base += (((size_t)D + 2 + 3) & ~(size_t)3) * 4;
    s.clen = (long long *)base;
    return s;
}

// The draft of trajectory b by the NT threads of the calling workgroup (all of them call this).
template <int NT>
__device__ __forceinline__ void draft_trajectory(const DraftArgs &a, int b, const DraftShared &sm)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    int32_t *tok = sm.tok, *t_first = sm.t_first, *t_nchild = sm.t_nchild, *t_level = sm.t_level;
    int32_t(*recent)[kMaxOrder] = sm.recent;
    const int N = a.tree.N, K = a.K;
    for (int u = tid; u < N; u += NT) {
        t_first[u] = a.tree.first_child[u];
        t_nchild[u] = a.tree.nchild[u];
        if (u > 0) tok[u] = -1;  // the root's token is set with the context below
        a.draft_has[(size_t)b * N + u] = 0;
    }
    if (tid < a.tree.D + 2) t_level[tid] = a.tree.level_start[tid];
    if (wave == 1 && lane == 0) {
        // context tail of this trajectory, after appending the tokens committed by this step
        int32_t t[kMaxOrder];
        for (int i = 0; i < kMaxOrder; ++i) t[i] = a.ctx_tail[(size_t)b * kMaxOrder + i];
        long long len = a.ctx_len[b];
        if (a.append_tok) {
            const int n = clamp_len(a.append_len[b], a.W);
            for (int j = 0; j < n; ++j) {
                for (int i = 0; i + 1 < kMaxOrder; ++i) t[i] = t[i + 1];
                t[kMaxOrder - 1] = a.append_tok[(size_t)b * a.W + j];
            }
            len += n;
            for (int i = 0; i < kMaxOrder; ++i) a.ctx_tail[(size_t)b * kMaxOrder + i] = t[i];
            a.ctx_len[b] = len;
        }
        for (int i = 0; i < kMaxOrder; ++i) recent[0][i] = t[kMaxOrder - 1 - i];
        tok[0] = len > 0 ? t[kMaxOrder - 1] : -1;
        *sm.clen = len;
    }
    __syncthreads();
    const long long clen = (long long)readlane_u64((unsigned long long)*sm.clen, 0);
    const int NO = a.omax - a.omin + 1;
    for (int d = 0; d < a.tree.D; ++d) {
        // values read from shared memory that are the same in every lane go to scalar registers
        const int lo = __builtin_amdgcn_readfirstlane(t_level[d]), hi = __builtin_amdgcn_readfirstlane(t_level[d + 1]);
        // a level without a drafted node ends the tree (tok is stable here: barrier below)
        bool any = false;
        for (int u = lo + lane; u < hi; u += 64) any |= tok[u] >= 0;
        if (!__ballot(any)) break;  // the same in every wave
        for (int u = lo + wave; u < hi; u += NT / 64) {
            const int nch = __builtin_amdgcn_readfirstlane(t_nchild[u]);
            if (nch == 0 || __builtin_amdgcn_readfirstlane(tok[u]) < 0) continue;
            // ---- multi-level lookup (paper Sec. 4.2): lane q < NO takes order n = omax - q.
            // The home slot of every order is read together with its payload in one round
            // trip; only a key that was displaced by linear probing needs further probes.
            // The node's recent tokens are the same for every lane: they are read once (two 16-byte
            // reads), their terms of the fingerprint are formed in scalar registers, and each lane adds
            // the first n of them by selects -- no lane-dependent branches or dependent reads.
            unsigned long long fp = 0ull;
            {
                const int4 r_lo = *(const int4 *)&recent[u][0], r_hi = *(const int4 *)&recent[u][4];
                const int32_t rt[kMaxOrder] = {r_lo.x, r_lo.y, r_lo.z, r_lo.w, r_hi.x, r_hi.y, r_hi.z, r_hi.w};
                const int n = a.omax - lane;
                unsigned long long acc = (unsigned long long)(uint32_t)n * 0x2545F4914F6CDD1DULL;
#pragma unroll
                for (int i = 0; i < kMaxOrder; ++i) {
                    const uint32_t x = (uint32_t)__builtin_amdgcn_readfirstlane(rt[i]);
                    const unsigned long long term = fingerprint_multiplier(i) * ((unsigned long long)x + 1u);
                    acc += i < n ? term : 0ull;
                }
                const unsigned long long hsh = fmix64(acc);
                if (lane < NO && clen + d >= n) fp = hsh ? hsh : 1ull;
            }
            unsigned long long home_fp = 0ull;
            uint32_t home_cnt = 0;
            if (fp) {
                const SlotHeader *h = slot_header(a.table, fp & a.mask, a.slot_bytes);
                home_fp = ld_agent(&h->fp);
                home_cnt = ld_agent(&h->count);
            }
            int32_t pid[kMaxOrder];
            float pmu[kMaxOrder];
#pragma unroll
            for (int q = 0; q < kMaxOrder; ++q) {
                pid[q] = -1; pmu[q] = 0.0f;
                const unsigned long long fq = readlane_u64(fp, q);  // uniform
                if (q < NO && fq && lane < K) {
                    pid[q] = ld_agent(&slot_ids(a.table, fq & a.mask, a.slot_bytes)[lane]);
                    pmu[q] = ld_agent(&slot_mu(a.table, fq & a.mask, a.slot_bytes, K)[lane]);
                }
            }
            long long hit_slot = -1;
            if (fp) {
                if (home_fp == fp) { if (home_cnt > 0) hit_slot = (long long)(fp & a.mask); }
                else if (home_fp != 0ull) {
                    for (int i = 1; i < a.max_probe; ++i) {  // displaced key: keep probing
                        const uint64_t slot = (fp + (uint64_t)i) & a.mask;
                        const SlotHeader *h = slot_header(a.table, slot, a.slot_bytes);
                        const unsigned long long cur = ld_agent(&h->fp);
                        if (cur == fp) { if (ld_agent(&h->count) > 0) hit_slot = (long long)slot; break; }
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
            const long long slot = (long long)readlane_u64((unsigned long long)hit_slot, win);
            const unsigned long long win_fp = readlane_u64(fp, win);
            if (lane == 0) atomicAdd(&a.stats[kStatHits + (a.omax - win)], 1ull);
            int32_t id = -1;
            float mu = 0.0f;
            if ((unsigned long long)slot == (win_fp & a.mask)) {
                // the payload fetched with the home slot is the entry's
#pragma unroll
                for (int q = 0; q < kMaxOrder; ++q) if (q == win) { id = pid[q]; mu = pmu[q]; }
            } else if (lane < K) {
                id = ld_agent(&slot_ids(a.table, (uint64_t)slot, a.slot_bytes)[lane]);
                mu = ld_agent(&slot_mu(a.table, (uint64_t)slot, a.slot_bytes, K)[lane]);
            }
            if (lane < K) {
                a.draft_qid[((size_t)b * N + u) * K + lane] = id;
                a.draft_qmu[((size_t)b * N + u) * K + lane] = mu;
            }
            const bool cand = lane < K && mu > 0.0f;
            int rank = kMaxK;  // child rank of this lane's candidate (>= nch: not drafted)
            if (a.mode == 1) {
                // ---- sequential sampling without replacement (the ablation's plain stochastic
                // drafting): draw j takes the first remaining candidate, in stored order, whose
                // running sum of mu exceeds U_j * (sum of the remaining mu)
                const float u_l = lane < nch ? uniform(a.seed, (uint32_t)b, a.step, (uint32_t)u, (uint32_t)lane, kStreamDraft) : 0.0f;
                bool left = cand;
                const int ncand_all = __popcll(__ballot(cand));
                const int draws = nch < ncand_all ? nch : ncand_all;
                for (int j = 0; j < draws; ++j) {
                    const float mleft = left ? mu : 0.0f;
                    const float z = wave_tree_sum(mleft);
                    const float t = u2f((uint32_t)__builtin_amdgcn_readlane((int)f2u(u_l), j)) * z;
                    float acc = 0.0f;
                    int pick = -1, last = -1;
                    const unsigned long long left_mask = __ballot(left);
                    for (int i = 0; i < K; ++i) {
                        const float mi = u2f((uint32_t)__builtin_amdgcn_readlane((int)f2u(mleft), i));
                        if (!((left_mask >> i) & 1ull)) continue;  // uniform
                        last = i;
                        acc = acc + mi;
                        if (pick < 0 && t < acc) pick = i;
                    }
                    if (pick < 0) pick = last;
                    if (lane == pick) { rank = j; left = false; }
                }
            } else {
                // ---- Gumbel-Top-K (paper Sec. 4.2): score = ln mu - ln(-ln U), the largest scores in
                // order; deterministic drafting (Sec. 3.1): the largest means themselves
                unsigned long long key = 0ull;
                if (cand) {
                    if (a.mode == 2) key = rank_key(mu, (uint32_t)id);
                    else {
                        const float U = uniform(a.seed, (uint32_t)b, a.step, (uint32_t)u, (uint32_t)id, kStreamDraft);
                        const float g = exact_log(-exact_log(U));
                        key = rank_key(exact_log(mu) - g, (uint32_t)id);
                    }
                }
                rank = 0;  // lanes without a candidate hold key 0, which is above no key
#pragma unroll
                for (int q = 0; q < kMaxK / 2; ++q) rank += readlane_u64(key, q) > key ? 1 : 0;
                if (K > kMaxK / 2) {  // lanes K.. hold key 0: the upper half is needed for large K only
#pragma unroll
                    for (int q = kMaxK / 2; q < kMaxK; ++q) rank += readlane_u64(key, q) > key ? 1 : 0;
                }
            }
            if (cand && rank < nch) {
                const int child = t_first[u] + rank;
                tok[child] = id;
                recent[child][0] = id;
#pragma unroll
                for (int i = 1; i < kMaxOrder; ++i) recent[child][i] = recent[u][i - 1];
            }
            const int ncand = __popcll(__ballot(cand));
            if (lane == 0) a.draft_has[(size_t)b * N + u] = ncand < nch ? ncand : nch;
        }
        __syncthreads();
    }
    for (int u = tid; u < N; u += NT) {
        a.draft_tok[(size_t)b * N + u] = tok[u];
        if (a.out_tok) a.out_tok[(size_t)b * N + u] = tok[u];
    }
    if (a.recent_out)
        for (int i = tid; i < N * kMaxOrder; i += NT)
            if (tok[i / kMaxOrder] >= 0) a.recent_out[(size_t)b * N * kMaxOrder + i] = recent[i / kMaxOrder][i % kMaxOrder];
}

__global__ __launch_bounds__(kDraftThreads) void draft_kernel(DraftArgs a)
{
    __shared__ __align__(16) char smem[(size_t)kMaxNodes * kMaxOrder * 4 + 3 * (size_t)kMaxNodes * 4 + (kMaxDepth + 5) * 4 + 16];
    draft_trajectory<kDraftThreads>(a, (int)blockIdx.x, draft_shared_carve(smem, a.tree.N, a.tree.D));
}

}  // namespace stand
