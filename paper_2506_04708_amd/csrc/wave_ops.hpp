// wave_ops.hpp -- shared by all kernels: limits, tree and table slot layout, 16-byte vector access to a
// logits row, wave-level reductions by data-parallel-primitive moves, and the accept / reject sequence
// of one tree node (paper Sec. 3.2).
#pragma once
#include "numeric.hpp"

namespace stand {

constexpr int kDtBf16 = 0, kDtF32 = 1;
// Row pass: one row per workgroup of WPR waves.  Four waves per row fill the device when there
// are thousands of rows; with few rows (one or a few trajectories) a row is spread over sixteen
// waves so that the pass is not limited by what four waves can keep in flight.
#ifndef STAND_ROW_WPR
#define STAND_ROW_WPR 4
#endif
constexpr int kRowWPR = STAND_ROW_WPR, kRowWPRFewRows = 16;
constexpr int kRowsFew = 768;               // at most this many rows: kRowWPRFewRows waves per row
constexpr int kRowsMany = 8192;             // more rows than this: the step's automatic plan keeps the separate launches
constexpr int kMaxNodes = 1024;
constexpr int kMaxDepth = 31;
constexpr int kPathThreads = 256;
constexpr float kFastEps = 5e-5f;  // bound on the relative error of the fast normaliser

enum StatSlot {
    kStatHits = 0,  // kStatHits + n, n = 1..8
    kStatMisses = 9, kStatInserts, kStatMerges, kStatDrops, kStatNear, kStatTokens, kStatTests, kStatMismatch,
    kStatWaitExpired,
    kStatLatePaths,  // accepted paths that reach below the tree levels whose rows the one-launch step schedules first
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

// Loads and stores of data that another workgroup of the SAME launch writes or reads (the one-launch
// step): performed at device scope, so they go past the caches that are private to a part of the device
// -- no cache-wide write-back or invalidation is needed to exchange a few words.  A producer waits for
// its stores (publish_fence), then moves a counter; a consumer that has seen the counter (consume_fence)
// reads with ld_agent.  Between kernels they behave like ordinary accesses.
template <typename T>
__device__ __forceinline__ T ld_agent(const T *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename T>
__device__ __forceinline__ void st_agent(T *p, T v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void publish_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");  // orders the stores before what follows ...
    __builtin_amdgcn_s_waitcnt(0);                           // ... and waits until the memory system has taken them
}
__device__ __forceinline__ void consume_fence() { __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup"); }

// Row results handed from a row's workgroup to the tail of the SAME launch (one-launch step) as
// self-validating 64-bit words: a single aligned store is seen whole or not at all, so the producer
// neither waits for its stores nor moves a counter (a wave that waits for a store to be acknowledged
// keeps its workgroup's place on the device occupied for microseconds), and the consumer polls the
// word it needs.  `row`: {maximum's bits, (tag & 0xFFFFFF) << 8 | outcome + 1}, tag = number of the
// one-launch step on the handle.  `top`: {logit's bits, id | (tag & 1) << 31}: every such launch
// rewrites every word, so a stale word always carries the other parity.
struct RowPub {
    unsigned long long *row;   // [B*N], or NULL: nothing is published (separate launches)
    unsigned long long *top;   // [B*N][K]
    unsigned tag;
};
__device__ __forceinline__ unsigned long long pack_row_pub(float m, int outcome, unsigned tag)
{
    return ((unsigned long long)(((tag & 0xFFFFFFu) << 8) | (unsigned)(outcome + 1)) << 32) | f2u(m);
}
__device__ __forceinline__ bool row_pub_there(unsigned long long w, unsigned tag) { return (unsigned)(w >> 40) == (tag & 0xFFFFFFu); }
__device__ __forceinline__ int row_pub_outcome(unsigned long long w) { return (int)((w >> 32) & 0xFFu) - 1; }
__device__ __forceinline__ float row_pub_max(unsigned long long w) { return u2f((uint32_t)w); }
__device__ __forceinline__ unsigned long long pack_top_pub(int32_t id, float l, unsigned tag)
{
    return ((unsigned long long)((uint32_t)id | ((tag & 1u) << 31)) << 32) | f2u(l);
}
__device__ __forceinline__ bool top_pub_there(unsigned long long w, unsigned tag) { return (unsigned)(w >> 63) == (tag & 1u); }
__device__ __forceinline__ int32_t top_pub_id(unsigned long long w) { return (int32_t)((w >> 32) & 0x7FFFFFFFu); }
__device__ __forceinline__ float top_pub_logit(unsigned long long w) { return u2f((uint32_t)w); }

// ---------------------------------------------------------------------------------------------
// Accept/reject sequence at one tree node, executed by one wave (lane i = stored id i).
// Returns the rank of the accepted child or -1.  With track_err the values r are taken to
// carry a relative error of at most eps and `near` reports a test that the error could flip.
// ---------------------------------------------------------------------------------------------
// Sum of the values of lanes 0..31 as a balanced pairwise tree: (x0 + x1) + (x2 + x3), then
// groups of 4, 8, 16 and finally the two rows of 16 lanes -- one rounding per addition, the
// same in every lane.  Lanes K..31 must hold +0.  Data-parallel-primitive moves only (no LDS).
template <int CTRL>
__device__ __forceinline__ float dpp_fetch_f32(float x)
{
    return u2f((uint32_t)__builtin_amdgcn_update_dpp(0, (int)f2u(x), CTRL, 0xF, 0xF, true));
}
__device__ __forceinline__ float wave_tree_sum(float x)
{
    x = x + dpp_fetch_f32<0xB1>(x);   // quad_perm [1,0,3,2]: neighbours
    x = x + dpp_fetch_f32<0x4E>(x);   // quad_perm [2,3,0,1]: pairs of pairs
    x = x + dpp_fetch_f32<0x141>(x);  // row_half_mirror: the two quads of 8 lanes
    x = x + dpp_fetch_f32<0x140>(x);  // row_mirror: the two halves of a row of 16
    const float lo = u2f((uint32_t)__builtin_amdgcn_readlane((int)f2u(x), 0));
    const float hi = u2f((uint32_t)__builtin_amdgcn_readlane((int)f2u(x), 16));
    return lo + hi;
}

// 64-bit key of lane i (i uniform)
__device__ __forceinline__ unsigned long long readlane_u64(unsigned long long v, int i)
{
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, i);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), i);
    return ((unsigned long long)hi << 32) | lo;
}

struct NodeResult { int accepted; int rounds; bool near; float r; float rho; };

// ch: the token of drafted child `lane` (lanes 0..nchild-1), so that the rounds wait on no memory.
// onehot (deterministic drafting, paper Sec. 3.1): the proposal of each round is the one-hot
// vector on that round's child instead of the renormalised stored means.
__device__ __forceinline__ NodeResult wave_node_outcome(int lane, int K, int32_t my_id, float my_mu, float my_p, int nchild,
                                        int32_t ch, uint64_t seed, uint32_t b, uint64_t step, int first_child,
                                        bool track_err, float eps, bool onehot)
{
    NodeResult res;
    res.accepted = -1; res.rounds = 0; res.near = false;
    const bool act = lane < K;
    nchild = nchild < kMaxK ? nchild : kMaxK;
    if (lane >= nchild) ch = -1;
    const float om_l = lane < nchild ? uniform(seed, b, step, (uint32_t)(first_child + lane), 0u, kStreamAccept) : 0.0f;
    float w = (act && my_mu > 0.0f) ? my_mu : 0.0f;
    float zw = wave_tree_sum(w);
    w = zw > 0.0f ? w / zw : 0.0f;
    float r = act ? my_p : 0.0f;
    float rho = 1.0f;
    float err = track_err ? eps * r : 0.0f;
    for (int j = 0; j < nchild; ++j) {
        const int32_t x = __builtin_amdgcn_readlane(ch, j);
        if (x < 0) break;
        const unsigned long long mask = __ballot(act && my_id == x);
        if (!mask) break;
        const int i = __ffsll((long long)mask) - 1;
        if (onehot) w = lane == i ? 1.0f : 0.0f;
        const float wi = u2f((uint32_t)__builtin_amdgcn_readlane((int)f2u(w), i));
        const float ri = u2f((uint32_t)__builtin_amdgcn_readlane((int)f2u(r), i));
        const float ei = u2f((uint32_t)__builtin_amdgcn_readlane((int)f2u(err), i));
        const float om = u2f((uint32_t)__builtin_amdgcn_readlane((int)f2u(om_l), j));
        const float lhs = om * wi;
        res.rounds++;
        if (track_err && fabsf(lhs - ri) <= ei + 4e-7f * ri) res.near = true;
        if (lhs < ri) { res.accepted = j; break; }
        const float mn = act ? (r < w ? r : w) : 0.0f;
        const float w_next = lane == i ? 0.0f : w;  // the rejected token leaves the proposal
        const float M = wave_tree_sum(mn), zw2 = wave_tree_sum(w_next);
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
        if (!onehot) w = zw2 > 0.0f ? w_next / zw2 : 0.0f;
    }
    res.r = r;
    res.rho = rho;
    return res;
}

}  // namespace stand
