// kernels.hpp -- HIP kernels of the STAND speculation step for gfx950 (wave64).
//
//   row_pass_kernel     softmax statistics + top-K of every logits row in one streaming pass, and
//                       the accept/reject outcome of the row's tree node      (paper Sec. 4.1, 3.2)
//   path_exact_kernel   exact integer partial sums of the rows on the accepted path; walks the
//                       path and gathers the stop node's proposal             (paper Sec. 3.2)
//   path_finish_kernel  observation of each path row with the exact normaliser, replay of the
//                       stop node, resampled token by inverting the residual's cumulative
//                       integer mass; claims the table slots of the merge     (paper Sec. 3.2, 4.1)
//   merge_apply_kernel  running-mean merge into the open-addressing table     (paper Sec. 4.1)
//   draft_kernel        multi-level lookup + Gumbel-Top-K along the static tree (paper Sec. 4.2)
//   commit_scan_kernel  top-K of caller-given rows (update without verify)
//
// The row pass is the only kernel that touches all of the logits; it is bound by HBM bandwidth.
// Its softmax normaliser uses the hardware exp2 and float accumulation (relative error below
// the 5e-5 bound assumed here); every accept test whose margin is inside that bound, and
// every probability that is stored in the table or used for resampling, is recomputed with
// the exact integer normaliser of numeric.hpp, so all decisions are those of exact arithmetic.
// The kernels after the row pass are chains of dependent memory round trips over little data;
// workgroups exchange data only across kernel boundaries (no device-scope atomics or fences).
#pragma once
#include "numeric.hpp"

namespace stand {

constexpr int kDtBf16 = 0, kDtF32 = 1;
// Row pass: one row per workgroup of WPR waves.  Four waves per row fill the device when there
// are thousands of rows; with few rows (one or a few trajectories) a row is spread over sixteen
// waves so that the pass is not limited by what four waves can keep in flight.
constexpr int kRowWPR = 4, kRowWPRFewRows = 16;
constexpr int kRowsFew = 768;               // at most this many rows: kRowWPRFewRows waves per row
constexpr int kMaxNodes = 1024;
constexpr int kMaxDepth = 31;
constexpr int kPathThreads = 256;
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

// ---------------------------------------------------------------------------------------------
// Row pass: kRowWPR waves share one logits row, each streaming every kRowWPR-th batch of it with
// no synchronisation until the row's end.  A wave keeps kRowPF batches of kRowU 16-byte vectors
// per lane in flight (non-temporal buffer loads), a wave-uniform running maximum as the reference
// of the fast exponentials, and a small list of top-K candidates: one (maximum, index) record per
// vector whose maximum is not below the wave's current threshold, pruned by a ballot bisection.
// Everything that is the same in all lanes of a wave (reference, threshold, list length, loop
// counters, the buffer descriptor) is kept in scalar registers.
// ---------------------------------------------------------------------------------------------
#ifndef STAND_ROW_U
#define STAND_ROW_U 3
#endif
#ifndef STAND_ROW_PF
#define STAND_ROW_PF 2
#endif
constexpr int kRowU = STAND_ROW_U;     // vectors per lane per batch
constexpr int kRowPF = STAND_ROW_PF;   // batches in flight per wave
constexpr int kWaveCap = 192;          // vector records per wave (pruned when above kWavePrune)
constexpr int kWavePrune = 128;

constexpr int kElemCap = 8 * kMaxK + 64;  // element candidates at the end of a row (<= 8 per kept vector + edges)

struct WaveScan {
    unsigned long long buf[kWaveCap + 8];   // vector records: (maximum of the vector, vector index)
    unsigned long long top[kMaxK];      // pruned / final keys, best first
};

// 16-byte load of data that is read once: marked non-temporal so that it does not displace
// the caches' contents (measured on this part: a bare read of the logits runs 12 % faster)
typedef uint32_t stream_u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_streamed(const uint4 *p)
{
    const stream_u32x4 t = __builtin_nontemporal_load((const stream_u32x4 *)p);
    return make_uint4(t.x, t.y, t.z, t.w);
}

__device__ __forceinline__ int lane_prefix_count(unsigned long long mask)
{
    return (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// a value that is the same in every lane, moved to a scalar register
__device__ __forceinline__ float uniform_f32(float x) { return u2f((uint32_t)__builtin_amdgcn_readfirstlane((int)f2u(x))); }

// maximum over the 64 lanes (all active), returned in a scalar register: four data-parallel-primitive
// steps inside each row of 16 lanes, then the four rows
__device__ __forceinline__ float wave_max_f32(float x)
{
    x = fmaxf(x, dpp_fetch_f32<0xB1>(x));   // quad_perm [1,0,3,2]
    x = fmaxf(x, dpp_fetch_f32<0x4E>(x));   // quad_perm [2,3,0,1]
    x = fmaxf(x, dpp_fetch_f32<0x141>(x));  // row_half_mirror
    x = fmaxf(x, dpp_fetch_f32<0x140>(x));  // row_mirror
    const float r0 = u2f((uint32_t)__builtin_amdgcn_readlane((int)f2u(x), 0));
    const float r1 = u2f((uint32_t)__builtin_amdgcn_readlane((int)f2u(x), 16));
    const float r2 = u2f((uint32_t)__builtin_amdgcn_readlane((int)f2u(x), 32));
    const float r3 = u2f((uint32_t)__builtin_amdgcn_readlane((int)f2u(x), 48));
    return uniform_f32(fmaxf(fmaxf(r0, r1), fmaxf(r2, r3)));
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
    // the same in every lane: returned in scalar registers
    return n >= K ? readlane_u64(top[K - 1], 0) : 0ull;
}

struct WaveScanState {
    unsigned long long theta_key;  // only records above it can enter the list
    float theta_val;               // value of theta_key (-inf if none): cheap pre-filter
    int cnt;                       // records in ws->buf (wave-uniform)
};

__device__ __forceinline__ void set_theta(WaveScanState &st, unsigned long long key)
{
    // wave-uniform state is kept in scalar registers
    key = readlane_u64(key, 0);
    st.theta_key = key;
    st.theta_val = uniform_f32(key ? rank_key_value(key) : -__builtin_inff());
}

// Prune the record list to its K best; they stay in ws->buf, the K-th best becomes the threshold.
__device__ __forceinline__ void wave_prune(WaveScan *ws, WaveScanState &st, int lane, int K)
{
    const unsigned long long th = wave_select(ws->buf, ws->top, lane, K, st.cnt);
    const int keep = st.cnt < K ? st.cnt : K;
    if (lane < keep) ws->buf[lane] = ws->top[lane];
    __builtin_amdgcn_wave_barrier();
    st.cnt = __builtin_amdgcn_readfirstlane(keep);
    if (th) set_theta(st, th);
}

// While a row is streamed the list holds raw records, (bits of the vector maximum) << 32 | vector
// index, which cost nothing to build; ranking keys are made from them when the list is pruned.
__device__ __forceinline__ unsigned long long raw_record(float cm, uint32_t vec)
{
    return ((unsigned long long)f2u(cm) << 32) | vec;
}
__device__ __forceinline__ unsigned long long key_of_raw(unsigned long long raw)
{
    return rank_key(u2f((uint32_t)(raw >> 32)), (uint32_t)raw);
}
__device__ __forceinline__ unsigned long long raw_of_key(unsigned long long key)
{
    return raw_record(rank_key_value(key), rank_key_id(key));
}

// Cheap prune: finds, by bisection on the upper key word (the vector maximum) with ballots, a
// threshold that at least K records reach, and keeps those records (unsorted; records whose
// maximum equals the threshold all stay).  RAW_IN / KEYS_OUT say whether the list holds raw
// records or ranking keys before / after.  Falls back to the exact prune when ties leave too
// many records.
// Every record's upper key word lies in [lo_word, hi_word] (the current threshold and the key of
// the largest value seen; 0 and ~0 if unknown), so the bits the two bounds share are not searched;
// LOWBIT is the lowest bit that can differ between two values of the logits' type (16 for bf16,
// whose binary32 images have sixteen constant low bits per sign).
constexpr int kPruneSlack = 16;
template <bool RAW_IN, bool KEYS_OUT, int LOWBIT>
__device__ __forceinline__ void wave_prune_fast(WaveScan *ws, WaveScanState &st, int lane, int K, uint32_t lo_word,
                                                uint32_t hi_word)
{
    const int n = st.cnt;  // <= kWaveCap = 3 * 64
    unsigned long long e0 = lane < n ? ws->buf[lane] : 0ull;
    unsigned long long e1 = 64 + lane < n ? ws->buf[64 + lane] : 0ull;
    unsigned long long e2 = 128 + lane < n ? ws->buf[128 + lane] : 0ull;
    if (RAW_IN) {  // ranking keys of existing records are never zero
        e0 = lane < n ? key_of_raw(e0) : 0ull;
        e1 = 64 + lane < n ? key_of_raw(e1) : 0ull;
        e2 = 128 + lane < n ? key_of_raw(e2) : 0ull;
    }
    const uint32_t h0 = (uint32_t)(e0 >> 32), h1 = (uint32_t)(e1 >> 32), h2 = (uint32_t)(e2 >> 32);
    uint32_t t = 0u;
    if (n > K) {
        const uint32_t diff = lo_word ^ hi_word;
        int top = -1;  // highest bit in which the bounds differ
        if (diff) {
            top = 31 - __builtin_clz(diff);
            t = top == 31 ? 0u : (hi_word & ~((2u << top) - 1u));
        } else {
            t = hi_word;
        }
        for (int bit = top; bit >= LOWBIT; --bit) {
            const uint32_t cand = t | (1u << bit);
            const int c = __popcll(__ballot(h0 >= cand)) + __popcll(__ballot(h1 >= cand)) + __popcll(__ballot(h2 >= cand));
            if (c >= K) {
                t = cand;
                if (c == K) break;
            }
        }
    }
    // n > K: at least K records have an upper word >= t > 0; otherwise t = 0 keeps every record
    const bool k0 = lane < n && h0 >= t, k1 = 64 + lane < n && h1 >= t, k2 = 128 + lane < n && h2 >= t;
    __builtin_amdgcn_wave_barrier();
    const unsigned long long b0 = __ballot(k0), b1 = __ballot(k1), b2 = __ballot(k2);
    const int c0 = __popcll(b0), c1 = __popcll(b1);
    const bool keys_now = KEYS_OUT || !RAW_IN;
    if (k0) ws->buf[lane_prefix_count(b0)] = (RAW_IN && !KEYS_OUT) ? raw_of_key(e0) : e0;
    if (k1) ws->buf[c0 + lane_prefix_count(b1)] = (RAW_IN && !KEYS_OUT) ? raw_of_key(e1) : e1;
    if (k2) ws->buf[c0 + c1 + lane_prefix_count(b2)] = (RAW_IN && !KEYS_OUT) ? raw_of_key(e2) : e2;
    __builtin_amdgcn_wave_barrier();
    st.cnt = __builtin_amdgcn_readfirstlane(c0 + c1 + __popcll(b2));
    if (t) {
        const unsigned long long key = (unsigned long long)t << 32;
        if (key > st.theta_key) { st.theta_key = key; st.theta_val = uniform_f32(order_key_inv(t)); }
    }
    if (st.cnt > K + kPruneSlack) {
        // too many ties at the threshold: rank exactly (on keys), then restore the list's form
        if (!keys_now) {
            for (int i = lane; i < st.cnt; i += 64) ws->buf[i] = key_of_raw(ws->buf[i]);
            __builtin_amdgcn_wave_barrier();
        }
        wave_prune(ws, st, lane, K);
        if (!keys_now) {
            if (lane < st.cnt) ws->buf[lane] = raw_of_key(ws->buf[lane]);
            __builtin_amdgcn_wave_barrier();
        }
    }
}

// Lanes with `pred` append the raw record (cm, vec); prune above kWavePrune records.
template <int LOWBIT>
__device__ __forceinline__ void wave_offer(WaveScan *ws, WaveScanState &st, int lane, int K, bool pred, float cm,
                                           uint32_t vec, float seen_max)
{
    const unsigned long long bal = __ballot(pred);
    if (!bal) return;
    if (pred) ws->buf[st.cnt + lane_prefix_count(bal)] = raw_record(cm, vec);
    st.cnt = __builtin_amdgcn_readfirstlane(st.cnt + __popcll(bal));
    __builtin_amdgcn_wave_barrier();
    if (st.cnt > kWavePrune)
        wave_prune_fast<true, false, LOWBIT>(ws, st, lane, K, (uint32_t)(st.theta_key >> 32), order_key(seen_max));
}

// Leaves the row's K best element keys (value desc, id asc) sorted in ws->top[0..K), returns
// the row maximum and the fast normaliser sum_v 2^((l_v - m) c).
//
// While streaming, only one record per 16-byte vector is kept: its maximum.  The K vectors
// with the largest maxima (ties: lower index) contain the K best elements, so the elements
// are ranked only at the end, among those kept vectors.
struct WavePartial {
    float m_ref, s;   // reference maximum of this wave's part and its fast sum relative to it
    int cnt;          // vector records left in ws->buf: the wave's K best and at most kPruneSlack more, unsorted
};

// Streaming part: wave `wsub` of `wpr` cooperating waves takes every wpr-th batch of the row.
template <int DT>
__device__ __forceinline__ WavePartial wave_row_stream(const void *rowp, int V, float c, int K, WaveScan *ws, int lane,
                                                       int wsub, int wpr)
{
    constexpr int EPV = VecTraits<DT>::EPV;
    constexpr int U = kRowU, PF = kRowPF;
    constexpr int LOWBIT = DT == kDtBf16 ? 16 : 0;
    // the row and the wave's share of it are the same in every lane: keep them in scalar registers
    rowp = (const void *)readlane_u64((unsigned long long)rowp, 0);
    wsub = __builtin_amdgcn_readfirstlane(wsub);
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
        const float nm = uniform_f32(fmaxf(wave_max_f32(cm), m_ref));
        s_t *= fast_exp2((m_ref - nm) * c);
        m_ref = nm;
        nb = -nm * c;
    };
    // Loads are issued unconditionally (indices clamped to the last vector) so that the number of
    // loads in flight is the same on every path and only the oldest batch is waited for.
    // Buffer loads: the descriptor (scalar registers) covers the row from the batch's first byte
    // to the row's end, every lane's offset is the constant 16 * lane + 1024 * u, and a lane past
    // the end gets zeros from the hardware's range check -- no address arithmetic in vector
    // registers and no access outside the row.
    const uint32_t row_bytes = (uint32_t)g.nvec * 16u;
    const int lane_off = lane * 16;
    auto load_batch = [&](uint4 (&w)[U], int k) {
        const uint32_t want = (uint32_t)((k * wpr + wsub) * U) * 1024u;
        const uint32_t off = want < row_bytes ? want : row_bytes;
        const __amdgpu_buffer_rsrc_t rsrc =
            __builtin_amdgcn_make_buffer_rsrc((void *)((const char *)g.vp + off), (short)0, (int)(row_bytes - off), 0x00020000);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const stream_u32x4 t = __builtin_amdgcn_raw_buffer_load_b128(rsrc, lane_off + u * 1024, 0, 2 /* non-temporal */);
            w[u] = make_uint4(t.x, t.y, t.z, t.w);
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
        if (__ballot(valid && cm >= st.theta_val))
            wave_offer<LOWBIT>(ws, st, lane, K, valid && cm >= st.theta_val, cm, (uint32_t)idx, m_ref);
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

    // leave at most K + kPruneSlack ranking keys, the wave's K best among them, in ws->buf
    wave_prune_fast<true, true, LOWBIT>(ws, st, lane, K, (uint32_t)(st.theta_key >> 32), order_key(m_ref));
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
__device__ __forceinline__ void wave_row_finish(const void *rowp, int V, int K, WaveScan *ws, unsigned long long *ebuf,
                                                int lane, int cnt)
{
    constexpr int EPV = VecTraits<DT>::EPV;
    const RowGeom g = row_geom<DT>(rowp, V);
    int edge_id = -1;
    if (lane < g.head) edge_id = lane;
    else if (lane < g.head + g.ntail) edge_id = g.tail0 + (lane - g.head);
    const float edge_val = edge_id >= 0 ? load_scalar<DT>(rowp, edge_id) : -__builtin_inff();

    {
        // cut the merged list down cheaply before the exact ranking
        WaveScanState st;
        st.cnt = cnt;
        set_theta(st, 0ull);
        wave_prune_fast<false, true, DT == kDtBf16 ? 16 : 0>(ws, st, lane, K, 0u, ~0u);
        cnt = st.cnt;
    }
    const unsigned long long th_vec = wave_select(ws->buf, ws->top, lane, K, cnt);
    const int kept = cnt < K ? cnt : K;
    const float th_val = th_vec ? rank_key_value(th_vec) : -__builtin_inff();
    int ne = 0;
    {
        const unsigned long long eb = __ballot(edge_id >= 0 && edge_val >= th_val);
        if (edge_id >= 0 && edge_val >= th_val) ebuf[lane_prefix_count(eb)] = rank_key(edge_val, (uint32_t)edge_id);
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
            if (pred) ebuf[ne + lane_prefix_count(bal)] = rank_key(x[j], (uint32_t)(g.head + (int)vec * EPV + j));
            ne += __popcll(bal);
        }
    }
    __builtin_amdgcn_wave_barrier();
    wave_select(ebuf, ws->top, lane, K, ne);
}

// floor(e * 2^40) for e in [0, 1] as hi * 2^20 + lo with hi = floor(e * 2^20) <= 2^20 and
// lo = floor((e * 2^20 - hi) * 2^20) < 2^20; every step is exact in binary32.
__device__ __forceinline__ void fixed_split(float e, uint32_t &hi, uint32_t &lo)
{
    const float t = e * 0x1p20f;
    hi = (uint32_t)t;
    const float r = t - (float)hi;
    lo = (uint32_t)(r * 0x1p20f);
}

// Exact fixed-point sum over the vectors [v0, v1) of a row (plus the edge elements if with_edge),
// strided over `nthreads` threads; returns this thread's partial sum_v floor(E((l_v - m) c) * 2^40).
template <int DT>
__device__ __forceinline__ unsigned long long thread_exact_partial(const void *rowp, const RowGeom &g, int v0, int v1,
                                                                   bool with_edge, float m, float c, int t, int nthreads)
{
    constexpr int EPV = VecTraits<DT>::EPV;
    unsigned long long S = 0ull;
    uint32_t ahi = 0, alo = 0;
    if (with_edge) {
        int edge_id = -1;
        if (t < g.head) edge_id = t;
        else if (t < g.head + g.ntail) edge_id = g.tail0 + (t - g.head);
        if (edge_id >= 0) {
            uint32_t hi, lo;
            fixed_split(exact_exp2(scaled_offset(load_scalar<DT>(rowp, edge_id), m, c)), hi, lo);
            ahi += hi; alo += lo;
        }
    }
    // four independent loads are issued before any of them is used (indices clamped, so the
    // number of loads in flight does not depend on the position in the row)
    const int vlast = v1 > v0 ? v1 - 1 : v0;
    auto add_vec = [&](const uint4 &w, int idx) {
        if (idx < v1) {
            float x[EPV];
            unpack<DT>(w, x);
#pragma unroll
            for (int j = 0; j < EPV; ++j) {
                uint32_t hi, lo;
                fixed_split(exact_exp2(scaled_offset(x[j], m, c)), hi, lo);
                ahi += hi; alo += lo;
            }
        }
    };
    for (int base = v0 + t; base < v1; base += 4 * nthreads) {
        const int i0 = base, i1 = base + nthreads, i2 = base + 2 * nthreads, i3 = base + 3 * nthreads;
        const uint4 w0 = g.vp[i0 < vlast ? i0 : vlast];
        const uint4 w1 = g.vp[i1 < vlast ? i1 : vlast];
        const uint4 w2 = g.vp[i2 < vlast ? i2 : vlast];
        const uint4 w3 = g.vp[i3 < vlast ? i3 : vlast];
        add_vec(w0, i0); add_vec(w1, i1); add_vec(w2, i2); add_vec(w3, i3);
        // at most 32 elements since the last flush: the 32-bit accumulators stay below 2^26
        S += ((unsigned long long)ahi << 20) + alo;
        ahi = 0; alo = 0;
    }
    return S + ((unsigned long long)ahi << 20) + alo;
}

// Exact normaliser of a row by one wave (rare path).
template <int DT>
__device__ unsigned long long wave_row_exact_sum(const void *rowp, int V, float m, float c, int lane)
{
    const RowGeom g = row_geom<DT>(rowp, V);
    unsigned long long S = thread_exact_partial<DT>(rowp, g, 0, g.nvec, true, m, c, lane, 64);
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
    bool onehot;                // deterministic drafting: one-hot proposals in the accept tests
    float eps;                  // relative error assumed for the fast normaliser (>= kFastEps)
};

template <int DT, int WPR>
__global__ __launch_bounds__(64 * WPR) void row_pass_kernel(RowPassArgs a)
{
    constexpr int ES = VecTraits<DT>::ES;
    __shared__ WaveScan wsh[WPR];
    __shared__ unsigned long long ebuf[kElemCap + 8];  // element keys offered to the row's final selection
    __shared__ float part_m[WPR], part_s[WPR];
    __shared__ int part_cnt[WPR];
    // the wave's number is the same in all its lanes: say so, so that everything derived from it
    // (its share of the row, the loop over its batches) is kept in scalar registers
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    // Workgroups are numbered node-major (all trajectories' rows of node 0, then of node 1, ...).
    // The nodes near the root carry drafted children, whose accept tests make the end of their
    // row the longest; started first, those ends overlap with the streaming of later rows, and the
    // rows that finish the kernel are leaves.
    const int slot = blockIdx.x;
    const int row = slot < a.B * a.N ? (slot % a.B) * a.N + slot / a.B : slot;
    const bool live = row < a.B * a.N;
    WaveScan *ws = &wsh[wave];
    const int b = live ? row / a.N : 0, u = live ? row % a.N : 0;
    const char *rowp = (const char *)a.logits + (size_t)(live ? row : 0) * (size_t)a.V * ES;
    float m, s;
    // The proposal of this node (needed for the accept tests at the end) is requested by the
    // finishing wave as soon as it has streamed its part, so that its two dependent round trips
    // to memory pass while the row is being ranked.
    int nch = 0, fc = -1;
    int32_t my_id = -1, ch = -1;
    float my_mu = 0.0f, my_l = 0.0f;
    auto request_proposal = [&]() {
        fc = a.tree.first_child[u];
        nch = a.draft_has[row];  // children drafted from this node's table entry (0: none)
        if (lane < a.K) {
            my_id = a.draft_qid[(size_t)row * a.K + lane];
            my_mu = a.draft_qmu[(size_t)row * a.K + lane];
        }
    };
    auto request_proposal_logits = [&]() {
        if (nch == 0) return;  // uniform over the wave
        if ((uint32_t)my_id >= (uint32_t)a.V) { my_id = -1; my_mu = 0.0f; }  // never index outside the row
        else my_l = load_scalar<DT>(rowp, my_id);
        if (lane < nch && lane < kMaxK && fc >= 0 && fc + lane < a.N) ch = a.draft_tok[(size_t)b * a.N + fc + lane];
    };
    // ---- accept / reject outcome of this node's children (paper Sec. 3.2, applied recursively)
    auto node_tests = [&](float m, float s) {
        if (nch == 0) {  // uniform over the wave
            if (lane == 0) a.outcome[row] = -1;
            return;
        }
        const float e = (lane < a.K && my_id >= 0) ? exact_exp2(scaled_offset(my_l, m, a.c)) : 0.0f;
        NodeResult nr = wave_node_outcome(lane, a.K, my_id, my_mu, e / s, nch, ch, a.seed, (uint32_t)b, a.step, fc,
                                          true, a.eps, a.onehot);
        if (nr.near) {
            // a test fell inside the error bound of the fast normaliser: decide with the exact one
            const unsigned long long S = wave_row_exact_sum<DT>(rowp, a.V, m, a.c, lane);
            const float sx = normaliser_from_fixed(S);
            nr = wave_node_outcome(lane, a.K, my_id, my_mu, e / sx, nch, ch, a.seed, (uint32_t)b, a.step, fc, false,
                                   0.0f, a.onehot);
            if (lane == 0) atomicAdd(&a.stats[kStatNear], 1ull);
        }
        if (lane == 0) a.outcome[row] = nr.accepted;
    };
    // Wave 0 ranks the row at its end, wave 1 runs the accept tests meanwhile.
    static_assert(WPR >= 2, "a row is shared by at least two waves");
    constexpr int kTestWave = 1;
    if (live) {
        const WavePartial wp = wave_row_stream<DT>(rowp, a.V, a.c, a.K, ws, lane, wave, WPR);
        if (lane == 0) { part_m[wave] = wp.m_ref; part_s[wave] = wp.s; part_cnt[wave] = wp.cnt; }
        if (wave == kTestWave) request_proposal();
    }
    __syncthreads();
    if (!live) return;
    // both finishing waves form the row's maximum and normaliser with the same expressions, so
    // they hold the same m and s (the ranking's maximum, top[0], has no negative zero either)
    m = part_m[0];
    for (int q = 1; q < WPR; ++q) m = fmaxf(m, part_m[q]);
    m = m + 0.0f;
    s = 0.0f;
    for (int q = 0; q < WPR; ++q) s += part_s[q] * fast_exp2((part_m[q] - m) * a.c);
    if (wave == kTestWave) {
        // the accept tests need the row's maximum and normaliser, not its ranking
        request_proposal_logits();
        node_tests(m, s);
        return;
    }
    if (wave != 0) return;
    // gather the partner waves' records behind this wave's own (each list holds at most
    // K + kPruneSlack ranking keys); with many partners the list is cut down on the way
    int cnt = part_cnt[0];
    for (int q = 1; q < WPR; ++q) {
        const int cq = part_cnt[q];
        if (cnt + cq > kWavePrune) {
            WaveScanState gs;
            gs.cnt = cnt;
            set_theta(gs, 0ull);
            __builtin_amdgcn_wave_barrier();
            wave_prune_fast<false, true, DT == kDtBf16 ? 16 : 0>(ws, gs, lane, a.K, 0u, ~0u);
            cnt = gs.cnt;
        }
        if (lane < cq) ws->buf[cnt + lane] = wsh[q].buf[lane];
        cnt += cq;
    }
    __builtin_amdgcn_wave_barrier();
    wave_row_finish<DT>(rowp, a.V, a.K, ws, ebuf, lane, cnt);

    if (lane < a.K) {
        const unsigned long long key = ws->top[lane];
        const float l = rank_key_value(key);
        a.top_idx[(size_t)row * a.K + lane] = (int32_t)rank_key_id(key);
        a.top_l[(size_t)row * a.K + lane] = l;
        a.top_p[(size_t)row * a.K + lane] = exact_exp2(scaled_offset(l, m, a.c)) / s;
    }
    if (lane == 0) { a.row_m[row] = m; a.row_s[row] = s; }
}

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
__device__ __forceinline__ unsigned long long fixed_mass(float e)
{
    uint32_t hi, lo;
    fixed_split(e, hi, lo);
    return ((unsigned long long)hi << 20) + lo;
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
        if (a.all_nodes) node = a.draft_tok[(size_t)b * a.N + jj] >= 0 ? jj : -1;
        else if (a.mode != 0) node = commit_row_of(a, b, jj);
        else if (jj == 0) node = 0;
        else {
            if (len < 0) {
                // most trajectories stop at the root: then there is no row below it and nothing to stage
                if (a.outcome[(size_t)b * a.N] < 0) return;
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
        unsigned long long S = thread_exact_partial<DT>(rowp, g, v0, v1, seg == 0, m, a.c, tid, kPathThreads);
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
};

// masked integer masses of the EPV elements of vector idx (elements e0 .. e0 + EPV - 1 of the row)
template <int DT>
__device__ __forceinline__ void vector_masses(const uint4 &w, int e0, float m, float c, const FinishShared &sh,
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
    for (int q = 0; q < EPV; ++q) f[q] = ((bits >> q) & 1u) ? 0ull : fixed_mass(exact_exp2(scaled_offset(x[q], m, c)));
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
    int R;                            // record slots per trajectory: W, or N in all-nodes mode
    bool all_nodes;                   // record (b, j, n) observes drafted node j under its path's context
    bool replace;                     // an existing entry becomes the newest observation (no running mean)
    const int32_t *draft_tok;         // [B][N]
    const int32_t *depth;             // [N]
    const int32_t *recent;            // [B][N][kMaxOrder] recent[.][i]: token i positions before the end of node's sequence
    long long *rec_slot;              // [B*R*NO]
    const int32_t *obs_idx;
    const float *obs_p;
    unsigned long long *stats;
};

// transient use of the slot header between claiming and applying the records of one merge
constexpr uint32_t kTagShift = 8, kTagMax = 0x7FFFFFu, kMultiBit = 0x80000000u;

__device__ __forceinline__ int clamp_len(int len, int W) { return len < 0 ? 0 : (len > W ? W : len); }

// claims the table slot of merge record rec = (b, position j, order n); run by one thread
__device__ __forceinline__ void merge_claim_record(const MergeArgs &a, int rec)
{
    const int NO = a.omax - a.omin + 1;
    if (rec >= a.B * a.R * NO) return;
    const int n = a.omin + rec % NO;
    const int j = (rec / NO) % a.R;
    const int b = rec / (NO * a.R);
    long long slot_out = -1;
    const long long base_len = a.ctx_len[b];
    bool valid;
    if (a.all_nodes) {
        valid = a.draft_tok[(size_t)b * a.N + j] >= 0 && base_len + a.depth[j] >= n;
    } else {
        const int len = clamp_len(a.commit_len[b], a.W);
        valid = j < len && base_len + j >= n;
        if (valid && a.commit_row) {
            const int r = a.commit_row[(size_t)b * a.W + j];
            valid = r >= 0 && r < a.N;
        }
    }
    if (valid) {
        int32_t key[kMaxOrder];
        for (int i = 0; i < n; ++i) {
            if (a.all_nodes) {
                // the last n tokens of context ++ path to node j, as the draft kernel left them
                key[i] = a.recent[((size_t)b * a.N + j) * kMaxOrder + (n - 1 - i)];
                continue;
            }
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
            if (old == 0ull || old == fp) {
                atomicAdd(&a.stats[old == 0ull ? kStatInserts : kStatMerges], 1ull);
                // Until the records are applied the order word also carries the smallest record
                // number that claimed the slot (stored inverted, so that atomicMax keeps it), and
                // the top bit of the count word says that more than one record did.
                const uint32_t tag = ((kTagMax - (uint32_t)rec) << kTagShift) | (uint32_t)n;
                const uint32_t before = atomicMax(&h->order, tag);
                if (before >> kTagShift) atomicOr(&h->count, kMultiBit);
                slot_out = (long long)slot; placed = true; break;
            }
        }
        if (!placed) atomicAdd(&a.stats[kStatDrops], 1ull);
    }
    a.rec_slot[rec] = slot_out;
}

// See the comment above PathArgs.  Blocks [0, finish_blocks) finish path row (b, j) =
// (block / W, block % W); the blocks after them claim merge records, kFinishThreads per block.
template <int DT>
__global__ __launch_bounds__(kFinishThreads) void path_finish_kernel(PathArgs a, MergeArgs mg, int finish_blocks)
{
    constexpr int ES = VecTraits<DT>::ES, EPV = VecTraits<DT>::EPV;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    if ((int)blockIdx.x >= finish_blocks) {
        merge_claim_record(mg, ((int)blockIdx.x - finish_blocks) * kFinishThreads + tid);
        return;
    }
    __shared__ FinishShared sh;
    const int j = (int)blockIdx.x / a.B, b = (int)blockIdx.x % a.B;  // slot-major, as in path_exact_kernel
    // Everything whose address depends on (b, j) only is requested at once: the partial sums and,
    // in verify mode, the stop record of the trajectory (used if this turns out to be its stop row).
    const int nseg = a.nseg;
    const unsigned long long part = (wave == 0 && lane < nseg) ? a.seg_part[((size_t)b * a.R + j) * kSegMax + lane] : 0ull;
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
        if (a.all_nodes) node = a.draft_tok[(size_t)b * a.N + j] >= 0 ? j : -1;
        else node = j < len ? (j == len - 1 ? stop_node : a.out_node[(size_t)b * a.W + j]) : -1;
        stop = node >= 0 && node == stop_node;
    } else {
        node = a.all_nodes ? (a.draft_tok[(size_t)b * a.N + j] >= 0 ? j : -1) : commit_row_of(a, b, j);
        m = 0.0f;
    }
    if (node < 0) return;  // block-uniform
    if (!stop && wave != 0) return;
    const int row = b * a.N + node;
    const int src = a.mode == 0 ? row : b * a.R + j;
    const char *rowp = (const char *)a.logits + (size_t)row * (size_t)a.V * ES;
    if (!stop) m = a.src_m[src];
    const RowGeom g = row_geom<DT>(rowp, a.V);
    const int per = (g.nvec + nseg - 1) / nseg;

    if (wave == 0) {
        int32_t o_idx = 0;
        float o_l = 0.0f;
        if (lane < a.K) { o_idx = a.src_top_idx[(size_t)src * a.K + lane]; o_l = a.src_top_l[(size_t)src * a.K + lane]; }
        if (!stop || nch <= 0 || lane >= a.K) { my_id = -1; my_mu = 0.0f; }
        const float my_e = my_id >= 0 ? exact_exp2(scaled_offset(my_l, m, a.c)) : 0.0f;
        int edge_id = -1;
        if (stop) {
            if (lane < g.head) edge_id = lane;
            else if (lane < g.head + g.ntail) edge_id = g.tail0 + (lane - g.head);
        }
        const unsigned long long edge_f =
            edge_id >= 0 ? fixed_mass(exact_exp2(scaled_offset(load_scalar<DT>(rowp, edge_id), m, a.c))) : 0ull;

        const unsigned long long S = wave_sum_u64(part);
        const float s = normaliser_from_fixed(S);
        if (!stop) {
            // observation of this row (paper Sec. 4.1: top-k ids and probabilities)
            if (lane < a.K) {
                a.obs_idx[((size_t)b * a.R + j) * a.K + lane] = o_idx;
                a.obs_p[((size_t)b * a.R + j) * a.K + lane] = exact_exp2(scaled_offset(o_l, m, a.c)) / s;
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
            a.obs_idx[((size_t)b * a.R + j) * a.K + lane] = o_idx;
            a.obs_p[((size_t)b * a.R + j) * a.K + lane] = exact_exp2(scaled_offset(o_l, m, a.c)) / s;
        }
        // ---- integer masses (unit 2^-40 / s * rho): support token i weighs floor(r_i * (S / rho)),
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
                my_f = fixed_mass(my_e);
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
    const int cpt = (ve - vs + kFinishThreads - 1) / kFinishThreads;
    const int r0 = vs + tid * cpt < ve ? vs + tid * cpt : ve;
    const int r1 = r0 + cpt < ve ? r0 + cpt : ve;
    // four independent loads per round (indices clamped, unused vectors skipped)
    const int rlast = r1 > r0 ? r1 - 1 : r0;
    unsigned long long mine = 0ull;
    auto vec_sum = [&](const uint4 &w, int idx) {
        if (idx < r1) {
            unsigned long long f[EPV];
            vector_masses<DT>(w, g.head + idx * EPV, m, a.c, sh, f);
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
            vector_masses<DT>(g.vp[r0], g.head + r0 * EPV, m, a.c, sh, f1);
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
                vector_masses<DT>(w, g.head + idx * EPV, m, a.c, sh, f);
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
        a.out_tok[(size_t)b * a.W + (len - 1)] = a.src_top_idx[(size_t)src * a.K];
        atomicAdd(&a.stats[kStatMismatch], 1ull);
    }
}

// One wave per record, kMergeWaves records per workgroup (most records of a step do not exist --
// paths are short -- and a launch of one small workgroup per record spends its time dispatching
// them).  The lowest record that claimed a slot (its leader, named in the slot header by the
// claim) applies all records of that slot in record order; the other records' waves leave at
// once.  A slot claimed by one record only needs no search for followers.  The waves of a
// workgroup do not interact.
constexpr int kMergeWaves = 16;
__global__ __launch_bounds__(64 * kMergeWaves) void merge_apply_kernel(MergeArgs a)
{
    __shared__ int32_t l_id_all[kMergeWaves][2 * kMaxK];
    __shared__ float l_val_all[kMergeWaves][2 * kMaxK];
    const int NO = a.omax - a.omin + 1;
    const int nrec = a.B * a.R * NO;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int rec = (int)blockIdx.x * kMergeWaves + wave;
    if (rec >= nrec) return;
    int32_t *l_id = l_id_all[wave];
    float *l_val = l_val_all[wave];
    const int K = a.K;
    const long long slot = a.rec_slot[rec];
    if (slot < 0) return;
    SlotHeader *h = slot_header(a.table, (uint64_t)slot, a.slot_bytes);
    int32_t *ids = slot_ids(a.table, (uint64_t)slot, a.slot_bytes);
    float *mus = slot_mu(a.table, (uint64_t)slot, a.slot_bytes, K);
    // header, stored entry and this record's observation are requested together
    const uint32_t order_word = h->order;
    uint32_t count = h->count;
    int32_t e_id = -1;
    float e_mu = 0.0f;
    if (lane < K) { e_id = ids[lane]; e_mu = mus[lane]; }
    // lanes 0..K-1: stored entry; lanes 32..32+K-1: observation
    int32_t o_id = -1;
    float o_p = 0.0f;
    if (lane >= 32 && lane < 32 + K) {
        o_id = a.obs_idx[(size_t)(rec / NO) * K + (lane - 32)];
        o_p = a.obs_p[(size_t)(rec / NO) * K + (lane - 32)];
    }
    if (kTagMax - (order_word >> kTagShift) != (uint32_t)rec) return;  // another record leads this slot
    const bool multi = (count & kMultiBit) != 0u;
    count &= ~kMultiBit;
    if (count == 0) { e_id = -1; e_mu = 0.0f; }

    auto apply = [&](int32_t o_id, float o_p) {
        if (count == 0 || a.replace) {
            // first sight, or a table that keeps only the newest observation: the entry is the observation
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
                const int32_t sid = __builtin_amdgcn_readlane(e_id, q);
                const int32_t oid = __builtin_amdgcn_readlane(o_id, 32 + q);
                const float op = u2f((uint32_t)__builtin_amdgcn_readlane((int)f2u(o_p), 32 + q));
                if (lane < 32 && act && oid == id) other = op;
                if (lane >= 32 && act && sid == id) dup = true;
            }
            float val;
            if (lane < 32) { float t = cf * e_mu; t = t + other; val = t / denom; }
            else { float t = cf * 0.0f; t = t + o_p; val = t / denom; act = act && !dup; }
            const unsigned long long key = act ? rank_key(val, (uint32_t)id) : 0ull;
            int rank = 0;
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                rank += readlane_u64(key, q) > key ? 1 : 0;
                rank += readlane_u64(key, 32 + q) > key ? 1 : 0;
            }
            if (K > 16) {  // the other lanes are inactive (key 0) for K <= 16
#pragma unroll
                for (int q = 16; q < 32; ++q) {
                    rank += readlane_u64(key, q) > key ? 1 : 0;
                    rank += readlane_u64(key, 32 + q) > key ? 1 : 0;
                }
            }
            if (act && rank < K) { l_id[rank] = id; l_val[rank] = val; }
            __builtin_amdgcn_wave_barrier();  // the wave's own part of shared memory: no other wave is involved
            if (lane < K) { e_id = l_id[lane]; e_mu = l_val[lane]; }
            __builtin_amdgcn_wave_barrier();
        }
        count++;
    };

    apply(o_id, o_p);
    if (multi) {
        // the later records of this slot, in record order
        for (int base = rec + 1; base < nrec; base += 64) {
            const int r = base + lane;
            unsigned long long hits = __ballot(r < nrec && a.rec_slot[r] == slot);
            while (hits) {
                const int bit = __ffsll((long long)hits) - 1;
                hits &= hits - 1;
                const int jb = (base + bit) / NO;  // = b * W + j
                int32_t f_id = -1;
                float f_p = 0.0f;
                if (lane >= 32 && lane < 32 + K) { f_id = a.obs_idx[(size_t)jb * K + (lane - 32)]; f_p = a.obs_p[(size_t)jb * K + (lane - 32)]; }
                apply(f_id, f_p);
            }
        }
    }
    if (lane < K) { ids[lane] = e_id; mus[lane] = e_mu; }
    if (lane == 0) { h->count = count; h->order = order_word & ((1u << kTagShift) - 1u); }
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

__global__ __launch_bounds__(kDraftThreads) void draft_kernel(DraftArgs a)
{
    __shared__ int32_t tok[kMaxNodes];
    // recent[u][i]: the token i positions before the end of the sequence that ends at node u
    // (recent[u][0] is the node's own token), so a key is read without walking up the tree
    __shared__ __align__(16) int32_t recent[kMaxNodes][kMaxOrder];
    __shared__ int32_t t_first[kMaxNodes], t_nchild[kMaxNodes];
    __shared__ int32_t t_level[kMaxDepth + 3];
    __shared__ long long s_clen;
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int N = a.tree.N, K = a.K;
    for (int u = tid; u < N; u += kDraftThreads) {
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
        s_clen = len;
    }
    __syncthreads();
    const long long clen = (long long)readlane_u64((unsigned long long)s_clen, 0);
    const int NO = a.omax - a.omin + 1;
    for (int d = 0; d < a.tree.D; ++d) {
        // values read from shared memory that are the same in every lane go to scalar registers
        const int lo = __builtin_amdgcn_readfirstlane(t_level[d]), hi = __builtin_amdgcn_readfirstlane(t_level[d + 1]);
        // a level without a drafted node ends the tree (tok is stable here: barrier below)
        bool any = false;
        for (int u = lo + lane; u < hi; u += 64) any |= tok[u] >= 0;
        if (!__ballot(any)) break;  // the same in every wave
        for (int u = lo + wave; u < hi; u += kDraftThreads / 64) {
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
                home_fp = h->fp;
                home_cnt = h->count;
            }
            int32_t pid[kMaxOrder];
            float pmu[kMaxOrder];
#pragma unroll
            for (int q = 0; q < kMaxOrder; ++q) {
                pid[q] = -1; pmu[q] = 0.0f;
                const unsigned long long fq = readlane_u64(fp, q);  // uniform
                if (q < NO && fq && lane < K) {
                    pid[q] = slot_ids(a.table, fq & a.mask, a.slot_bytes)[lane];
                    pmu[q] = slot_mu(a.table, fq & a.mask, a.slot_bytes, K)[lane];
                }
            }
            long long hit_slot = -1;
            if (fp) {
                if (home_fp == fp) { if (home_cnt > 0) hit_slot = (long long)(fp & a.mask); }
                else if (home_fp != 0ull) {
                    for (int i = 1; i < a.max_probe; ++i) {  // displaced key: keep probing
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
                id = slot_ids(a.table, (uint64_t)slot, a.slot_bytes)[lane];
                mu = slot_mu(a.table, (uint64_t)slot, a.slot_bytes, K)[lane];
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
    for (int u = tid; u < N; u += kDraftThreads) {
        a.draft_tok[(size_t)b * N + u] = tok[u];
        if (a.out_tok) a.out_tok[(size_t)b * N + u] = tok[u];
    }
    if (a.recent_out)
        for (int i = tid; i < N * kMaxOrder; i += kDraftThreads)
            if (tok[i / kMaxOrder] >= 0) a.recent_out[(size_t)b * N * kMaxOrder + i] = recent[i / kMaxOrder][i % kMaxOrder];
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

// Attention mask and positions of the pending tree (paper Sec. 3.2: the tree is scored by the
// target model in one pass).  anc[u] is the set of ancestors-or-self of node u as a bit set of
// `words` 64-bit words.  One thread per (u, 8 consecutive v): eight mask bytes per store.
__global__ __launch_bounds__(256) void tree_packing_kernel(int B, int N, int words, const unsigned long long *anc,
                                                           const int32_t *depth, const int32_t *draft_tok,
                                                           const long long *ctx_len, uint8_t *mask, long long *pos)
{
    const int b = blockIdx.y;
    const int groups = (N + 7) / 8;                 // groups of 8 columns per row
    const int item = blockIdx.x * blockDim.x + threadIdx.x;
    if (item >= N * groups) return;
    const int u = item / groups, v0 = (item % groups) * 8;
    const bool drafted = draft_tok[(size_t)b * N + u] >= 0;
    const unsigned long long bits = drafted ? anc[(size_t)u * words + (v0 >> 6)] >> (v0 & 63) : 0ull;
    uint8_t *row = mask + ((size_t)b * N + u) * N;
    for (int q = 0; q < 8 && v0 + q < N; ++q) row[v0 + q] = (uint8_t)((bits >> q) & 1ull);
    if (v0 == 0) pos[(size_t)b * N + u] = drafted ? ctx_len[b] - 1 + depth[u] : -1;
}

// plain copy of 16-byte words: the known-size kernel against which HBM traffic counters are scaled
__global__ __launch_bounds__(256) void copy_words_kernel(const uint4 *src, uint4 *dst, size_t nwords)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < nwords; i += stride) dst[i] = src[i];
}

// Bare read of `rows` rows of `vpr` 16-byte words in the row pass's launch shape (one workgroup
// of 256 threads per row, two batches of two loads per thread in flight): what a kernel that only
// fetches the logits takes on this device.  Each wave leaves one word so the loads are not removed.
__global__ __launch_bounds__(256) void read_rows_kernel(const uint4 *src, size_t vpr, uint32_t *sink)
{
    const uint4 *r = src + (size_t)blockIdx.x * vpr;
    const size_t t = threadIdx.x, last = vpr - 1;
    constexpr int U = 2, PF = 2;
    const size_t per_batch = 256 * U;
    const size_t nbatch = (vpr + per_batch - 1) / per_batch;
    uint4 ring[PF][U];
    auto load = [&](uint4 (&w)[U], size_t k) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const size_t i = (k * U + u) * 256 + t;
            w[u] = load_streamed(r + (i < last ? i : last));
        }
    };
#pragma unroll
    for (int s = 0; s < PF; ++s) load(ring[s], s);
    uint32_t acc = 0;
    for (size_t k0 = 0; k0 < nbatch; k0 += PF) {
#pragma unroll
        for (int s = 0; s < PF; ++s) {
#pragma unroll
            for (int u = 0; u < U; ++u) acc += ring[s][u].x ^ ring[s][u].y ^ ring[s][u].z ^ ring[s][u].w;
            load(ring[s], k0 + s + PF);
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
    if ((threadIdx.x & 63) == 0) sink[(size_t)blockIdx.x * 4 + (threadIdx.x >> 6)] = acc;
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
