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
constexpr int kRowThreads = 256;
constexpr int kMaxNodes = 256;
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
// Sum of the values of lanes 0..K-1 in lane order (one rounding per addition), the same in
// every lane.  Lanes K..31 must hold +0, which leaves the sum unchanged.
__device__ __forceinline__ float wave_ordered_sum(float x)
{
    float t = 0.0f;
#pragma unroll
    for (int i = 0; i < kMaxK; ++i) t = t + u2f((uint32_t)__builtin_amdgcn_readlane((int)f2u(x), i));
    return t;
}

// 64-bit key of lane i (i uniform)
__device__ __forceinline__ unsigned long long readlane_u64(unsigned long long v, int i)
{
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, i);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), i);
    return ((unsigned long long)hi << 32) | lo;
}

struct NodeResult { int accepted; int rounds; bool near; float r; float rho; };

__device__ __forceinline__ NodeResult wave_node_outcome(int lane, int K, int32_t my_id, float my_mu, float my_p, int nchild,
                                        const int32_t *child_tok, uint64_t seed, uint32_t b, uint64_t step,
                                        int first_child, bool track_err, float eps)
{
    NodeResult res;
    res.accepted = -1; res.rounds = 0; res.near = false;
    const bool act = lane < K;
    float w = (act && my_mu > 0.0f) ? my_mu : 0.0f;
    float zw = wave_ordered_sum(w);
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
        const float mn = act ? (r < w ? r : w) : 0.0f;
        const float M = wave_ordered_sum(mn);
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
        const float zw2 = wave_ordered_sum(w);
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
    // accumulators of the path pass, cleared here for the kernels that follow
    int W;
    unsigned long long *rowS, *race;
    unsigned int *done;
};

template <int DT>
__global__ __launch_bounds__(kRowThreads) void row_pass_kernel(RowPassArgs a)
{
    if (blockIdx.x == 0) {
        for (int i = threadIdx.x; i < a.B * a.W; i += kRowThreads) { a.rowS[i] = 0ull; a.done[i] = 0u; }
        for (int i = threadIdx.x; i < a.B; i += kRowThreads) a.done[a.B * a.W + i] = 0u;
    }
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
    const int fc = a.tree.first_child[u];
    const int nch = a.draft_has[row];  // children drafted from this node's table entry (0: none)
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
                                      true, kFastEps);
    if (nr.near) {
        // a test fell inside the error bound of the fast normaliser: decide with the exact one
        const unsigned long long S = wave_row_exact_sum<DT>(rowp, a.V, m, a.c, lane);
        const float sx = normaliser_from_fixed(S);
        nr = wave_node_outcome(lane, a.K, my_id, my_mu, e / sx, nch, child_tok, a.seed, (uint32_t)b, a.step, fc, false,
                               0.0f);
        if (lane == 0) atomicAdd(&a.stats[kStatNear], 1ull);
    }
    if (lane == 0) a.outcome[row] = nr.accepted;
}

// ---------------------------------------------------------------------------------------------
// Path pass.  The accepted path of trajectory b follows `outcome` from the root (verify), or is
// given as commit rows (update).  For each path row the exact normaliser is needed (its
// observation is stored in the table), for the last one also the resampled token.  The work is
// cut into segments so that it spreads over all compute units:
//   path_exact_kernel  block (seg, j, b): exact partial sum of a segment of path row j; the last
//                      block of a trajectory to finish writes the observations of its path rows
//                      and the residual state of its stop node
//   race_kernel        block (seg, b): exponential race over a segment of the stop row; the last
//                      block of a trajectory writes the winner
// ---------------------------------------------------------------------------------------------
struct PathArgs {
    const void *logits;
    int B, N, V, K, W, mode;   // mode 0: verify (path from outcome), 1: update (rows given)
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
    unsigned long long *rowS;  // [B][W] exact fixed-point sums, zero on entry of path_exact_kernel
    unsigned long long *race;  // [B][kRaceSlots] best (time, token) of each race block
    unsigned int *done;        // [B*W] finished blocks per path row, then [B] finished race blocks; zero on entry
    int32_t *obs_idx;          // [B][W][K]
    float *obs_p;              // [B][W][K]
    // residual state of the stop node: written by path_exact_kernel, read by race_kernel
    int32_t *res_id;           // [B][K] stored ids of the stop node's proposal
    float *res_r;              // [B][K] residual target on them
    float *res_f;              // [B][4] rho, s, m of the stop row
    int32_t *res_i;            // [B][4] number of stored ids (0: no proposal), stop node, path length
    unsigned long long *stats;
};

// Walks the accepted path of trajectory b and leaves it in path[0..len) (shared memory).  The
// outcomes of the trajectory's nodes are staged in shared memory first, so the walk itself
// does not wait on global memory.  Must be called by the whole workgroup; returns len.
__device__ __forceinline__ int resolve_path(const PathArgs &a, int b, int *path, int *oc /* [kMaxNodes] shared */,
                                            int *len_sh)
{
    for (int u = threadIdx.x; u < a.N; u += blockDim.x) oc[u] = a.outcome[(size_t)b * a.N + u];
    __syncthreads();
    if (threadIdx.x == 0) {
        int cur = 0, len = 0;
        for (;;) {
            path[len++] = cur;
            const int acc = oc[cur];
            if (acc < 0 || len > a.tree.D) break;
            cur = a.tree.first_child[cur] + acc;
        }
        *len_sh = len;
    }
    __syncthreads();
    return *len_sh;
}

__device__ __forceinline__ int path_row_of(const PathArgs &a, int b, int j, const int *path, int len)
{
    // returns the tree node of path position j, or -1 if there is none
    if (a.mode == 0) return j < len ? path[j] : -1;
    int cl = a.commit_len[b];
    cl = cl < 0 ? 0 : (cl > a.W ? a.W : cl);
    if (j >= cl) return -1;
    const int node = a.commit_row[(size_t)b * a.W + j];
    return (node < 0 || node >= a.N) ? -1 : node;
}

template <int DT>
__global__ __launch_bounds__(kPathThreads) void path_exact_kernel(PathArgs a)
{
    constexpr int ES = VecTraits<DT>::ES;
    __shared__ int path[32];
    __shared__ int oc[kMaxNodes];
    __shared__ int s_len, s_last;
    __shared__ unsigned long long s_part[kPathThreads / 64];
    const int seg = blockIdx.x, nseg = gridDim.x, j = blockIdx.y, b = blockIdx.z, tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int len = a.mode == 0 ? resolve_path(a, b, path, oc, &s_len) : 0;
    if (a.mode == 0 && seg == 0 && j == 0) {
        // accepted tokens are the tokens of the path nodes after the root; the last emitted
        // token (position len - 1) is written by race_kernel
        if (tid < a.W) {
            a.out_node[(size_t)b * a.W + tid] = tid < len ? path[tid] : -1;
            if (tid + 1 < len) a.out_tok[(size_t)b * a.W + tid] = a.draft_tok[(size_t)b * a.N + path[tid + 1]];
            else if (tid >= len) a.out_tok[(size_t)b * a.W + tid] = -1;
        }
        if (tid == 0) { a.out_len[b] = len; atomicAdd(&a.stats[kStatTokens], (unsigned long long)len); }
    }
    {
        const int node = path_row_of(a, b, j, path, len);
        if (node >= 0) {
            const int row = b * a.N + node;
            const char *rowp = (const char *)a.logits + (size_t)row * (size_t)a.V * ES;
            const float m = a.src_m[a.mode == 0 ? row : b * a.W + j];
            const RowGeom g = row_geom<DT>(rowp, a.V);
            const int per = (g.nvec + nseg - 1) / nseg;
            const int v0 = seg * per, v1 = (v0 + per < g.nvec) ? v0 + per : g.nvec;
            unsigned long long S = thread_exact_partial<DT>(rowp, g, v0, v1, seg == 0, m, a.c, tid, kPathThreads);
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) S += __shfl_xor(S, off);
            if (lane == 0) s_part[wave] = S;
        }
    }
    // ---- the last block of this row to get here finishes the row.  Everything that crosses
    // blocks (row sum, ticket) goes through device-scope atomics, one per block and address, so
    // no cache flush is needed and few atomics queue up on one address.
    __syncthreads();
    const int my_node = path_row_of(a, b, j, path, len);
    if (my_node < 0) return;  // block-uniform: no such path row
    if (tid == 0) {
        unsigned long long S = 0ull;
        for (int q = 0; q < kPathThreads / 64; ++q) S += s_part[q];
        // the returned value makes the thread wait until the addition has been performed
        const unsigned long long old = atomicAdd(&a.rowS[(size_t)b * a.W + j], S);
        asm volatile("" : : "v"((uint32_t)old));
        const unsigned int ticket = atomicAdd(&a.done[(size_t)b * a.W + j], 1u);
        s_last = ticket == (unsigned int)nseg - 1u;
    }
    __syncthreads();
    if (!s_last || wave != 0) return;

    // observation of this row (paper Sec. 4.1: top-k ids and probabilities)
    {
        const int src = a.mode == 0 ? b * a.N + my_node : b * a.W + j;
        const float m = a.src_m[src];
        const float s = normaliser_from_fixed(atomicAdd(&a.rowS[(size_t)b * a.W + j], 0ull));
        if (lane < a.K) {
            a.obs_idx[((size_t)b * a.W + j) * a.K + lane] = a.src_top_idx[(size_t)src * a.K + lane];
            a.obs_p[((size_t)b * a.W + j) * a.K + lane] =
                exact_exp2(scaled_offset(a.src_top_l[(size_t)src * a.K + lane], m, a.c)) / s;
        }
    }
    if (a.mode != 0 || j != len - 1) return;

    // residual state at the stop node: replay its accept sequence with exact probabilities
    const int node = path[len - 1];
    const int row = b * a.N + node;
    const char *rowp = (const char *)a.logits + (size_t)row * (size_t)a.V * ES;
    const float m = a.src_m[row];
    const float s = normaliser_from_fixed(atomicAdd(&a.rowS[(size_t)b * a.W + (len - 1)], 0ull));
    const int fc = a.tree.first_child[node];
    const int nch = a.draft_has[row];
    float rho = 1.0f;
    if (nch > 0) {
        int32_t my_id = -1;
        float my_mu = 0.0f, my_p = 0.0f;
        if (lane < a.K) {
            my_id = a.draft_qid[(size_t)row * a.K + lane];
            my_mu = a.draft_qmu[(size_t)row * a.K + lane];
            if ((uint32_t)my_id >= (uint32_t)a.V) { my_id = -1; my_mu = 0.0f; }
            else my_p = exact_exp2(scaled_offset(load_scalar<DT>(rowp, my_id), m, a.c)) / s;
        }
        NodeResult nr = wave_node_outcome(lane, a.K, my_id, my_mu, my_p, nch, a.draft_tok + (size_t)b * a.N + fc, a.seed,
                                          (uint32_t)b, a.step, fc, false, 0.0f);
        if (lane < a.K) { a.res_id[(size_t)b * a.K + lane] = my_id; a.res_r[(size_t)b * a.K + lane] = nr.r; }
        rho = nr.rho;
        if (lane == 0 && nr.accepted != -1) atomicAdd(&a.stats[kStatMismatch], 1ull);  // the stop node rejects all
    }
    if (lane == 0) {
        a.res_f[(size_t)b * 4 + 0] = rho; a.res_f[(size_t)b * 4 + 1] = s; a.res_f[(size_t)b * 4 + 2] = m;
        a.res_i[(size_t)b * 4 + 0] = nch > 0 ? a.K : 0; a.res_i[(size_t)b * 4 + 1] = node; a.res_i[(size_t)b * 4 + 2] = len;
        // accept tests along the path: rank + 1 at every accepted node, all children at the stop node
        unsigned long long tests = (unsigned long long)nch;
        for (int q = 0; q + 1 < len; ++q) tests += (unsigned long long)(oc[path[q]] + 1);
        atomicAdd(&a.stats[kStatTests], tests);
    }
}

// Fast approximations used only to rank tokens and to skip those that provably cannot win the
// race; every token that may win is evaluated with the exact functions.
__device__ __forceinline__ float fast_exp_time(float U)
{
    // -ln U: series in d = 1 - U (exact) close to 1, hardware log2 elsewhere
    const float d = 1.0f - U;
    const float ser = d * __builtin_fmaf(d, __builtin_fmaf(d, 0.33333334f, 0.5f), 1.0f);
    const float lg = -0.6931472f * __builtin_amdgcn_logf(U);
    return d < 0.0078125f ? ser : lg;
}
constexpr int kRaceSlots = 64;         // most race blocks per trajectory
constexpr int kRaceVecs = 2;           // vectors per thread and round
constexpr float kRaceMargin = 1.001f;  // the fast time is within 1e-4 relative of the exact one

struct RaceShared {
    int32_t sup_id[kMaxK];
    float sup_r[kMaxK];
    unsigned long long best;      // best exact key of the block
    unsigned long long sup_mask;  // bit (vector index & 63) set if the vector may hold a stored id
    int last;
};

// Exact finishing time of token v as a key (time bits, token); all ones if the token has no
// residual mass.  Kept out of line: it runs for one or two tokens per thread only.
__device__ __noinline__ unsigned long long race_exact_key(float l, uint32_t v, uint32_t uword, float m, float c, float s,
                                                           float rho, const int32_t *sup_id, const float *sup_r, int nsup)
{
    float r = (exact_exp2(scaled_offset(l, m, c)) / s) * rho;
    for (int q = 0; q < nsup; ++q) if (sup_id[q] == (int32_t)v) r = sup_r[q];
    if (!(r > 0.0f)) return ~0ull;
    const float xv = -exact_log(word_to_uniform(uword));
    const float t = xv / r;
    return ((unsigned long long)f2u(t) << 32) | (unsigned long long)v;
}

template <int DT>
__global__ __launch_bounds__(kPathThreads) void race_kernel(PathArgs a)
{
    // Resample at the stop node (paper Sec. 3.2, "resampled from an adjusted distribution"):
    // token v finishes at -ln(U_v) / r(v), r = residual target; the earliest wins, ties to the
    // lowest id.
    //
    // Per round every thread estimates the finishing times of its tokens with the hardware
    // exp2 / log2 / rcp, evaluates its own front-runner exactly, and the block's best exact time
    // then bounds the winner: only tokens whose estimate is within the margin of that bound are
    // evaluated exactly as well.  Tokens stored in the node's proposal (their residual differs
    // from p * rho) are always evaluated exactly.
    constexpr int ES = VecTraits<DT>::ES, EPV = VecTraits<DT>::EPV, BS = kPathThreads, NV = kRaceVecs;
    __shared__ RaceShared rs;
    const int seg = blockIdx.x, nseg = gridDim.x, b = blockIdx.y, tid = threadIdx.x, lane = tid & 63;
    const int nsup = a.res_i[(size_t)b * 4 + 0], node = a.res_i[(size_t)b * 4 + 1], len = a.res_i[(size_t)b * 4 + 2];
    const float rho = a.res_f[(size_t)b * 4 + 0], s = a.res_f[(size_t)b * 4 + 1], m = a.res_f[(size_t)b * 4 + 2];
    const int row = b * a.N + node;
    const char *rowp = (const char *)a.logits + (size_t)row * (size_t)a.V * ES;
    const RowGeom g = row_geom<DT>(rowp, a.V);
    if (tid == 0) { rs.best = (0x7F800000ull << 32) | 0xFFFFFFFFull; rs.sup_mask = 0ull; }  // time = +inf
    __syncthreads();
    if (tid < nsup) {
        const int32_t id = a.res_id[(size_t)b * a.K + tid];
        rs.sup_id[tid] = id;
        rs.sup_r[tid] = a.res_r[(size_t)b * a.K + tid];
        if (id >= g.head) atomicOr(&rs.sup_mask, 1ull << (((id - g.head) / EPV) & 63));
    }
    __syncthreads();
    const unsigned long long sup_mask = rs.sup_mask;
    const float scale_fast = rho / s;
    unsigned long long best = ~0ull;

    auto exact_token = [&](float l, uint32_t v, uint32_t uword, bool near_support) {
        const unsigned long long key = race_exact_key(l, v, uword, m, a.c, s, rho, rs.sup_id, rs.sup_r, near_support ? nsup : 0);
        if (key < best) best = key;
    };
    // the scalar edge elements and the stored ids: exact, by the first block
    if (seg == 0) {
        int edge_id = -1;
        if (tid < g.head) edge_id = tid;
        else if (tid < g.head + g.ntail) edge_id = g.tail0 + (tid - g.head);
        if (edge_id >= 0) {
            const Philox4 ph = philox_group(a.seed, (uint32_t)b, a.step, (uint32_t)node, (uint32_t)edge_id >> 2, kStreamBonus);
            exact_token(load_scalar<DT>(rowp, edge_id), (uint32_t)edge_id, philox_word(ph, (uint32_t)edge_id & 3u), true);
        }
        if (tid >= 64 && tid < 64 + nsup) {
            const uint32_t v = (uint32_t)rs.sup_id[tid - 64];
            if (v < (uint32_t)a.V) {
                const Philox4 ph = philox_group(a.seed, (uint32_t)b, a.step, (uint32_t)node, v >> 2, kStreamBonus);
                exact_token(load_scalar<DT>(rowp, (int)v), v, philox_word(ph, v & 3u), true);
            }
        }
    }

    const int per = (g.nvec + nseg - 1) / nseg;
    const int v0 = seg * per, v1 = (v0 + per < g.nvec) ? v0 + per : g.nvec;
    const int vlast = v1 > v0 ? v1 - 1 : v0;
    const int nrounds = (v1 - v0 + NV * BS - 1) / (NV * BS);  // block-uniform
    for (int round = 0; round < nrounds; ++round) {
        // ---- estimates of all tokens of this thread's vectors (kept in registers)
        float tf[NV][EPV];
        uint4 w[NV];
        int vidx[NV];
        unsigned long long front = ~0ull;  // (estimate, token) of the thread's front-runner
#pragma unroll
        for (int u = 0; u < NV; ++u) {
            vidx[u] = v0 + (round * NV + u) * BS + tid;
            w[u] = g.vp[vidx[u] < vlast ? vidx[u] : vlast];
        }
#pragma unroll
        for (int u = 0; u < NV; ++u) {
            const bool valid = vidx[u] < v1;
            float x[EPV];
            unpack<DT>(w[u], x);
            const uint32_t id0 = (uint32_t)(g.head + vidx[u] * EPV);
            Philox4 ph = philox_group(a.seed, (uint32_t)b, a.step, (uint32_t)node, id0 >> 2, kStreamBonus);
#pragma unroll
            for (int q = 0; q < EPV; ++q) {
                const uint32_t v = id0 + q;
                if (q > 0 && (v & 3u) == 0u) ph = philox_group(a.seed, (uint32_t)b, a.step, (uint32_t)node, v >> 2, kStreamBonus);
                const float rf = fast_exp2(scaled_offset(x[q], m, a.c)) * scale_fast;
                const float t = fast_exp_time(word_to_uniform(philox_word(ph, v & 3u))) * __builtin_amdgcn_rcpf(rf);
                tf[u][q] = valid ? t : __builtin_inff();
                const unsigned long long k = ((unsigned long long)f2u(tf[u][q]) << 32) | v;
                front = k < front ? k : front;
            }
        }
        // ---- the front-runner, exactly (stored ids were handled above and are skipped here)
        const uint32_t fv = (uint32_t)front;
        if ((uint32_t)(front >> 32) < 0x7F800000u) {
            const int fvec = ((int)fv - g.head) / EPV;
            const bool in_sup = (sup_mask >> (fvec & 63)) & 1ull;
            bool is_sup = false;
            if (in_sup) for (int q = 0; q < nsup; ++q) is_sup |= rs.sup_id[q] == (int32_t)fv;
            if (!is_sup) {
                const Philox4 ph = philox_group(a.seed, (uint32_t)b, a.step, (uint32_t)node, fv >> 2, kStreamBonus);
                exact_token(load_scalar<DT>(rowp, (int)fv), fv, philox_word(ph, fv & 3u), false);
            }
        }
        atomicMin(&rs.best, best);
        __syncthreads();
        // ---- every other token whose estimate is not clearly behind the best exact time
        const float bound = u2f((uint32_t)(rs.best >> 32)) * kRaceMargin;
#pragma unroll
        for (int u = 0; u < NV; ++u) {
            const uint32_t id0 = (uint32_t)(g.head + vidx[u] * EPV);
            const bool in_sup = (sup_mask >> (vidx[u] & 63)) & 1ull;
#pragma unroll
            for (int q = 0; q < EPV; ++q) {
                const uint32_t v = id0 + q;
                if (vidx[u] < v1 && !(tf[u][q] > bound) && v != fv) {
                    bool is_sup = false;
                    if (in_sup) for (int z = 0; z < nsup; ++z) is_sup |= rs.sup_id[z] == (int32_t)v;
                    if (!is_sup) {
                        const Philox4 ph = philox_group(a.seed, (uint32_t)b, a.step, (uint32_t)node, v >> 2, kStreamBonus);
                        exact_token(load_scalar<DT>(rowp, (int)v), v, philox_word(ph, v & 3u), false);
                    }
                }
            }
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        unsigned long long o = __shfl_xor(best, off);
        best = o < best ? o : best;
    }
    if (lane == 0) atomicMin(&rs.best, best);
    __syncthreads();
    // Each block publishes its best key in a slot of its own (no two blocks queue on one address);
    // the last block of the trajectory to arrive reduces the slots.  All of it goes through
    // device-scope atomics, so no cache flush is needed.
    if (tid == 0) {
        const unsigned long long old = atomicExch(&a.race[(size_t)b * kRaceSlots + seg], rs.best);  // returned: performed
        asm volatile("" : : "v"((uint32_t)old));
        const unsigned int ticket = atomicAdd(&a.done[(size_t)a.B * a.W + b], 1u);
        rs.last = ticket == (unsigned int)nseg - 1u;
    }
    __syncthreads();
    if (!rs.last || tid >= 64) return;
    unsigned long long win = ~0ull;
    for (int q = lane; q < nseg; q += 64) {
        const unsigned long long o = atomicAdd(&a.race[(size_t)b * kRaceSlots + q], 0ull);
        win = o < win ? o : win;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        unsigned long long o = __shfl_xor(win, off);
        win = o < win ? o : win;
    }
    if (lane == 0) a.out_tok[(size_t)b * a.W + (len - 1)] = (int32_t)(uint32_t)win;
}

// Update mode: maximum and top-K of the given commit rows (one workgroup of 4 waves per row).
struct CommitScanArgs {
    const void *logits;
    int B, N, V, K, W;
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
    __shared__ int part_cnt[4];
    const int j = blockIdx.x, b = blockIdx.y, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int cl = a.commit_len[b];
    cl = cl < 0 ? 0 : (cl > a.W ? a.W : cl);
    if (j >= cl) return;
    const int node = a.commit_row[(size_t)b * a.W + j];
    if (node < 0 || node >= a.N) return;
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
    wave_row_finish<DT>(rowp, a.V, a.K, ws, lane, cnt);
    const size_t src = (size_t)b * a.W + j;
    if (lane < a.K) {
        a.pr_top_idx[src * a.K + lane] = (int32_t)rank_key_id(ws->top[lane]);
        a.pr_top_l[src * a.K + lane] = rank_key_value(ws->top[lane]);
    }
    if (lane == 0) a.pr_m[src] = rank_key_value(ws->top[0]);
}

// clears the accumulators of the path pass
__global__ void path_reset_kernel(int B, int W, unsigned long long *rowS, unsigned long long *race, unsigned int *done)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < B * W) { rowS[i] = 0ull; done[i] = 0u; }
    if (i < B) done[B * W + i] = 0u;
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
#pragma unroll
                for (int q = 0; q < kMaxK; ++q) {
                    const int32_t sid = __builtin_amdgcn_readlane(e_id, q);
                    const int32_t oid = __builtin_amdgcn_readlane(o_id, 32 + q);
                    const float op = u2f((uint32_t)__builtin_amdgcn_readlane((int)f2u(o_p), 32 + q));
                    if (q < K && lane < 32 && act && oid == id) other = op;
                    if (q < K && lane >= 32 && act && sid == id) dup = true;
                }
                float val;
                if (lane < 32) { float t = cf * e_mu; t = t + other; val = t / denom; }
                else { float t = cf * 0.0f; t = t + o_p; val = t / denom; act = act && !dup; }
                const unsigned long long key = act ? rank_key(val, (uint32_t)id) : 0ull;
                int rank = 0;
#pragma unroll
                for (int q = 0; q < 64; ++q) rank += readlane_u64(key, q) > key ? 1 : 0;
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
};

constexpr int kDraftThreads = 256;

__global__ __launch_bounds__(kDraftThreads) void draft_kernel(DraftArgs a)
{
    __shared__ int32_t tok[kMaxNodes];
    __shared__ int32_t tail[kMaxOrder];
    __shared__ long long s_clen;
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int N = a.tree.N, K = a.K;
    if (tid == 0) {
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
        for (int i = 0; i < kMaxOrder; ++i) tail[i] = t[i];
        s_clen = len;
    }
    for (int u = tid; u < N; u += kDraftThreads) {
        tok[u] = -1;
        a.draft_has[(size_t)b * N + u] = 0;
    }
    __syncthreads();
    const long long clen = s_clen;
    if (tid == 0 && clen > 0) tok[0] = tail[kMaxOrder - 1];
    __syncthreads();
    const int NO = a.omax - a.omin + 1;
    for (int d = 0; d < a.tree.D; ++d) {
        const int lo = a.tree.level_start[d], hi = a.tree.level_start[d + 1];
        for (int u = lo + wave; u < hi; u += kDraftThreads / 64) {
            const int nch = a.tree.nchild[u];
            if (nch == 0 || tok[u] < 0) continue;  // uniform per wave
            // ---- multi-level lookup (paper Sec. 4.2): lane q < NO takes order n = omax - q.
            // The home slot of every order is read together with its payload in one round
            // trip; only a key that was displaced by linear probing needs further probes.
            unsigned long long fp = 0ull;
            if (lane < NO) {
                const int n = a.omax - lane;
                if (clen + d >= n) {
                    int32_t key[kMaxOrder];
                    int x = u;
                    for (int i = n - 1; i >= 0; --i) {
                        const int back = n - 1 - i;  // tokens back from the node itself
                        if (back < d) { key[i] = tok[x]; x = a.tree.parent[x]; }
                        else key[i] = tail[kMaxOrder - 1 - (back - d)];
                    }
                    fp = fingerprint(n, key);
                }
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
            const long long slot = __shfl(hit_slot, win);
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
            // ---- Gumbel-Top-K: score = ln mu - ln(-ln U); children get the largest scores in order
            const bool cand = lane < K && mu > 0.0f;
            unsigned long long key = 0ull;
            if (cand) {
                const float U = uniform(a.seed, (uint32_t)b, a.step, (uint32_t)u, (uint32_t)id, kStreamDraft);
                const float g = exact_log(-exact_log(U));
                key = rank_key(exact_log(mu) - g, (uint32_t)id);
            }
            int rank = 0;
#pragma unroll
            for (int q = 0; q < kMaxK; ++q) rank += readlane_u64(key, q) > key ? 1 : 0;
            if (cand && rank < nch) tok[a.tree.first_child[u] + rank] = id;
            const int ncand = __popcll(__ballot(cand));
            if (lane == 0) a.draft_has[(size_t)b * N + u] = ncand < nch ? ncand : nch;
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
