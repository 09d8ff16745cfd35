// row_pass.hpp -- row_pass_kernel: softmax statistics, top-K and node outcome of every logits row in one
// streaming pass (paper Sec. 4.1, 3.2).
#pragma once
#include "wave_ops.hpp"

namespace stand {

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
    // The exponent of a term is formed as fma(l, c, nb) with nb = -m_ref * c rounded to binary32.  That rounding
    // shifts EVERY exponent by the same dlt = (-m_ref * c) - nb (exact; a fused multiply-add recovers it), i.e.
    // the whole sum is off by the factor 2^dlt -- negligible for ordinary logits, 1e-4 for |m_ref| c in the
    // thousands (large logits at a low temperature).  The sum is kept in those shifted units and corrected where
    // the reference changes and at the end, in the rare path only.
    float dlt = 0.0f;

    auto raise_reference = [&](float cm) {
        // some lane saw a value above the reference: move the reference to the wave's maximum
        const float nm = uniform_f32(fmaxf(wave_max_f32(cm), m_ref));
        const float nb_new = -nm * c;
        const float dlt_new = __builtin_fmaf(-nm, c, -nb_new);
        s_t *= fast_exp2((m_ref - nm) * c + (dlt - dlt_new));
        m_ref = nm;
        nb = nb_new;
        dlt = dlt_new;
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

    // One vector: its maximum (returned; -inf for a lane without a vector) and its share of the fast sum.
    auto one_vector = [&](const uint4 &w, bool valid) {
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
        return cm;
    };
    // The candidate list is looked at once per batch, not once per vector: a wave sees only a few dozen
    // batches of a row, and early in the row nearly every vector has some lane at or above the threshold.
    // Each lane keeps the maxima of its vectors of the batch; if any of them reaches the threshold, the
    // vectors are offered in order (the threshold may rise between them).
    auto offer_batch = [&](const float (&cm)[U], const bool (&vld)[U], int kb) {
        bool any = false;
#pragma unroll
        for (int u = 0; u < U; ++u) any |= vld[u] && cm[u] >= st.theta_val;
        if (!__ballot(any)) return;
#pragma unroll
        for (int u = 0; u < U; ++u)
            wave_offer<LOWBIT>(ws, st, lane, K, vld[u] && cm[u] >= st.theta_val, cm[u], (uint32_t)((kb * U + u) * 64 + lane), m_ref);
    };
    auto do_batch = [&](uint4 (&w)[U], int k) {
        const int kb = k * wpr + wsub;        // batch of the row
        float cm[U];
        bool vld[U];
        if ((kb + 1) * per_batch <= g.nvec) {  // wave-uniform: every lane has all its vectors
#pragma unroll
            for (int u = 0; u < U; ++u) { vld[u] = true; cm[u] = one_vector(w[u], true); }
        } else {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                vld[u] = (kb * U + u) * 64 + lane < g.nvec;
                cm[u] = one_vector(vld[u] ? w[u] : make_uint4(0, 0, 0, 0), vld[u]);
            }
        }
        offer_batch(cm, vld, kb);
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
    out.s = s * fast_exp2(dlt);
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
// strided over `nthreads` threads; returns this thread's partial sum_v floor(E((l_v - m) c) * 2^(40 - shift)).
// floor(e 2^40) = hi 2^20 + lo, and hi 2^20 is a multiple of 2^shift (shift <= 20), so
// floor(e 2^(40 - shift)) = hi 2^(20 - shift) + (lo >> shift): the parts are shifted, then summed.
template <int DT, int INFLIGHT = 4, bool SHORT_FORM = true>
__device__ __forceinline__ unsigned long long thread_exact_partial(const void *rowp, const RowGeom &g, int v0, int v1,
                                                                   bool with_edge, float m, float c, int t, int nthreads,
                                                                   int shift)
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
            ahi += hi; alo += lo >> shift;
        }
    }
    // INFLIGHT independent loads are issued before any of them is used (indices clamped, so the
    // number of loads in flight does not depend on the position in the row)
    const int vlast = v1 > v0 ? v1 - 1 : v0;
    // A term below 2^-14 (nearly all of a row) needs no split: e * 2^40 < 2^26 is an integer-valued binary32 once
    // truncated, so floor(e * 2^40) is one multiplication and one conversion.  The wave takes the split form
    // for a vector in which any lane holds a larger term.  (y is clamped at -64 instead of tested: E(-64) = 2^-64
    // contributes 0 like the E = 0 of smaller y, and a NaN is clamped as well.)
    auto add_vec = [&](const uint4 &w, int idx) {
        if (idx < v1) {
            float x[EPV], e[EPV];
            unpack<DT>(w, x);
            float emax = 0.0f;
#pragma unroll
            for (int j = 0; j < EPV; ++j) {
                e[j] = exact_exp2_noguard(fmaxf(scaled_offset(x[j], m, c), -64.0f));
                emax = fmaxf(emax, e[j]);
            }
            if (SHORT_FORM && !__any(emax >= 0x1p-14f)) {
#pragma unroll
                for (int j = 0; j < EPV; ++j) alo += (uint32_t)(e[j] * 0x1p40f) >> shift;
            } else {
#pragma unroll
                for (int j = 0; j < EPV; ++j) {
                    uint32_t hi, lo;
                    fixed_split(e[j], hi, lo);
                    ahi += hi; alo += lo >> shift;
                }
            }
        }
    };
    for (int base = v0 + t; base < v1; base += INFLIGHT * nthreads) {
        uint4 w[INFLIGHT];
#pragma unroll
        for (int q = 0; q < INFLIGHT; ++q) {
            const int i = base + q * nthreads;
            w[q] = load_streamed(&g.vp[i < vlast ? i : vlast]);  // (read once more, then never: 0.5 % of a step against plain loads)
        }
#pragma unroll
        for (int q = 0; q < INFLIGHT; ++q) {
            add_vec(w[q], base + q * nthreads);
            if ((q & 3) == 3 || q == INFLIGHT - 1) {
                // at most 32 elements since the last flush: the 32-bit accumulators stay below 2^31 (terms
                // below 2^26 in the short form, below 2^20 and 2^21 in the split form)
                S += ((unsigned long long)ahi << (20 - shift)) + alo;
                ahi = 0; alo = 0;
            }
        }
    }
    return S + ((unsigned long long)ahi << (20 - shift)) + alo;
}

// Exact normaliser of a row by one wave (rare path).
template <int DT>
__device__ unsigned long long wave_row_exact_sum(const void *rowp, int V, float m, float c, int lane, int shift)
{
    const RowGeom g = row_geom<DT>(rowp, V);
    // (the split form only: this rare path shares its registers with the streaming loop of the same kernel)
    unsigned long long S = thread_exact_partial<DT, 4, false>(rowp, g, 0, g.nvec, true, m, c, lane, 64, shift);
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
    float eps;                  // relative error assumed for the fast normaliser from its additions (>= kFastEps)
    int fx_shift;               // the exact normaliser counts in units of 2^-(40 - fx_shift) (0 up to V = 2^22)
};

// Shared memory of one row's workgroup of WPR waves.
template <int WPR>
struct RowShared {
    WaveScan wsh[WPR];
    unsigned long long ebuf[kElemCap + 8];  // element keys offered to the row's final selection
    float part_m[WPR], part_s[WPR];
    int part_cnt[WPR];
};

// One logits row by the WPR waves of the calling workgroup (all of its 64 * WPR threads call this).
// With pub.row set, the testing wave and the ranking wave also publish what the tail of the same launch
// reads (maximum and outcome; top-K ids and logits) as self-validating words (RowPub).
template <int DT, int WPR>
__device__ __forceinline__ void row_role(const RowPassArgs &a, int row, RowShared<WPR> *sm, const RowPub &pub)
{
    constexpr int ES = VecTraits<DT>::ES;
    // the wave's number is the same in all its lanes: say so, so that everything derived from it
    // (its share of the row, the loop over its batches) is kept in scalar registers
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    WaveScan *ws = &sm->wsh[wave];
    const int b = row / a.N, u = row % a.N;
    const char *rowp = (const char *)a.logits + (size_t)row * (size_t)a.V * ES;
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
    auto node_tests = [&](float m, float s) -> int {
        if (nch == 0) {  // uniform over the wave
            if (lane == 0) a.outcome[row] = -1;
            return -1;
        }
        const float e = (lane < a.K && my_id >= 0) ? exact_exp2(scaled_offset(my_l, m, a.c)) : 0.0f;
        // Relative error assumed for s: the part that grows with the terms a lane adds (a.eps, from the host);
        // the offset every exponent shares is corrected in the streaming loop, what is left of it (the
        // rounding of each term's own argument, relative to that argument, and of the waves' combination)
        // is covered by a term in |m| c that stays far below a.eps for ordinary inputs.
        const float eps_row = a.eps + 1e-9f * fabsf(m) * a.c;
        NodeResult nr = wave_node_outcome(lane, a.K, my_id, my_mu, e / s, nch, ch, a.seed, (uint32_t)b, a.step, fc,
                                          true, eps_row, a.onehot);
        if (nr.near) {
            // a test fell inside the error bound of the fast normaliser: decide with the exact one
            const unsigned long long S = wave_row_exact_sum<DT>(rowp, a.V, m, a.c, lane, a.fx_shift);
            const float sx = normaliser_from_fixed(S, a.fx_shift);
            nr = wave_node_outcome(lane, a.K, my_id, my_mu, e / sx, nch, ch, a.seed, (uint32_t)b, a.step, fc, false,
                                   0.0f, a.onehot);
            if (lane == 0) atomicAdd(&a.stats[kStatNear], 1ull);
        }
        if (lane == 0) a.outcome[row] = (int32_t)nr.accepted;
        return nr.accepted;
    };
    // Wave 0 ranks the row at its end, wave 1 runs the accept tests meanwhile.
    static_assert(WPR >= 2, "a row is shared by at least two waves");
    constexpr int kTestWave = 1;
    {
        const WavePartial wp = wave_row_stream<DT>(rowp, a.V, a.c, a.K, ws, lane, wave, WPR);
        if (lane == 0) { sm->part_m[wave] = wp.m_ref; sm->part_s[wave] = wp.s; sm->part_cnt[wave] = wp.cnt; }
        if (wave == kTestWave) request_proposal();
    }
    __syncthreads();
    // both finishing waves form the row's maximum and normaliser with the same expressions, so
    // they hold the same m and s (the ranking's maximum, top[0], has no negative zero either)
    m = sm->part_m[0];
    for (int q = 1; q < WPR; ++q) m = fmaxf(m, sm->part_m[q]);
    m = m + 0.0f;
    s = 0.0f;
    for (int q = 0; q < WPR; ++q) s += sm->part_s[q] * fast_exp2((sm->part_m[q] - m) * a.c);
    if (wave == kTestWave) {
        // the accept tests need the row's maximum and normaliser, not its ranking
        request_proposal_logits();
        const int oc = node_tests(m, s);
        if (pub.row && lane == 0) st_agent(&pub.row[row], pack_row_pub(m, oc, pub.tag));
        return;
    }
    if (wave != 0) return;
    // gather the partner waves' records behind this wave's own (each list holds at most
    // K + kPruneSlack ranking keys); with many partners the list is cut down on the way
    int cnt = sm->part_cnt[0];
    for (int q = 1; q < WPR; ++q) {
        const int cq = sm->part_cnt[q];
        if (cnt + cq > kWavePrune) {
            WaveScanState gs;
            gs.cnt = cnt;
            set_theta(gs, 0ull);
            __builtin_amdgcn_wave_barrier();
            wave_prune_fast<false, true, DT == kDtBf16 ? 16 : 0>(ws, gs, lane, a.K, 0u, ~0u);
            cnt = gs.cnt;
        }
        if (lane < cq) ws->buf[cnt + lane] = sm->wsh[q].buf[lane];
        cnt += cq;
    }
    __builtin_amdgcn_wave_barrier();
    wave_row_finish<DT>(rowp, a.V, a.K, ws, sm->ebuf, lane, cnt);

    if (lane < a.K) {
        const unsigned long long key = ws->top[lane];
        const float l = rank_key_value(key);
        a.top_idx[(size_t)row * a.K + lane] = (int32_t)rank_key_id(key);
        a.top_l[(size_t)row * a.K + lane] = l;
        a.top_p[(size_t)row * a.K + lane] = exact_exp2(scaled_offset(l, m, a.c)) / s;
        if (pub.top) st_agent(&pub.top[(size_t)row * a.K + lane], pack_top_pub((int32_t)rank_key_id(key), l, pub.tag));
    }
    if (lane == 0) { a.row_m[row] = m; a.row_s[row] = s; }
}

template <int DT, int WPR>
__global__ __launch_bounds__(64 * WPR) void row_pass_kernel(RowPassArgs a)
{
    __shared__ RowShared<WPR> sm;
    // Workgroups are numbered node-major (all trajectories' rows of node 0, then of node 1, ...).
    // The nodes near the root carry drafted children, whose accept tests make the end of their
    // row the longest; started first, those ends overlap with the streaming of later rows, and the
    // rows that finish the kernel are leaves.
    const int slot = blockIdx.x;
    if (slot >= a.B * a.N) return;
    row_role<DT, WPR>(a, (slot % a.B) * a.N + slot / a.B, &sm, RowPub{nullptr, nullptr, 0u});
}

}  // namespace stand
