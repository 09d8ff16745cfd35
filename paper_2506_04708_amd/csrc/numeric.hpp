// numeric.hpp -- device-side arithmetic of the STAND speculation step (gfx950).
//
// Every function here is a fixed sequence of correctly rounded binary32 operations, so that
// probabilities, scores and decisions do not depend on launch shape or lane order.  The file
// is compiled with -ffp-contract=off; the only fused operations are the explicit fmaf calls.
//
// Paper: arxiv 2506.04708 -- Sec. 4.1 (temperature softmax rows, top-k storage),
// Sec. 4.2 (Gumbel-Top-K: phi - log(-log U)), Sec. 3.2 (accept with min(1, p/q)).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace stand {

constexpr int kMaxK = 32;
constexpr int kMaxOrder = 8;
constexpr uint32_t kStreamDraft = 0u, kStreamAccept = 1u, kStreamBonus = 2u;

__device__ __forceinline__ float u2f(uint32_t u) { return __uint_as_float(u); }
__device__ __forceinline__ uint32_t f2u(float f) { return __float_as_uint(f); }

// ---- counter-based uniforms: Philox4x32, 10 rounds (Salmon et al., SC'11) ----------------------
struct Philox4 { uint32_t x, y, z, w; };

__device__ __forceinline__ Philox4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint64_t seed)
{
    uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return Philox4{c0, c1, c2, c3};
}

// counter = (token >> 2, node | stream << 24, step low word, b | step high word << 20)
__device__ __forceinline__ Philox4 philox_group(uint64_t seed, uint32_t b, uint64_t step, uint32_t node,
                                                uint32_t token_group, uint32_t stream)
{
    return philox4x32_10(token_group, node | (stream << 24), (uint32_t)step, b | ((uint32_t)(step >> 32) << 20), seed);
}

// U = (2 * (x >> 9) + 1) * 2^-24: odd 24-bit integer, exact, strictly inside (0, 1)
__device__ __forceinline__ float word_to_uniform(uint32_t x) { return (float)(2u * (x >> 9) + 1u) * 0x1p-24f; }

__device__ __forceinline__ uint32_t philox_word(const Philox4 &p, uint32_t i)
{
    return i == 0 ? p.x : (i == 1 ? p.y : (i == 2 ? p.z : p.w));
}

__device__ __forceinline__ float uniform(uint64_t seed, uint32_t b, uint64_t step, uint32_t node, uint32_t token, uint32_t stream)
{
    Philox4 p = philox_group(seed, b, step, node, token >> 2, stream);
    return word_to_uniform(philox_word(p, token & 3u));
}

// ---- 2^y for y <= ~0: 0 below -64, else 2^k * (1 + f Q(f)) with k = rint(y), f = y - k ----------
__device__ __forceinline__ float exact_exp2(float y)
{
    if (!(y >= -64.0f)) return 0.0f;
    float k = __builtin_rintf(y);
    float f = y - k;
    float q = 0x1.44138ap-13f;
    q = __builtin_fmaf(q, f, 0x1.5f0890p-10f);
    q = __builtin_fmaf(q, f, 0x1.3b2a54p-7f);
    q = __builtin_fmaf(q, f, 0x1.c6af6cp-5f);
    q = __builtin_fmaf(q, f, 0x1.ebfbe0p-3f);
    q = __builtin_fmaf(q, f, 0x1.62e430p-1f);
    float p = __builtin_fmaf(q, f, 1.0f);
    return __builtin_ldexpf(p, (int)k);
}

// The same for -64 <= y <= 0 without the test (callers that clamp y themselves).
__device__ __forceinline__ float exact_exp2_noguard(float y)
{
    float k = __builtin_rintf(y);
    float f = y - k;
    float q = 0x1.44138ap-13f;
    q = __builtin_fmaf(q, f, 0x1.5f0890p-10f);
    q = __builtin_fmaf(q, f, 0x1.3b2a54p-7f);
    q = __builtin_fmaf(q, f, 0x1.c6af6cp-5f);
    q = __builtin_fmaf(q, f, 0x1.ebfbe0p-3f);
    q = __builtin_fmaf(q, f, 0x1.62e430p-1f);
    float p = __builtin_fmaf(q, f, 1.0f);
    return __builtin_ldexpf(p, (int)k);
}

// ---- ln x for positive normal x ---------------------------------------------------------------
__device__ __forceinline__ float exact_log(float x)
{
    uint32_t bits = f2u(x);
    int e = (int)(bits >> 23) - 127;
    float m = u2f((bits & 0x007FFFFFu) | 0x3F800000u);
    if (m > 0x1.6a09e6p+0f) { m = m * 0.5f; e += 1; }
    float t = m - 1.0f;
    float s = t / (2.0f + t);
    float z = s * s;
    float w = 0x1.c71c72p-3f;
    w = __builtin_fmaf(w, z, 0x1.24924ap-2f);
    w = __builtin_fmaf(w, z, 0x1.99999ap-2f);
    w = __builtin_fmaf(w, z, 0x1.555556p-1f);
    float lnm = __builtin_fmaf(s * z, w, 2.0f * s);
    return __builtin_fmaf((float)e, 0x1.62e430p-1f, lnm);
}

// y = (l - m) * c: subtraction, then multiplication (two roundings)
__device__ __forceinline__ float scaled_offset(float l, float m, float c)
{
    float d = l - m;
    return d * c;
}

// The row normaliser is the integer S = sum_v floor(E(y_v) * 2^fx) with fx = min(40, 62 - ceil(log2 V)), so
// that S < 2^63 for every vocabulary; s = (float)((double)S * 2^-fx).  `shift` below is 40 - fx (0 up to
// V = 2^22).
__device__ __forceinline__ float normaliser_from_fixed(uint64_t S, int shift)
{
    double d = (double)S;
    d = __builtin_ldexp(d, shift - 40);
    return (float)d;
}

// ---- ordering keys --------------------------------------------------------------------------
// Monotone map float -> uint32 (larger value, larger key); -0 is folded onto +0 first.
__device__ __forceinline__ uint32_t order_key(float f)
{
    uint32_t b = f2u(f + 0.0f);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float order_key_inv(uint32_t k)
{
    uint32_t b = (k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k;
    return u2f(b);
}
// (value desc, id asc) as one integer: larger is better
__device__ __forceinline__ uint64_t rank_key(float value, uint32_t id)
{
    return ((uint64_t)order_key(value) << 32) | (uint64_t)(0xFFFFFFFFu - id);
}
__device__ __forceinline__ uint32_t rank_key_id(uint64_t k) { return 0xFFFFFFFFu - (uint32_t)k; }
__device__ __forceinline__ float rank_key_value(uint64_t k) { return order_key_inv((uint32_t)(k >> 32)); }

// ---- key fingerprint ------------------------------------------------------------------------
__host__ __device__ inline uint64_t fmix64(uint64_t h)
{
    h ^= h >> 33; h *= 0xff51afd7ed558ccdULL;
    h ^= h >> 33; h *= 0xc4ceb9fe1a85ec53ULL;
    h ^= h >> 33;
    return h;
}
// Key fingerprint: fmix64(n * C + sum_i M_i * (x_i + 1)), x_i = the token i positions before the
// end of the key (x_0 = newest); 0 is mapped to 1.  The terms are independent of each other.
__host__ __device__ inline uint64_t fingerprint_multiplier(int i)
{
    constexpr uint64_t m[kMaxOrder] = {0x9E3779B97F4A7C15ULL, 0xC2B2AE3D27D4EB4FULL, 0x165667B19E3779F9ULL,
                                       0xD6E8FEB86659FD93ULL, 0xA0761D6478BD642FULL, 0xE7037ED1A0B428DBULL,
                                       0x8EBC6AF09C88C6E3ULL, 0x589965CC75374CC3ULL};
    return m[i];
}
// newest_first[i] = token i positions before the end of the key
__host__ __device__ inline uint64_t fingerprint_newest_first(int n, const int32_t *newest_first)
{
    uint64_t acc = (uint64_t)n * 0x2545F4914F6CDD1DULL;
#pragma unroll
    for (int i = 0; i < kMaxOrder; ++i)
        if (i < n) acc += fingerprint_multiplier(i) * ((uint64_t)(uint32_t)newest_first[i] + 1u);
    const uint64_t h = fmix64(acc);
    return h ? h : 1;
}
// tokens[0..n) oldest first
__host__ __device__ inline uint64_t fingerprint(int n, const int32_t *tokens)
{
    uint64_t acc = (uint64_t)n * 0x2545F4914F6CDD1DULL;
    for (int i = 0; i < n; ++i) acc += fingerprint_multiplier(i) * ((uint64_t)(uint32_t)tokens[n - 1 - i] + 1u);
    const uint64_t h = fmix64(acc);
    return h ? h : 1;
}

}  // namespace stand
