// aux_kernels.hpp -- fills, copies, tree packing for the target model's verify pass, table export.
#pragma once
#include "wave_ops.hpp"

namespace stand {

// small helpers --------------------------------------------------------------------------------
__global__ void fill_i32_kernel(int32_t *p, int32_t v, size_t n)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

// Beam copy: context tail and length of trajectory b become those of trajectory src_of[b].  The new
// values go to a second pair of arrays (a map may name a trajectory as source and destination at once).
__global__ void reorder_gather_kernel(int B, const int32_t *src_of, const int32_t *tail_in, const long long *len_in,
                                      int32_t *tail_out, long long *len_out)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= B * kMaxOrder) return;
    const int b = i / kMaxOrder, q = i % kMaxOrder;
    int s = src_of[b];
    s = s < 0 ? 0 : (s >= B ? B - 1 : s);  // validated on the host; never index outside
    tail_out[i] = tail_in[(size_t)s * kMaxOrder + q];
    if (q == 0) len_out[b] = len_in[s];
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
