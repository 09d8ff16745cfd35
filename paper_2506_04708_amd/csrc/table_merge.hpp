// table_merge.hpp -- the n-gram table's update: slot claims, merge_apply_kernel, context append (paper Sec. 4.1).
#pragma once
#include "wave_ops.hpp"

namespace stand {

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
    st_agent(&a.rec_slot[rec], slot_out);
}


// One wave per record, kMergeWaves records per workgroup (most records of a step do not exist --
// paths are short -- and a launch of one small workgroup per record spends its time dispatching
// them).  The lowest record that claimed a slot (its leader, named in the slot header by the
// claim) applies all records of that slot in record order; the other records' waves leave at
// once.  A slot claimed by one record only needs no search for followers.  The waves of a
// workgroup do not interact.
constexpr int kMergeWaves = 16;

// Record `rec` by one wave (all 64 lanes call this; l_id / l_val: 2 * kMaxK words of shared memory
// owned by the wave).  Does nothing unless the record exists and leads its slot.
__device__ __forceinline__ void apply_record(const MergeArgs &a, int rec, int lane, int32_t *l_id, float *l_val)
{
    const int NO = a.omax - a.omin + 1;
    const int nrec = a.B * a.R * NO;
    const int K = a.K;
    const long long slot = ld_agent(&a.rec_slot[rec]);
    if (slot < 0) return;
    SlotHeader *h = slot_header(a.table, (uint64_t)slot, a.slot_bytes);
    int32_t *ids = slot_ids(a.table, (uint64_t)slot, a.slot_bytes);
    float *mus = slot_mu(a.table, (uint64_t)slot, a.slot_bytes, K);
    // header, stored entry and this record's observation are requested together
    const uint32_t order_word = ld_agent(&h->order);
    uint32_t count = ld_agent(&h->count);
    int32_t e_id = -1;
    float e_mu = 0.0f;
    if (lane < K) { e_id = ld_agent(&ids[lane]); e_mu = ld_agent(&mus[lane]); }
    // lanes 0..K-1: stored entry; lanes 32..32+K-1: observation
    int32_t o_id = -1;
    float o_p = 0.0f;
    if (lane >= 32 && lane < 32 + K) {
        o_id = ld_agent(&a.obs_idx[(size_t)(rec / NO) * K + (lane - 32)]);
        o_p = ld_agent(&a.obs_p[(size_t)(rec / NO) * K + (lane - 32)]);
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
        // the later records of this slot, in record order (four groups of 64 record slots are read per round)
        for (int base = rec + 1; base < nrec; base += 256) {
            long long rs[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int r = base + 64 * q + lane;
                rs[q] = r < nrec ? ld_agent(&a.rec_slot[r]) : -1;
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                unsigned long long hits = __ballot(rs[q] == slot);
                while (hits) {
                    const int bit = __ffsll((long long)hits) - 1;
                    hits &= hits - 1;
                    const int jb = (base + 64 * q + bit) / NO;  // = b * R + j
                    int32_t f_id = -1;
                    float f_p = 0.0f;
                    if (lane >= 32 && lane < 32 + K) { f_id = ld_agent(&a.obs_idx[(size_t)jb * K + (lane - 32)]); f_p = ld_agent(&a.obs_p[(size_t)jb * K + (lane - 32)]); }
                    apply(f_id, f_p);
                }
            }
        }
    }
    if (lane < K) { st_agent(&ids[lane], e_id); st_agent(&mus[lane], e_mu); }
    if (lane == 0) { st_agent(&h->count, count); st_agent(&h->order, order_word & ((1u << kTagShift) - 1u)); }
}

__global__ __launch_bounds__(64 * kMergeWaves) void merge_apply_kernel(MergeArgs a)
{
    __shared__ int32_t l_id_all[kMergeWaves][2 * kMaxK];
    __shared__ float l_val_all[kMergeWaves][2 * kMaxK];
    const int NO = a.omax - a.omin + 1;
    const int nrec = a.B * a.R * NO;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int rec = (int)blockIdx.x * kMergeWaves + wave;
    if (rec >= nrec) return;
    apply_record(a, rec, lane, l_id_all[wave], l_val_all[wave]);
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

}  // namespace stand
