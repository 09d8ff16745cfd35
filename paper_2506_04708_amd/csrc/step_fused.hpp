// step_fused.hpp -- stand_step_kernel: one speculation step in ONE launch (paper Sec. 3.2, 4.1, 4.2).
//
// The step's dependent part (path walk, exact sums of the path rows, resampled token, table merge,
// next draft) needs only the rows on the accepted paths, which lie in the upper levels of the tree,
// and moves under 2 % of the step's bytes; run after the row pass it still costs a quarter of the
// step, because it is a chain of dependent round trips to memory.  Here it runs BESIDE the row pass:
//
//   workgroups [0, P)          rows: first those of the tree's upper levels (node-major), one row per
//                              workgroup, then others up to what the device holds at once less two tail
//                              workgroups per trajectory
//   workgroups [P, P + B*G)    the tail: G workgroups per trajectory (all first ones, then all second ones, ...)
//   the rest                   all other rows
//
// Workgroups start in index order, so the first P rows and the first two tail workgroups of every trajectory
// fill the device: the rows finish together, those tail workgroups wait in place and follow the path the moment
// its rows are there; the other tail workgroups take the first places that become free.  All of the tail works
// while the remaining rows stream.  A tail workgroup never assumes anything about timing: it WAITS for what it
// needs -- the published results of each row on its path (any row, also one that is dispatched after it;
// self-validating words, see RowPub), the partial sums of its trajectory's other workgroups, and twice for all
// trajectories (every claim before the first apply, every apply before the first lookup of the draft).  Every
// wait polls a word at device scope, sleeps between the polls and gives up after a bounded time (counted in the
// statistics; the trajectory's outputs are then void); counters only ever grow (launch number times arrivals
// per launch) and published words carry the launch number, so nothing needs clearing between launches.  What a
// workgroup waits for is always produced by workgroups that need nothing from it.
#pragma once
#include "draft.hpp"
#include "path_pass.hpp"

namespace stand {

#ifndef STAND_STEP_WPR
#define STAND_STEP_WPR 8
#endif
constexpr int kStepWPR = STAND_STEP_WPR;     // waves per workgroup; a row is shared by all of them
constexpr int kStepThreads = 64 * kStepWPR;
#ifndef STAND_STEP_MINWAVES
#define STAND_STEP_MINWAVES 6   // waves per SIMD the kernel's register use must leave room for
#endif
#ifndef STAND_POLL_SLEEP
#define STAND_POLL_SLEEP 8   // argument of s_sleep between two polls of a wait (units of 64 clocks)
#endif
#ifndef STAND_TAIL_INFLIGHT
#define STAND_TAIL_INFLIGHT 8
#endif
constexpr int kTailInflight = STAND_TAIL_INFLIGHT;  // 16-byte loads a lane of the tail keeps in flight while it sums a row segment
constexpr int kPathPub = 2 * (kMaxDepth + 2) + 2;  // words per trajectory of the published path
constexpr unsigned long long kPartThere = 1ull << 63;  // set in a stored partial sum of this launch
constexpr unsigned kWaitMaxPolls = 1u << 24;  // a wait ends after this many polls whatever the clock says

struct StepSync {
    RowPub pub;                     // what a row hands to the tail: self-validating words, tag = epoch
    unsigned *item_next;            // [B]    next (path row, segment) item to hand out: (launch number & 0xFFFF) << 16 | item
    unsigned *path_flag;            // [B]    launch number once the trajectory's path is published
    int32_t *path_pub;              // [B][kPathPub] the path: length, nodes, then the bit patterns of the rows' maxima
    unsigned *bar;                  // [2]    +B per launch each: all claims made / all records applied
    unsigned epoch;                 // number of this launch on the handle, from 1
    unsigned long long wait_ticks;  // bound of every wait in ticks of the device's constant clock (wall_clock64)
    unsigned long long *stamps;     // NULL, or [2 + 8 * B] clock readings of this launch: earliest row start, latest row
                                    // end, then per trajectory: tail start, path known, sums done, claims made, rows
                                    // finished, all claims in, all records applied, draft done
};

struct StepArgs {
    RowPassArgs row;
    PathArgs path;       // mode 0, accepted-path update
    MergeArgs mg;
    DraftArgs draft;     // writes the OTHER copy of the draft state: rows still streaming read the pending one
    StepSync sync;
    int upper_nodes;     // rows of tree nodes [0, upper_nodes) are the first row slots
    int rows_first;      // row workgroups (>= upper_nodes * B) that come before the tail's
    int G;               // tail workgroups per trajectory
    uint32_t shuffle_mul, shuffle_add;  // row slots inside each group are permuted by slot * mul + add (1, 0: identity)
};

// Polls *p until it has reached `target` (wrap-safe: counters are at most one launch behind).
__device__ __forceinline__ bool wait_reached(const unsigned *p, unsigned target, unsigned long long ticks)
{
    // The polls are relaxed device-scope loads.  What the arriving workgroups stored before they arrived was
    // stored at device scope and had completed (publish_fence); it is read with ld_agent after this returns.
    bool seen = (int)(__hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - target) >= 0;
    if (!seen) {
        const unsigned long long t0 = wall_clock64();
        // bounded twice: by the device's constant clock and by a count of polls (each takes a fraction of a microsecond)
        for (unsigned polls = 0; polls < kWaitMaxPolls && !seen; ++polls) {
            __builtin_amdgcn_s_sleep(STAND_POLL_SLEEP);
            seen = (int)(__hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - target) >= 0;
            if (!seen && wall_clock64() - t0 > ticks) break;
        }
    }
    if (seen) consume_fence();
    return seen;
}

// Polls a row's published word until it carries this launch's tag (bounded like every wait).
__device__ __forceinline__ bool wait_row_pub(const unsigned long long *p, unsigned tag, unsigned long long ticks,
                                             unsigned long long &w)
{
    w = ld_agent(p);
    bool seen = row_pub_there(w, tag);
    if (!seen) {
        const unsigned long long t0 = wall_clock64();
        for (unsigned polls = 0; polls < kWaitMaxPolls && !seen; ++polls) {
            __builtin_amdgcn_s_sleep(STAND_POLL_SLEEP);
            w = ld_agent(p);
            seen = row_pub_there(w, tag);
            if (!seen && wall_clock64() - t0 > ticks) break;
        }
    }
    return seen;
}

__device__ __forceinline__ void stamp(const StepSync &sy, int b, int k)
{
    if (sy.stamps) sy.stamps[2 + 8 * b + k] = wall_clock64();
}

struct TailShared {
    int path[kMaxDepth + 2];   // nodes of the accepted path
    int acc[kMaxDepth + 2];    // outcome of each of them
    float pm[kMaxDepth + 2];   // maximum of each of their rows
    int len, ok;
    FinishShared fin;
    int32_t l_id[kStepWPR][2 * kMaxK];
    float l_val[kStepWPR][2 * kMaxK];
};

// All workgroups of one count arrive, then wait for the rest.  Called by the whole workgroup.
__device__ __forceinline__ void tail_barrier(const StepSync &sy, int which, unsigned arrivals, TailShared *ts)
{
    publish_fence();  // this workgroup's stores (table, records, observations) are complete before its arrival
    __syncthreads();
    if (threadIdx.x == 0) {
        atomicAdd(&sy.bar[which], 1u);
        if (!wait_reached(&sy.bar[which], arrivals * sy.epoch, sy.wait_ticks)) ts->ok = 0;
    }
    __syncthreads();
    consume_fence();
}

template <int DT>
__device__ __forceinline__ void tail_role(const StepArgs &A, int b, int g, char *smem)
{
    constexpr int ES = VecTraits<DT>::ES;
    const PathArgs &a = A.path;
    const StepSync &sy = A.sync;
    TailShared *ts = (TailShared *)smem;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int N = a.N, W = a.W, K = a.K;

    // ---- the accepted path: the trajectory's first workgroup follows the outcomes from the root, waiting for
    // each row on the way, and publishes the path; the others wait for the publication
    const unsigned tag = (sy.epoch & 0xFFFFu) << 16;
    int32_t *pub = sy.path_pub + (size_t)b * kPathPub;
    if (g == 0) {
        if (tid == 0) {
            stamp(sy, b, 0);
            int cur = 0, len = 0, ok = 1;
            for (;;) {
                unsigned long long rw;
                if (!wait_row_pub(&sy.pub.row[(size_t)b * N + cur], sy.epoch, sy.wait_ticks, rw)) { ok = 0; break; }
                const int acc = row_pub_outcome(rw);
                ts->pm[len] = row_pub_max(rw);
                ts->path[len] = cur;
                ts->acc[len] = acc;
                ++len;
                if (acc < 0 || len > a.tree.D) break;
                const int nxt = a.tree.first_child[cur] + acc;
                if (nxt <= cur || nxt >= N) break;  // not reachable for outcomes of this tree
                cur = nxt;
            }
            ts->len = ok ? len : 0;
            ts->ok = ok;
            // the first items belong to the trajectory's own waves, one each; the counter hands out the rest
            st_agent(&sy.item_next[b], tag + (unsigned)(A.G * kStepWPR - 1));
            stamp(sy, b, 1);
        }
        __syncthreads();
        // the partial sums this launch will produce are marked "not there yet"
        for (int i = tid; i < ts->len * a.nseg; i += kStepThreads)
            st_agent(&a.seg_part[((size_t)b * a.R + i / a.nseg) * kSegMax + i % a.nseg], 0ull);
        if (tid < ts->len) {
            st_agent(&pub[1 + tid], (int32_t)ts->path[tid]);
            st_agent(&pub[1 + (kMaxDepth + 2) + tid], (int32_t)f2u(ts->pm[tid]));
        }
        if (tid == 0) st_agent(&pub[0], (int32_t)ts->len);
        publish_fence();
        __syncthreads();
        if (tid == 0) st_agent(&sy.path_flag[b], sy.epoch);
    } else {
        if (tid == 0) {
            ts->ok = wait_reached(&sy.path_flag[b], sy.epoch, sy.wait_ticks) ? 1 : 0;
            ts->len = ts->ok ? ld_agent(&pub[0]) : 0;
        }
        __syncthreads();
        if (tid < ts->len) {
            ts->path[tid] = ld_agent(&pub[1 + tid]);
            ts->pm[tid] = u2f((uint32_t)ld_agent(&pub[1 + (kMaxDepth + 2) + tid]));
        }
        __syncthreads();
    }
    consume_fence();
    const int len = ts->len;

    // ---- exact partial sums.  An item is (path row j, segment).  The first G * waves - 1 items of a trajectory
    // belong to its own waves, one each (a row has at most that many segments; the first wave of the first
    // workgroup has other work, see below); further items (paths of several rows) are handed out by a counter
    // to whichever wave asks next: the trajectory's own waves, then those of other trajectories' helper
    // workgroups that have run out of work.  A partial sum is stored with its top bit set ("there").
    const int nseg = a.nseg;
    auto sum_item = [&](int t, int item, int node, float m) {
        const int j = item / nseg, seg = item % nseg;
        const int row = t * N + node;
        const char *rowp = (const char *)a.logits + (size_t)row * (size_t)a.V * ES;
        const RowGeom geo = row_geom<DT>(rowp, a.V);
        const int per = (geo.nvec + nseg - 1) / nseg;
        const int v0 = seg * per < geo.nvec ? seg * per : geo.nvec;
        const int v1 = (v0 + per < geo.nvec) ? v0 + per : geo.nvec;
#ifdef STAND_DEBUG_SKIP_SUMS
        unsigned long long S = (unsigned long long)(v1 - v0);
#else
        unsigned long long S = thread_exact_partial<DT, kTailInflight>(rowp, geo, v0, v1, seg == 0, m, a.c, lane, 64, a.fx_shift);
#endif
        S = wave_sum_u64(S);  // below 2^62 (a whole row's sum is)
        if (lane == 0) st_agent(&a.seg_part[((size_t)t * a.R + j) * kSegMax + seg], S | kPartThere);
    };
    // asks for the next item of trajectory t; the answer (lane 0's register) is looked at after the current
    // item has been summed, so the round trip of the request is not waited for
    auto request = [&](int t) {
        unsigned v = 0u;
        if (lane == 0) v = atomicAdd(&sy.item_next[t], 1u);
        return v;
    };
    auto answer = [&](unsigned v) { return (unsigned)__builtin_amdgcn_readfirstlane((int)v) - tag; };
    const bool control = g == 0 && wave == 0;  // this wave writes the outputs and claims the table slots meanwhile
    if (!control) {
        const unsigned n_items = (unsigned)(len * nseg), own = (unsigned)(A.G * kStepWPR - 1);
        unsigned it = (unsigned)(g * kStepWPR + wave - 1);
        while (it < n_items) {
            const bool more = n_items > own;  // uniform: only paths of several rows have items beyond the first round
            const unsigned req = more ? request(b) : 0u;
            sum_item(b, (int)it, ts->path[it / nseg], ts->pm[it / nseg]);
            it = more ? answer(req) : n_items;
        }
    }
    if (g != 0) {
        // help the trajectories that still have items (one look at all of them, starting behind this one)
        for (int k0 = 0; k0 < a.B; k0 += 64) {
            const int t = (b + 1 + k0 + lane) % a.B;
            int tl = 0;
            bool has = false;
            if (k0 + lane < a.B - 1 && ld_agent(&sy.path_flag[t]) == sy.epoch) {
                tl = ld_agent(&sy.path_pub[(size_t)t * kPathPub]);
                has = ld_agent(&sy.item_next[t]) - tag < (unsigned)(tl * nseg);
            }
            unsigned long long todo = __ballot(has);
            while (todo) {
                const int src = __ffsll((long long)todo) - 1;
                todo &= todo - 1;
                const int tt = __builtin_amdgcn_readlane(t, src);
                const unsigned n_items = (unsigned)(__builtin_amdgcn_readlane(tl, src) * nseg);
                const int32_t *tp = sy.path_pub + (size_t)tt * kPathPub;
                unsigned it = answer(request(tt));
                while (it < n_items) {
                    const int j = (int)it / nseg;
                    const int node = ld_agent(&tp[1 + j]);
                    const float m = u2f((uint32_t)ld_agent(&tp[1 + (kMaxDepth + 2) + j]));
                    const unsigned req = request(tt);
                    if ((uint32_t)node < (uint32_t)N) sum_item(tt, (int)it, node, m);  // (always true for a published path)
                    it = answer(req);
                }
            }
        }
        return;  // the trajectory's other workgroups only help with the sums
    }

    // (the code from here on runs in the trajectory's first workgroup only)
    // ---- its first wave, while the others sum: the outputs of the verification, the stop node's proposal
    // (requested now, used after the sums) and the table slots of the trajectory's merge records, which
    // depend on the path's tokens only
    const int stop_node = len > 0 ? ts->path[len - 1] : 0;
    const int stop_row = b * N + stop_node;
    const char *stop_rowp = (const char *)a.logits + (size_t)stop_row * (size_t)a.V * ES;
    int nch = 0, fc = -1;
    int32_t my_id = -1, ch = -1;
    float my_mu = 0.0f, my_l = 0.0f, stop_m = 0.0f;
    if (len > 0) {
        fc = a.tree.first_child[stop_node];
        nch = a.draft_has[stop_row];
        stop_m = ts->pm[len - 1];
    }
    if (control) {
        if (len > 0) {
            if (lane < K) { my_id = a.draft_qid[(size_t)stop_row * K + lane]; my_mu = a.draft_qmu[(size_t)stop_row * K + lane]; }
            if (lane < nch && lane < kMaxK && fc >= 0 && fc + lane < N) ch = a.draft_tok[(size_t)b * N + fc + lane];
            if ((uint32_t)my_id >= (uint32_t)a.V) { my_id = -1; my_mu = 0.0f; }  // never index outside the row
            else my_l = load_scalar<DT>(stop_rowp, my_id);
        }
        if (lane < W) {  // W <= 32
            a.out_node[(size_t)b * W + lane] = lane < len ? ts->path[lane] : -1;
            // accepted tokens are the tokens of the path nodes after the root; the last emitted token
            // (position len - 1) is written by finish_row
            if (lane + 1 < len) a.out_tok[(size_t)b * W + lane] = a.draft_tok[(size_t)b * N + ts->path[lane + 1]];
            else if (lane >= len - 1) a.out_tok[(size_t)b * W + lane] = -1;
        }
        if (lane < len) atomicAdd(&a.node_count[ts->path[lane]], 1ull);  // paper Sec. 4.3: acceptance statistics per node
        if (lane == 0) {
            a.out_len[b] = len;
            if (len > 0) {
                unsigned long long tests = (unsigned long long)nch;
                for (int q = 0; q + 1 < len; ++q) tests += (unsigned long long)(ts->acc[q] + 1);
                atomicAdd(&a.stats[kStatTokens], (unsigned long long)len);
                atomicAdd(&a.stats[kStatTests], tests);
                if (len > a.late_len) atomicAdd(&a.stats[kStatLatePaths], 1ull);
            } else {
                atomicAdd(&a.stats[kStatWaitExpired], 1ull);
            }
        }
        publish_fence();  // out_len and the accepted tokens, written by this wave, are what its claims read
        const int per_traj = A.mg.R * (A.mg.omax - A.mg.omin + 1);
        for (int i = lane; i < per_traj; i += 64) merge_claim_record(A.mg, b * per_traj + i);
    }
    // ---- the partial sums (of whichever waves summed them), then the rows' observations and the resampled token
    if (tid == 0) stamp(sy, b, 3);
    auto wait_parts = [&](int j) {  // one wave: lanes < nseg each wait for their segment of path row j,
                                    // lanes < K for their word of the row's top-K (its ranking wave may still be at work)
        const unsigned long long *p = &a.seg_part[((size_t)b * a.R + j) * kSegMax];
        const unsigned long long *tp = &sy.pub.top[((size_t)b * N + ts->path[j]) * K];
        unsigned long long v = lane < nseg ? ld_agent(p + lane) : kPartThere;
        bool top_ok = lane < K ? top_pub_there(ld_agent(tp + lane), sy.epoch) : true;
        if (!__all((v & kPartThere) != 0ull && top_ok)) {
            const unsigned long long t0 = wall_clock64();
            for (unsigned polls = 0; polls < kWaitMaxPolls; ++polls) {
                __builtin_amdgcn_s_sleep(STAND_POLL_SLEEP);
                if (!(v & kPartThere)) v = ld_agent(p + lane);
                if (!top_ok) top_ok = top_pub_there(ld_agent(tp + lane), sy.epoch);
                if (__all((v & kPartThere) != 0ull && top_ok)) break;
                if (wall_clock64() - t0 > sy.wait_ticks) break;
            }
        }
        if (!__all((v & kPartThere) != 0ull && top_ok) && lane == 0) ts->ok = 0;
        consume_fence();
        return v & ~kPartThere;
    };
    if (len > 0) {
        const unsigned long long part_stop = wave == 0 ? wait_parts(len - 1) : 0ull;
        if (tid == 0) stamp(sy, b, 2);
        for (int j = wave; j + 1 < len; j += kStepWPR) {  // rows above the stop row: one wave each
            const int node = ts->path[j];
            const unsigned long long part = wait_parts(j);
            finish_row<DT, kStepThreads>(a, ts->fin, b, j, node, false, ts->pm[j], 0, -1, len, -1, 0.0f, 0.0f, -1, part, lane, 0, ts->acc[j]);
        }
        __syncthreads();
        if (ts->ok) {
            finish_row<DT, kStepThreads>(a, ts->fin, b, len - 1, stop_node, true, stop_m, nch, fc, len, my_id, my_mu, my_l, ch, part_stop,
                                         tid, wave);
        } else if (tid == 0) {
            a.out_tok[(size_t)b * W + (len - 1)] = -1;
            atomicAdd(&a.stats[kStatWaitExpired], 1ull);
        }
    }

    // ---- every trajectory's claims and observations, then this trajectory's records
    if (tid == 0) stamp(sy, b, 4);
    tail_barrier(sy, 0, (unsigned)a.B, ts);
    if (tid == 0) stamp(sy, b, 5);
    {
        const int NO = A.mg.omax - A.mg.omin + 1;
        for (int i = wave; i < len * NO; i += kStepWPR) apply_record(A.mg, b * A.mg.R * NO + i, lane, ts->l_id[wave], ts->l_val[wave]);
    }
    // ---- every trajectory's records applied, then the next draft
    tail_barrier(sy, 1, (unsigned)a.B, ts);
    if (tid == 0) stamp(sy, b, 6);
    if (tid == 0 && !ts->ok) atomicAdd(&a.stats[kStatWaitExpired], 1ull);
    draft_trajectory<kStepThreads>(A.draft, b, draft_shared_carve(smem + ((sizeof(TailShared) + 15) & ~(size_t)15), A.draft.tree.N, A.draft.tree.D));
    if (tid == 0) stamp(sy, b, 7);
}

__host__ __device__ inline size_t step_shared_bytes(int N, int D)
{
    const size_t tail = ((sizeof(TailShared) + 15) & ~(size_t)15) + draft_shared_bytes(N, D);
    return tail > sizeof(RowShared<kStepWPR>) ? tail : sizeof(RowShared<kStepWPR>);
}

template <int DT>
__global__ __launch_bounds__(kStepThreads) __attribute__((amdgpu_waves_per_eu(STAND_STEP_MINWAVES, 8))) void stand_step_kernel(StepArgs A)
{
    extern __shared__ __align__(16) char step_smem[];
    const int B = A.row.B, rows = A.row.B * A.row.N;
    const int n_up = A.upper_nodes * B, n_first = A.rows_first, n_tail = B * A.G;
    const int i = (int)blockIdx.x;
    if (i >= n_first && i < n_first + n_tail) {
        const int t = i - n_first;
        // the tail's waves go first where they share a SIMD with streaming waves: the chain of dependent steps is
        // what the launch ends with in its heavy steps (0.1254-0.1265 against 0.1265-0.1273 ms per step; the other
        // way round, rows first, costs 8 %)
        __builtin_amdgcn_s_setprio(3);
        tail_role<DT>(A, t % B, t / B, step_smem);
        return;
    }
    // row slots: [0, n_up) the upper levels, [n_up, rows) the others; node-major inside each group
    int slot = i < n_first ? i : i - n_tail;
    if (slot >= rows) return;
    {
        const int base = slot < n_up ? 0 : n_up, n = slot < n_up ? n_up : rows - n_up;
        slot = base + (int)(((unsigned long long)(slot - base) * A.shuffle_mul + A.shuffle_add) % (unsigned)n);
    }
    const int row = (slot % B) * A.row.N + slot / B;
    if (A.sync.stamps && threadIdx.x == 0) atomicMin(&A.sync.stamps[0], (unsigned long long)wall_clock64());
    row_role<DT, kStepWPR>(A.row, row, (RowShared<kStepWPR> *)step_smem, A.sync.pub);
    if (A.sync.stamps && (threadIdx.x == 0 || threadIdx.x == 64)) atomicMax(&A.sync.stamps[1], (unsigned long long)wall_clock64());
}

}  // namespace stand
