// stand_api.hip -- host side of libstand: the C ABI declared in include/stand.h.
// Validates arguments, owns the device state of a handle and launches the kernels of
// kernels.hpp.  No CPU fallback exists: every step of the path runs in the HIP kernels.
#include "../../include/stand.h"
#include "kernels.hpp"

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

using namespace stand;

// Device memory that one verification uses between its kernels (results of the row pass, partial sums,
// the stop records, observations).  A handle owns one set; the entry point that must not allocate carves
// the same set out of the file-scope array below.
struct VerifyScratch {
    float *row_m, *row_s, *top_l, *top_p;
    int32_t *top_idx, *outcome;
    int32_t *obs_idx;
    float *obs_p;
    unsigned long long *seg_part;
    int32_t *stop_i, *stop_qid, *stop_child;
    float *stop_m, *stop_qmu, *stop_ql;
};

struct stand_handle {
    stand_config cfg;
    int N, D, K, B, V, W, NO, slot_bytes;
    float c;
    int last_hip;
    std::vector<int32_t> parent, depth, nchild, first_child, level_start;
    int32_t *d_tree;  // parent | depth | nchild | first_child | level_start
    char *table;
    int32_t *ctx_tail, *ctx_tail2;   // context tails; the second array receives the result of a beam copy
    long long *ctx_len, *ctx_len2;
    int32_t *reorder_map;            // [B] device copy of the map of the last stand_reorder
    char *export_buf;                // compacted table of the last stand_table_export (kept, grown on demand)
    uint64_t export_cap;
    int32_t *draft_tok, *draft_has, *draft_qid;   // the pending draft
    float *draft_qmu;
    int32_t *draft_tok2, *draft_has2, *draft_qid2;  // second copy: the one-launch step writes the next draft here
    float *draft_qmu2;                              // while rows that are still streaming read the pending one
    // one-launch step (stand_step_kernel)
    unsigned long long *row_pub, *top_pub;  // what a row hands to the tail of the same launch (RowPub)
    unsigned *bar;             // counters that only grow, see step_fused.hpp
    unsigned *item_next, *path_flag;
    int32_t *path_pub;
    unsigned step_epoch;
    int step_mode;       // STAND_STEP_AUTO / SERIAL / FUSED
    int upper_depth;     // rows of nodes up to this depth are dispatched before the tail
    int tail_groups;     // tail workgroups per trajectory (0: chosen from the batch size)
    int rows_first;      // row workgroups dispatched before the tail's (0: as many as the device holds at once)
    int step_slots;      // workgroups of stand_step_kernel the device holds at once (0: not asked yet)
    uint32_t shuffle;    // non-zero: row slots are permuted (a test of independence from the work mapping)
    uint64_t wait_limit_us;
    int wall_khz;        // rate of the device's constant clock (wall_clock64)
    int fx_shift;        // 40 - (fraction bits of the exact normaliser's terms): 0 up to V = 2^22
    // STAND_STEP_AUTO watches how often accepted paths reach below the rows that are scheduled first and
    // takes the separate launches while that is common (plan_observe)
    unsigned long long *probe_host;  // pinned: kStatLatePaths as last copied
    hipEvent_t probe_ev;
    bool probe_pending, plan_serial;
    uint64_t probe_steps, probe_issue_steps, probe_base_steps, probe_base_late;
    unsigned long long *stamps;  // [2 + 8 * B] clock readings of the last one-launch step, or NULL (stand_step_timeline)
    VerifyScratch vs;  // row results, partial sums, stop records, observations (hipMalloc'ed at create)
    long long *rec_slot;
    int R;            // row / record slots per trajectory: W, or N with STAND_UPDATE_ALL_NODES
    int32_t *recent;  // [B][N][kMaxOrder], all-nodes mode only
    unsigned long long *node_count, *anc;  // anc: [N][anc_words] ancestor-or-self bit sets
    int anc_words;
    float *pr_m, *pr_top_l;
    int32_t *pr_top_idx;
    unsigned long long *stats;
    unsigned long long *counter;
    bool table_used;
    // optional timing of the row pass: event pairs recorded on the caller's stream
    bool profiling;
    float filter_margin;  // relative error assumed for the fast normaliser in the accept tests
    std::vector<hipEvent_t> ev_begin, ev_end;
    size_t ev_used;
};

// Scratch of stand_verify_static: one copy per GPU, held until the process ends.  In host code this
// name is only a handle for hipGetSymbolAddress, never an address: every use goes through the
// per-device pointer resolved in static_scratch_ptr().
static __device__ __align__(256) unsigned char scratch[STAND_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
static void *g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each GPU (NULL: not resolved yet)

// Resolves the array's address on `device` (which must be the current device).  Called from
// stand_create, i.e. once per device before any entry point can need it; no allocation involved.
static hipError_t static_scratch_ptr(int device, void **out)
{
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    if (!g_scratch_ptr[device]) {
        void *p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[device] = p;
    }
    *out = g_scratch_ptr[device];
    return hipSuccess;
}

#define HIP_TRY(h, expr)                                   \
    do {                                                   \
        hipError_t e_ = (expr);                            \
        if (e_ != hipSuccess) {                            \
            if (h) (h)->last_hip = (int)e_;                \
            return STAND_EHIP;                             \
        }                                                  \
    } while (0)

static TreeDev tree_dev(const stand_handle *h)
{
    TreeDev t;
    t.parent = h->d_tree;
    t.depth = h->d_tree + h->N;
    t.nchild = h->d_tree + 2 * h->N;
    t.first_child = h->d_tree + 3 * h->N;
    t.level_start = h->d_tree + 4 * h->N;
    t.N = h->N;
    t.D = h->D;
    return t;
}

template <typename T>
static hipError_t dmalloc(T **p, size_t n)
{
    return hipMalloc((void **)p, n * sizeof(T) ? n * sizeof(T) : sizeof(T));
}

static void free_all(stand_handle *h)
{
    if (!h) return;
    void *ptrs[] = {h->d_tree, h->table, h->ctx_tail, h->ctx_len, h->ctx_tail2, h->ctx_len2, h->reorder_map, h->export_buf, h->draft_tok, h->draft_has, h->draft_qid, h->draft_qmu,
                    h->vs.row_m, h->vs.row_s, h->vs.top_l, h->vs.top_p, h->vs.top_idx, h->vs.outcome, h->vs.obs_idx, h->vs.obs_p, h->rec_slot,
                    h->recent, h->draft_tok2, h->draft_has2, h->draft_qid2, h->draft_qmu2, h->row_pub, h->top_pub, h->bar, h->item_next, h->path_flag, h->path_pub, h->stamps, h->vs.seg_part, h->node_count, h->anc, h->vs.stop_i, h->vs.stop_qid, h->vs.stop_child, h->vs.stop_m, h->vs.stop_qmu, h->vs.stop_ql, h->pr_m, h->pr_top_l, h->pr_top_idx, h->stats, h->counter};
    for (void *p : ptrs) (void)hipFree(p);
    for (hipEvent_t e : h->ev_begin) (void)hipEventDestroy(e);
    for (hipEvent_t e : h->ev_end) (void)hipEventDestroy(e);
    if (h->probe_ev) (void)hipEventDestroy(h->probe_ev);
    if (h->probe_host) (void)hipHostFree(h->probe_host);
    delete h;
}

extern "C" int stand_create(const stand_config *cfg, stand_handle **out)
{
    if (!cfg || !out || !cfg->tree_parent) return STAND_EINVAL;
    *out = nullptr;
    const int N = cfg->tree_nodes, K = cfg->topk;
    if (K < 1 || K > STAND_MAX_TOPK) return STAND_EINVAL;
    // a row is addressed with 32-bit byte offsets (buffer loads, prefetch a few batches past its end):
    // it must stay 128 KiB below 4 GiB
    if (cfg->vocab < K || cfg->vocab < 2) return STAND_EINVAL;
    if ((uint64_t)cfg->vocab * (cfg->logits_dtype == STAND_F32 ? 4u : 2u) > (1ull << 32) - (1ull << 17)) return STAND_EINVAL;
    if (cfg->max_batch < 1 || cfg->max_batch >= (1 << 20)) return STAND_EINVAL;
    if (cfg->order_min < 1 || cfg->order_max < cfg->order_min || cfg->order_max > STAND_MAX_ORDER) return STAND_EINVAL;
    if (N < 1 || N > STAND_MAX_NODES) return STAND_EINVAL;
    if (!(cfg->temperature > 0.0f) || !(cfg->temperature < 1e6f)) return STAND_EINVAL;
    if (cfg->table_capacity < 16 || (cfg->table_capacity & (cfg->table_capacity - 1))) return STAND_EINVAL;
    if (cfg->max_probe < 1) return STAND_EINVAL;
    if (cfg->logits_dtype != STAND_BF16 && cfg->logits_dtype != STAND_F32) return STAND_EINVAL;
    if (cfg->update_mode != STAND_UPDATE_ACCEPTED_PATH && cfg->update_mode != STAND_UPDATE_ALL_NODES) return STAND_EINVAL;
    if (cfg->draft_mode < STAND_DRAFT_GUMBEL_TOPK || cfg->draft_mode > STAND_DRAFT_DETERMINISTIC) return STAND_EINVAL;
    if (cfg->merge_policy != STAND_MERGE_MEAN && cfg->merge_policy != STAND_MERGE_REPLACE) return STAND_EINVAL;
    if ((int64_t)cfg->max_batch * N * (int64_t)cfg->vocab >= ((int64_t)1 << 40)) return STAND_EINVAL;
    // merge records are numbered in 23 bits (kTagMax); max_batch * tree depth * orders stays far below
    if ((int64_t)cfg->max_batch * (cfg->update_mode == STAND_UPDATE_ALL_NODES ? (int64_t)N : (int64_t)(kMaxDepth + 1)) * STAND_MAX_ORDER >
        (int64_t)kTagMax)
        return STAND_EINVAL;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || cfg->device < 0 || cfg->device >= ndev) return STAND_EINVAL;

    stand_handle *h = new (std::nothrow) stand_handle();
    if (!h) return STAND_ENOMEM;
    h->cfg = *cfg;
    h->N = N; h->K = K; h->B = cfg->max_batch; h->V = cfg->vocab;
    h->NO = cfg->order_max - cfg->order_min + 1;
    h->slot_bytes = 16 + 8 * K;
    h->c = (float)(1.4426950408889634 / (double)cfg->temperature);
    {
        // the exact normaliser sums floor(E * 2^fx) over the row; fx = min(40, 62 - ceil(log2 V)) keeps it below 2^63
        int lg = 0;
        while (((int64_t)1 << lg) < (int64_t)cfg->vocab) ++lg;
        const int fx = 62 - lg < 40 ? 62 - lg : 40;
        h->fx_shift = 40 - fx;
    }
    h->last_hip = 0;
    h->table_used = false;
    h->profiling = false;
    h->filter_margin = kFastEps;
    h->step_epoch = 0;
    h->export_buf = nullptr;
    h->export_cap = 0;
    h->step_mode = STAND_STEP_AUTO;
    h->upper_depth = 2;
    h->tail_groups = 0;
    h->rows_first = 0;
    h->step_slots = 0;
    h->shuffle = 0;
    h->wait_limit_us = 200000;
    h->stamps = nullptr;
    h->probe_host = nullptr; h->probe_ev = nullptr;
    h->probe_pending = false; h->plan_serial = false;
    h->probe_steps = h->probe_issue_steps = h->probe_base_steps = h->probe_base_late = 0;
    {
        int khz = 0;
        if (hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, cfg->device) != hipSuccess || khz <= 0) khz = 100000;
        h->wall_khz = khz;
    }
    h->ev_used = 0;

    // tree: breadth-first numbering with contiguous siblings <=> parents non-decreasing
    h->parent.assign(cfg->tree_parent, cfg->tree_parent + N);
    h->depth.assign(N, 0); h->nchild.assign(N, 0); h->first_child.assign(N, -1);
    bool ok = h->parent[0] == -1;
    for (int u = 1; ok && u < N; ++u) {
        const int p = h->parent[u];
        ok = p >= 0 && p < u && (u == 1 || p >= h->parent[u - 1]);
        if (!ok) break;
        h->depth[u] = h->depth[p] + 1;
        if (h->nchild[p] == 0) h->first_child[p] = u;
        h->nchild[p]++;
    }
    h->D = 0;
    for (int u = 0; ok && u < N; ++u) {
        h->D = std::max(h->D, h->depth[u]);
        if (h->nchild[u] > K) ok = false;
    }
    if (!ok || h->D > STAND_MAX_DEPTH) { delete h; return STAND_EINVAL; }
    h->cfg.tree_parent = nullptr;
    h->W = h->D + 1;
    h->R = cfg->update_mode == STAND_UPDATE_ALL_NODES ? N : h->W;
    h->level_start.assign(h->D + 2, N);
    for (int u = N - 1; u >= 0; --u) h->level_start[h->depth[u]] = u;

    if (hipSetDevice(cfg->device) != hipSuccess) { delete h; return STAND_EHIP; }
    {
        // address of the static scratch array on this device, for stand_verify_static
        void *sp = nullptr;
        const hipError_t se = static_scratch_ptr(cfg->device, &sp);
        if (se != hipSuccess) { h->last_hip = (int)se; delete h; return STAND_EHIP; }
    }
    const size_t B = h->B, rows = B * N;
    const size_t nrec = B * h->R * h->NO;
    hipError_t e = hipSuccess;
    auto acc = [&](hipError_t x) { if (e == hipSuccess) e = x; };
    acc(dmalloc(&h->d_tree, 4 * (size_t)N + h->D + 2));
    acc(hipMalloc((void **)&h->table, (size_t)cfg->table_capacity * h->slot_bytes));
    acc(dmalloc(&h->ctx_tail, B * kMaxOrder));
    acc(dmalloc(&h->ctx_len, B));
    acc(dmalloc(&h->ctx_tail2, B * kMaxOrder)); acc(dmalloc(&h->ctx_len2, B)); acc(dmalloc(&h->reorder_map, B));
    acc(dmalloc(&h->draft_tok, rows)); acc(dmalloc(&h->draft_has, rows));
    acc(dmalloc(&h->draft_qid, rows * K)); acc(dmalloc(&h->draft_qmu, rows * K));
    acc(dmalloc(&h->draft_tok2, rows)); acc(dmalloc(&h->draft_has2, rows));
    acc(dmalloc(&h->draft_qid2, rows * K)); acc(dmalloc(&h->draft_qmu2, rows * K));
    acc(dmalloc(&h->row_pub, rows)); acc(dmalloc(&h->top_pub, rows * (size_t)K)); acc(dmalloc(&h->bar, 2));
    acc(dmalloc(&h->item_next, B)); acc(dmalloc(&h->path_flag, B));
    acc(dmalloc(&h->path_pub, B * kPathPub));
    acc(dmalloc(&h->vs.row_m, rows)); acc(dmalloc(&h->vs.row_s, rows));
    acc(dmalloc(&h->vs.top_l, rows * K)); acc(dmalloc(&h->vs.top_p, rows * K)); acc(dmalloc(&h->vs.top_idx, rows * K));
    acc(dmalloc(&h->vs.outcome, rows));
    acc(dmalloc(&h->vs.obs_idx, B * h->R * K)); acc(dmalloc(&h->vs.obs_p, B * h->R * K));
    acc(dmalloc(&h->rec_slot, nrec));
    acc(dmalloc(&h->vs.seg_part, B * h->R * kSegMax));
    acc(dmalloc(&h->recent, rows * kMaxOrder));
    acc(dmalloc(&h->node_count, (size_t)N));
    h->anc_words = (N + 63) / 64;
    acc(dmalloc(&h->anc, (size_t)N * h->anc_words));
    acc(dmalloc(&h->vs.stop_i, B * 4)); acc(dmalloc(&h->vs.stop_m, B)); acc(dmalloc(&h->vs.stop_qid, B * kMaxK));
    acc(dmalloc(&h->vs.stop_qmu, B * kMaxK)); acc(dmalloc(&h->vs.stop_ql, B * kMaxK)); acc(dmalloc(&h->vs.stop_child, B * kMaxK));
    acc(dmalloc(&h->pr_m, B * h->R)); acc(dmalloc(&h->pr_top_l, B * h->R * K)); acc(dmalloc(&h->pr_top_idx, B * h->R * K));
    acc(dmalloc(&h->stats, (size_t)kStatCount));
    acc(dmalloc(&h->counter, 1));
    if (e != hipSuccess) { free_all(h); return e == hipErrorOutOfMemory ? STAND_ENOMEM : STAND_EHIP; }

    std::vector<int32_t> tree(4 * (size_t)N + h->D + 2);
    std::copy(h->parent.begin(), h->parent.end(), tree.begin());
    std::copy(h->depth.begin(), h->depth.end(), tree.begin() + N);
    std::copy(h->nchild.begin(), h->nchild.end(), tree.begin() + 2 * N);
    std::copy(h->first_child.begin(), h->first_child.end(), tree.begin() + 3 * N);
    std::copy(h->level_start.begin(), h->level_start.end(), tree.begin() + 4 * N);
    acc(hipMemcpy(h->d_tree, tree.data(), tree.size() * sizeof(int32_t), hipMemcpyHostToDevice));
    acc(hipMemset(h->table, 0, (size_t)cfg->table_capacity * h->slot_bytes));
    acc(hipMemset(h->ctx_tail, 0, B * kMaxOrder * sizeof(int32_t)));
    acc(hipMemset(h->ctx_len, 0, B * sizeof(long long)));
    acc(hipMemset(h->draft_tok, 0xFF, rows * sizeof(int32_t)));
    acc(hipMemset(h->draft_has, 0, rows * sizeof(int32_t)));
    acc(hipMemset(h->draft_qid, 0, rows * K * sizeof(int32_t)));
    acc(hipMemset(h->draft_qmu, 0, rows * K * sizeof(float)));
    acc(hipMemset(h->draft_tok2, 0xFF, rows * sizeof(int32_t)));
    acc(hipMemset(h->draft_has2, 0, rows * sizeof(int32_t)));
    acc(hipMemset(h->draft_qid2, 0, rows * K * sizeof(int32_t)));
    acc(hipMemset(h->draft_qmu2, 0, rows * K * sizeof(float)));
    acc(hipMemset(h->row_pub, 0, rows * sizeof(unsigned long long)));
    acc(hipMemset(h->top_pub, 0, rows * (size_t)K * sizeof(unsigned long long)));
    acc(hipMemset(h->bar, 0, 2 * sizeof(unsigned)));
    acc(hipMemset(h->item_next, 0, B * sizeof(unsigned)));
    acc(hipMemset(h->path_flag, 0, B * sizeof(unsigned))); acc(hipMemset(h->path_pub, 0, B * kPathPub * sizeof(int32_t)));
    acc(hipMemset(h->vs.outcome, 0xFF, rows * sizeof(int32_t)));
    acc(hipMemset(h->node_count, 0, (size_t)N * sizeof(unsigned long long)));
    {
        // a node's set is its parent's set plus itself (parents come first in the numbering)
        std::vector<unsigned long long> anc((size_t)N * h->anc_words, 0ull);
        for (int u = 0; u < N; ++u) {
            if (u > 0)
                for (int q = 0; q < h->anc_words; ++q) anc[(size_t)u * h->anc_words + q] = anc[(size_t)cfg->tree_parent[u] * h->anc_words + q];
            anc[(size_t)u * h->anc_words + (u >> 6)] |= 1ull << (u & 63);
        }
        acc(hipMemcpy(h->anc, anc.data(), anc.size() * sizeof(unsigned long long), hipMemcpyHostToDevice));
    }
    acc(hipMemset(h->vs.row_m, 0, rows * sizeof(float))); acc(hipMemset(h->vs.row_s, 0, rows * sizeof(float)));
    acc(hipMemset(h->vs.top_l, 0, rows * K * sizeof(float))); acc(hipMemset(h->vs.top_p, 0, rows * K * sizeof(float)));
    acc(hipMemset(h->vs.top_idx, 0, rows * K * sizeof(int32_t)));
    acc(hipMemset(h->stats, 0, kStatCount * sizeof(unsigned long long)));
    acc(hipHostMalloc((void **)&h->probe_host, sizeof(unsigned long long), hipHostMallocDefault));
    if (h->probe_host) *h->probe_host = 0;
    acc(hipEventCreateWithFlags(&h->probe_ev, hipEventDisableTiming));
    acc(hipDeviceSynchronize());
    if (e != hipSuccess) { free_all(h); return STAND_EHIP; }
    *out = h;
    return STAND_OK;
}

extern "C" int stand_destroy(stand_handle *h)
{
    if (!h) return STAND_EINVAL;
    (void)hipSetDevice(h->cfg.device);
    (void)hipDeviceSynchronize();
    free_all(h);
    return STAND_OK;
}

extern "C" int stand_depth(const stand_handle *h) { return h ? h->D : STAND_EINVAL; }

static int drop_drafts(stand_handle *h, int b0, int nb, hipStream_t s)
{
    const size_t n = (size_t)nb * h->N;
    fill_i32_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s>>>(h->draft_tok + (size_t)b0 * h->N, -1, n);
    fill_i32_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s>>>(h->draft_has + (size_t)b0 * h->N, 0, n);
    HIP_TRY(h, hipGetLastError());
    return STAND_OK;
}

extern "C" int stand_set_context(stand_handle *h, int32_t b, const int32_t *host_tokens, int32_t n, void *stream)
{
    if (!h || b < 0 || b >= h->B || n < 0 || (n > 0 && !host_tokens)) return STAND_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    HIP_TRY(h, hipSetDevice(h->cfg.device));
    int32_t tail[kMaxOrder] = {0};
    for (int i = 0; i < kMaxOrder && i < n; ++i) tail[kMaxOrder - 1 - i] = host_tokens[n - 1 - i];
    long long len = n;
    HIP_TRY(h, hipMemcpyAsync(h->ctx_tail + (size_t)b * kMaxOrder, tail, sizeof(tail), hipMemcpyHostToDevice, s));
    HIP_TRY(h, hipMemcpyAsync(h->ctx_len + b, &len, sizeof(len), hipMemcpyHostToDevice, s));
    int rc = drop_drafts(h, b, 1, s);
    if (rc) return rc;
    HIP_TRY(h, hipStreamSynchronize(s));
    return STAND_OK;
}

extern "C" int stand_reorder(stand_handle *h, const int32_t *host_src_of, void *stream)
{
    if (!h || !host_src_of) return STAND_EINVAL;
    for (int b = 0; b < h->B; ++b) if (host_src_of[b] < 0 || host_src_of[b] >= h->B) return STAND_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    HIP_TRY(h, hipSetDevice(h->cfg.device));
    // the map goes to the device once (the copy from pageable memory is staged before the call returns);
    // one kernel gathers the contexts into the second pair of arrays, which then becomes the current one
    HIP_TRY(h, hipMemcpyAsync(h->reorder_map, host_src_of, (size_t)h->B * sizeof(int32_t), hipMemcpyHostToDevice, s));
    const int n = h->B * kMaxOrder;
    reorder_gather_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s>>>(h->B, h->reorder_map, h->ctx_tail, h->ctx_len,
                                                                                  h->ctx_tail2, h->ctx_len2);
    HIP_TRY(h, hipGetLastError());
    std::swap(h->ctx_tail, h->ctx_tail2);
    std::swap(h->ctx_len, h->ctx_len2);
    return drop_drafts(h, 0, h->B, s);
}

// ---- launches ----------------------------------------------------------------------------------
// Relative error assumed for the row pass's fast normaliser when `wpr` waves share a row: every lane adds
// ceil(vectors / (64 wpr)) vector sums of EPV terms in binary32, then lanes and waves are combined; each
// addition may lose 2^-24 of the running sum (the worst case, all roundings one way), doubled for the hardware
// exponential and the rescaling of partial sums.  Never below the caller's margin (default 5e-5).
static float fast_eps(const stand_handle *h, int wpr)
{
    const int epv = h->cfg.logits_dtype == STAND_BF16 ? 8 : 4;
    const double per_lane = std::ceil((double)h->V / epv / (64.0 * wpr)) + epv + 6 + wpr + 16;
    const double bound = 2.0 * per_lane * 5.9604644775390625e-08;
    return (float)std::max((double)h->filter_margin, bound);
}

static RowPassArgs make_row_args(const stand_handle *h, const VerifyScratch &vs, uint64_t step, const void *d_logits, int wpr)
{
    RowPassArgs a;
    a.logits = d_logits; a.B = h->B; a.N = h->N; a.V = h->V; a.K = h->K; a.c = h->c;
    a.seed = h->cfg.seed; a.step = step; a.tree = tree_dev(h);
    a.draft_tok = h->draft_tok; a.draft_has = h->draft_has; a.draft_qid = h->draft_qid; a.draft_qmu = h->draft_qmu;
    a.row_m = vs.row_m; a.row_s = vs.row_s; a.top_idx = vs.top_idx; a.top_l = vs.top_l; a.top_p = vs.top_p;
    a.outcome = vs.outcome; a.stats = h->stats;
    a.onehot = h->cfg.draft_mode == STAND_DRAFT_DETERMINISTIC;
    a.eps = fast_eps(h, wpr);
    a.fx_shift = h->fx_shift;
    return a;
}

static int launch_row_pass(stand_handle *h, const VerifyScratch &vs, uint64_t step, const void *d_logits, hipStream_t s)
{
    const int rows_all = h->B * h->N;
    RowPassArgs a = make_row_args(h, vs, step, d_logits, rows_all <= kRowsFew ? kRowWPRFewRows : kRowWPR);
    const int rows = h->B * h->N;
    const bool few = rows <= kRowsFew;  // one workgroup per row; more waves per row when rows are few
    const bool bf16 = h->cfg.logits_dtype == STAND_BF16;
    const dim3 grid((unsigned)rows), block(64u * (unsigned)(few ? kRowWPRFewRows : kRowWPR));
    const void *fn = bf16 ? (few ? (const void *)row_pass_kernel<kDtBf16, kRowWPRFewRows> : (const void *)row_pass_kernel<kDtBf16, kRowWPR>)
                          : (few ? (const void *)row_pass_kernel<kDtF32, kRowWPRFewRows> : (const void *)row_pass_kernel<kDtF32, kRowWPR>);
    void *args[] = {&a};
    const bool timed = h->profiling && h->ev_used < h->ev_begin.size();
    if (timed) {
        // the events are attached to the dispatch itself: their difference is the kernel's own
        // start-to-end time, without the marker packets a hipEventRecord pair would add
        hipEvent_t e0 = h->ev_begin[h->ev_used], e1 = h->ev_end[h->ev_used];
        h->ev_used++;
        HIP_TRY(h, hipExtLaunchKernel(fn, grid, block, args, 0, s, e0, e1, 0));
    } else {
        HIP_TRY(h, hipLaunchKernel(fn, grid, block, args, 0, s));
    }
    HIP_TRY(h, hipGetLastError());
    return STAND_OK;
}

static int clampi(int x, int lo, int hi) { return x < lo ? lo : (x > hi ? hi : x); }

static MergeArgs merge_args(stand_handle *h, const int32_t *commit_tok, const int32_t *commit_row, const int32_t *commit_len)
{
    MergeArgs a;
    a.table = h->table; a.mask = h->cfg.table_capacity - 1; a.slot_bytes = h->slot_bytes; a.K = h->K;
    a.max_probe = h->cfg.max_probe; a.B = h->B; a.W = h->W; a.omin = h->cfg.order_min; a.omax = h->cfg.order_max;
    a.R = h->R; a.all_nodes = h->cfg.update_mode == STAND_UPDATE_ALL_NODES; a.draft_tok = h->draft_tok;
    a.replace = h->cfg.merge_policy == STAND_MERGE_REPLACE;
    a.depth = tree_dev(h).depth; a.recent = h->recent;
    a.ctx_tail = h->ctx_tail; a.ctx_len = h->ctx_len; a.commit_tok = commit_tok; a.commit_row = commit_row;
    a.commit_len = commit_len; a.N = h->N; a.rec_slot = h->rec_slot; a.obs_idx = h->vs.obs_idx; a.obs_p = h->vs.obs_p;
    a.stats = h->stats;
    return a;
}

static PathArgs make_path_args(const stand_handle *h, const VerifyScratch &vs, uint64_t step, const void *d_logits, int mode,
                               const int32_t *commit_row, const int32_t *commit_len, int32_t *out_tok, int32_t *out_node,
                               int32_t *out_len, int seg_vectors)
{
    const bool bf16 = h->cfg.logits_dtype == STAND_BF16;
    PathArgs a;
    a.logits = d_logits; a.B = h->B; a.N = h->N; a.V = h->V; a.K = h->K; a.W = h->W; a.mode = mode; a.c = h->c;
    a.R = h->R; a.all_nodes = h->cfg.update_mode == STAND_UPDATE_ALL_NODES;
    a.seed = h->cfg.seed; a.step = step; a.tree = tree_dev(h);
    a.draft_tok = h->draft_tok; a.draft_has = h->draft_has; a.draft_qid = h->draft_qid; a.draft_qmu = h->draft_qmu;
    a.src_m = mode == 0 ? vs.row_m : h->pr_m;
    a.src_top_idx = mode == 0 ? vs.top_idx : h->pr_top_idx;
    a.src_top_l = mode == 0 ? vs.top_l : h->pr_top_l;
    a.outcome = vs.outcome; a.commit_row = commit_row; a.commit_len = commit_len;
    a.out_tok = out_tok; a.out_node = out_node; a.out_len = out_len;
    a.seg_part = vs.seg_part; a.node_count = h->node_count;
    a.onehot = h->cfg.draft_mode == STAND_DRAFT_DETERMINISTIC;
    a.stop_i = vs.stop_i; a.stop_m = vs.stop_m; a.stop_qid = vs.stop_qid; a.stop_qmu = vs.stop_qmu; a.stop_ql = vs.stop_ql;
    a.stop_child = vs.stop_child;
    a.obs_idx = vs.obs_idx; a.obs_p = vs.obs_p; a.stats = h->stats;
    a.late_len = (h->upper_depth < h->D ? h->upper_depth : h->D) + 1;
    a.fx_shift = h->fx_shift;
    a.top_pub = nullptr;
    // segments of seg_vectors 16-byte vectors where kSegMax allows it
    const int row_vectors = (int)(((size_t)h->V * (bf16 ? 2 : 4) + 15) / 16);
    a.nseg = clampi((row_vectors + seg_vectors - 1) / seg_vectors, 1, kSegMax);
    return a;
}

// mode 0 (verify): path from the row pass's outcomes; mode 1 (update): rows given by the caller.
// With `claim` the launch that finishes the path rows also claims the table slots of that merge.
static int launch_path_pass(stand_handle *h, const VerifyScratch &vs, uint64_t step, const void *d_logits, int mode, const int32_t *commit_row,
                            const int32_t *commit_len, int32_t *out_tok, int32_t *out_node, int32_t *out_len,
                            const MergeArgs *claim, hipStream_t s)
{
    const bool bf16 = h->cfg.logits_dtype == STAND_BF16;
    if (mode == 1) {
        CommitScanArgs c;
        c.logits = d_logits; c.B = h->B; c.N = h->N; c.V = h->V; c.K = h->K; c.W = h->W; c.c = h->c;
        c.R = h->R; c.all_nodes = h->cfg.update_mode == STAND_UPDATE_ALL_NODES; c.draft_tok = h->draft_tok;
        c.commit_row = commit_row; c.commit_len = commit_len;
        c.pr_m = h->pr_m; c.pr_top_idx = h->pr_top_idx; c.pr_top_l = h->pr_top_l;
        const dim3 grid((unsigned)h->R, (unsigned)h->B);
        if (bf16) commit_scan_kernel<kDtBf16><<<grid, dim3(256), 0, s>>>(c);
        else commit_scan_kernel<kDtF32><<<grid, dim3(256), 0, s>>>(c);
    }
    // segments: one round of loads per thread (4 vectors of 16 bytes) where kSegMax allows it;
    // one more block per (row, trajectory) slot for the outputs and the stop record
    PathArgs a = make_path_args(h, vs, step, d_logits, mode, commit_row, commit_len, out_tok, out_node, out_len, 4 * kPathThreads);
    // row slots of the grid: every slot in update / all-nodes mode; in verify mode three (paths are
    // mostly short; the kernel loops over longer ones)
    const int row_slots = (mode == 0 && !a.all_nodes) ? (h->R < 3 ? h->R : 3) : h->R;
    const dim3 g1((unsigned)a.nseg + 1, (unsigned)h->B, (unsigned)row_slots), block(kPathThreads);
    const int finish_blocks = h->B * h->R;
    const int claim_blocks = claim ? (h->B * h->R * h->NO + kFinishThreads - 1) / kFinishThreads : 0;
    const MergeArgs mg = claim ? *claim : merge_args(h, nullptr, nullptr, nullptr);
    const dim3 g2((unsigned)(finish_blocks + claim_blocks));
    if (bf16) {
        path_exact_kernel<kDtBf16><<<g1, block, 0, s>>>(a);
        path_finish_kernel<kDtBf16><<<g2, dim3(kFinishThreads), 0, s>>>(a, mg, finish_blocks);
    } else {
        path_exact_kernel<kDtF32><<<g1, block, 0, s>>>(a);
        path_finish_kernel<kDtF32><<<g2, dim3(kFinishThreads), 0, s>>>(a, mg, finish_blocks);
    }
    HIP_TRY(h, hipGetLastError());
    return STAND_OK;
}

// applies the records whose slots the path pass claimed
static int launch_merge_apply(stand_handle *h, const MergeArgs &a, bool append_ctx, hipStream_t s)
{
    const int nrec = h->B * h->R * h->NO;
    merge_apply_kernel<<<dim3((unsigned)((nrec + kMergeWaves - 1) / kMergeWaves)), dim3(64 * kMergeWaves), 0, s>>>(a);
    if (append_ctx)
        ctx_append_kernel<<<dim3((unsigned)((h->B + 63) / 64)), dim3(64), 0, s>>>(h->B, h->W, h->ctx_tail, h->ctx_len,
                                                                                a.commit_tok, a.commit_len);
    HIP_TRY(h, hipGetLastError());
    h->table_used = true;
    return STAND_OK;
}

static DraftArgs make_draft_args(const stand_handle *h, uint64_t step, int32_t *d_draft_tok, const int32_t *append_tok,
                                 const int32_t *append_len)
{
    DraftArgs a;
    a.table = h->table; a.mask = h->cfg.table_capacity - 1; a.slot_bytes = h->slot_bytes; a.K = h->K;
    a.max_probe = h->cfg.max_probe; a.B = h->B; a.W = h->W; a.omin = h->cfg.order_min; a.omax = h->cfg.order_max;
    a.seed = h->cfg.seed; a.step = step; a.tree = tree_dev(h);
    a.ctx_tail = h->ctx_tail; a.ctx_len = h->ctx_len; a.append_tok = append_tok; a.append_len = append_len;
    a.draft_tok = h->draft_tok; a.draft_has = h->draft_has; a.draft_qid = h->draft_qid; a.draft_qmu = h->draft_qmu;
    a.out_tok = d_draft_tok; a.stats = h->stats; a.mode = h->cfg.draft_mode;
    a.recent_out = h->cfg.update_mode == STAND_UPDATE_ALL_NODES ? h->recent : nullptr;
    return a;
}

static int launch_draft(stand_handle *h, uint64_t step, int32_t *d_draft_tok, const int32_t *append_tok,
                        const int32_t *append_len, hipStream_t s)
{
    DraftArgs a = make_draft_args(h, step, d_draft_tok, append_tok, append_len);
    draft_kernel<<<dim3((unsigned)h->B), dim3(kDraftThreads), 0, s>>>(a);
    HIP_TRY(h, hipGetLastError());
    return STAND_OK;
}

extern "C" int stand_update(stand_handle *h, uint64_t step, const void *d_logits, const int32_t *d_commit_tok,
                            const int32_t *d_commit_row, const int32_t *d_commit_len, void *stream)
{
    if (!h || !d_logits || !d_commit_tok || !d_commit_row || !d_commit_len) return STAND_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    HIP_TRY(h, hipSetDevice(h->cfg.device));
    const MergeArgs mg = merge_args(h, d_commit_tok, d_commit_row, d_commit_len);
    int rc = launch_path_pass(h, h->vs, step, d_logits, 1, d_commit_row, d_commit_len, nullptr, nullptr, nullptr, &mg, s);
    if (rc) return rc;
    return launch_merge_apply(h, mg, true, s);
}

extern "C" int stand_draft(stand_handle *h, uint64_t step, int32_t *d_draft_tok, void *stream)
{
    if (!h) return STAND_EINVAL;
    HIP_TRY(h, hipSetDevice(h->cfg.device));
    return launch_draft(h, step, d_draft_tok, nullptr, nullptr, (hipStream_t)stream);
}

extern "C" int stand_tree_packing(stand_handle *h, uint8_t *d_mask, int64_t *d_pos, void *stream)
{
    if (!h || !d_mask || !d_pos) return STAND_EINVAL;
    HIP_TRY(h, hipSetDevice(h->cfg.device));
    const int items = h->N * ((h->N + 7) / 8);
    const dim3 grid((unsigned)((items + 255) / 256), (unsigned)h->B);
    tree_packing_kernel<<<grid, dim3(256), 0, (hipStream_t)stream>>>(h->B, h->N, h->anc_words, h->anc, tree_dev(h).depth,
                                                                     h->draft_tok, h->ctx_len, d_mask, (long long *)d_pos);
    HIP_TRY(h, hipGetLastError());
    return STAND_OK;
}

extern "C" int stand_verify(stand_handle *h, uint64_t step, const void *d_logits, int32_t *d_out_tok, int32_t *d_out_node,
                            int32_t *d_out_len, void *stream)
{
    if (!h || !d_logits || !d_out_tok || !d_out_node || !d_out_len) return STAND_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    HIP_TRY(h, hipSetDevice(h->cfg.device));
    int rc = launch_row_pass(h, h->vs, step, d_logits, s);
    if (rc) return rc;
    return launch_path_pass(h, h->vs, step, d_logits, 0, nullptr, nullptr, d_out_tok, d_out_node, d_out_len, nullptr, s);
}

// Bytes of scratch a verification of this handle's shape needs, laid out as carve_scratch does.
static size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }
static size_t carve_scratch(const stand_handle *h, unsigned char *base, VerifyScratch *out)
{
    const size_t B = h->B, rows = B * h->N, K = h->K, R = h->R;
    size_t off = 0;
    auto take = [&](size_t bytes) { unsigned char *p = base ? base + off : nullptr; off += align256(bytes); return p; };
    VerifyScratch v;
    v.row_m = (float *)take(rows * 4); v.row_s = (float *)take(rows * 4);
    v.top_l = (float *)take(rows * K * 4); v.top_p = (float *)take(rows * K * 4);
    v.top_idx = (int32_t *)take(rows * K * 4); v.outcome = (int32_t *)take(rows * 4);
    v.obs_idx = (int32_t *)take(B * R * K * 4); v.obs_p = (float *)take(B * R * K * 4);
    v.seg_part = (unsigned long long *)take(B * R * kSegMax * 8);
    v.stop_i = (int32_t *)take(B * 4 * 4); v.stop_qid = (int32_t *)take(B * kMaxK * 4);
    v.stop_child = (int32_t *)take(B * kMaxK * 4); v.stop_m = (float *)take(B * 4);
    v.stop_qmu = (float *)take(B * kMaxK * 4); v.stop_ql = (float *)take(B * kMaxK * 4);
    if (out) *out = v;
    return off;
}

extern "C" int stand_verify_static(stand_handle *h, uint64_t step, const void *d_logits, int32_t *d_out_tok,
                                   int32_t *d_out_node, int32_t *d_out_len, void *stream)
{
    if (!h || !d_logits || !d_out_tok || !d_out_node || !d_out_len) return STAND_EINVAL;
    if (carve_scratch(h, nullptr, nullptr) > (size_t)STAND_STATIC_SCRATCH_BYTES) return STAND_ELIMIT;
    hipStream_t s = (hipStream_t)stream;
    HIP_TRY(h, hipSetDevice(h->cfg.device));
    void *base = nullptr;
    HIP_TRY(h, static_scratch_ptr(h->cfg.device, &base));  // resolved by stand_create already; no allocation
    VerifyScratch vs;
    carve_scratch(h, (unsigned char *)base, &vs);
    // Nothing in the scratch has to start at zero: every word a kernel of the verification reads was written
    // by an earlier kernel of the same call (row results and outcomes for all rows; partial sums, stop records
    // and observations for exactly the path rows that are read back).
    int rc = launch_row_pass(h, vs, step, d_logits, s);
    if (rc) return rc;
    return launch_path_pass(h, vs, step, d_logits, 0, nullptr, nullptr, d_out_tok, d_out_node, d_out_len, nullptr, s);
}

extern "C" uint64_t stand_static_scratch_need(const stand_handle *h)
{
    return h ? (uint64_t)carve_scratch(h, nullptr, nullptr) : 0;
}

// The whole step in one launch (step_fused.hpp).
// Whether the one launch is among the choices at all (whatever the acceptance depth at present).
static bool step_fused_possible(const stand_handle *h)
{
    if (h->cfg.update_mode != STAND_UPDATE_ACCEPTED_PATH) return false;
    if (h->step_mode == STAND_STEP_SERIAL) return false;
    // the tail's workgroups wait inside the launch for rows that may be dispatched after them: they must
    // never hold more than a fraction of the device (256 compute units, three such workgroups each)
    if (h->B * (h->tail_groups > 0 ? h->tail_groups : 1) > 256) return false;
    if (h->step_mode == STAND_STEP_FUSED) return true;
    // With few rows the pass is latency-bound and sixteen waves per row serve it better.  With very many the
    // dependent launches are a few per cent of the step, which is all one launch could save, and it varied more
    // from run to run than that (B=128 x 128 nodes: 0.84-0.96 ms against 0.85-0.88 ms).
    return h->B * h->N > kRowsFew && h->B * h->N <= kRowsMany;
}
static bool step_fused_wanted(const stand_handle *h)
{
    if (!step_fused_possible(h)) return false;
    // (automatic plan: not while deep accepted paths are common, see plan_observe)
    return h->step_mode == STAND_STEP_FUSED || !h->plan_serial;
}

// STAND_STEP_AUTO only.  In the one-launch step a trajectory whose accepted path reaches below the tree
// levels scheduled first waits for a row that streams late, and everything after the first barrier waits
// with it; the separate launches do not care.  Both kinds of step count such paths (kStatLatePaths).
// Every kPlanWindow steps the counter is copied to pinned memory without waiting; when a copy has arrived,
// the late paths per step over the window it closed decide the plan: above kPlanSerialAbove the separate
// launches, below kPlanFusedBelow the one launch again.  Results do not depend on the plan.  Nothing is
// observed while the stream is being captured.
constexpr uint64_t kPlanWindow = 32;
constexpr double kPlanSerialAbove = 0.40, kPlanFusedBelow = 0.25;
static void plan_observe(stand_handle *h, hipStream_t s, bool capturing)
{
    if (h->step_mode != STAND_STEP_AUTO || !h->probe_host || !h->probe_ev || capturing) return;
    if (!step_fused_possible(h)) return;  // nothing to decide where the one launch is not among the choices
    ++h->probe_steps;
    if (h->probe_pending) {
        if (hipEventQuery(h->probe_ev) != hipSuccess) { (void)hipGetLastError(); return; }  // (not there yet)
        h->probe_pending = false;
        const uint64_t late = *(volatile unsigned long long *)h->probe_host;
        const uint64_t steps = h->probe_issue_steps - h->probe_base_steps;
        if (steps > 0 && late >= h->probe_base_late) {
            const double per_step = (double)(late - h->probe_base_late) / (double)steps;
            if (per_step > kPlanSerialAbove) h->plan_serial = true;
            else if (per_step < kPlanFusedBelow) h->plan_serial = false;
        }
        h->probe_base_steps = h->probe_issue_steps; h->probe_base_late = late;
    }
    if (h->probe_steps - h->probe_issue_steps >= kPlanWindow) {
        // (the copy is ordered after the steps enqueued so far: it sees the count up to the step before this one)
        if (hipMemcpyAsync(h->probe_host, h->stats + kStatLatePaths, sizeof(unsigned long long), hipMemcpyDeviceToHost, s) == hipSuccess &&
            hipEventRecord(h->probe_ev, s) == hipSuccess) {
            h->probe_pending = true;
            h->probe_issue_steps = h->probe_steps - 1;
        } else {
            (void)hipGetLastError();
        }
    }
}
static int step_tail_groups(const stand_handle *h)
{
    // (three against four at B = 32: 0.1239-0.1245 against 0.1247-0.1252 ms per step; two: 0.1263)
    return h->tail_groups > 0 ? h->tail_groups : (h->B <= 32 ? 3 : (h->B <= 64 ? 2 : 1));
}

static uint32_t gcd_u32(uint32_t a, uint32_t b) { while (b) { const uint32_t t = a % b; a = b; b = t; } return a; }

static int launch_step_fused(stand_handle *h, uint64_t step, const void *d_logits, int32_t *out_tok, int32_t *out_node,
                             int32_t *out_len, int32_t *next_draft_tok, const int32_t *commit, hipStream_t s)
{
    const bool bf16 = h->cfg.logits_dtype == STAND_BF16;
    StepArgs A;
    A.row = make_row_args(h, h->vs, step, d_logits, kStepWPR);
    A.G = step_tail_groups(h);
    // one wave sums one segment: a few rounds of loads per lane; a row has at most as many segments as the
    // trajectory has summing waves (all waves of its tail workgroups but one)
    A.path = make_path_args(h, h->vs, step, d_logits, 0, nullptr, nullptr, out_tok, out_node, out_len, 4 * 64 * 2);
    if (A.path.nseg > A.G * kStepWPR - 1) A.path.nseg = A.G * kStepWPR - 1;
    A.mg = merge_args(h, commit, nullptr, out_len);
    A.draft = make_draft_args(h, step + 1, next_draft_tok, commit, out_len);
    // the next draft goes to the second copy of the draft state; the copies change roles after the launch
    A.draft.draft_tok = h->draft_tok2; A.draft.draft_has = h->draft_has2;
    A.draft.draft_qid = h->draft_qid2; A.draft.draft_qmu = h->draft_qmu2;
    A.sync.bar = h->bar;
    A.sync.item_next = h->item_next; A.sync.path_flag = h->path_flag;
    A.sync.path_pub = h->path_pub;
    A.sync.epoch = h->step_epoch + 1;  // (taken only once the launch has been accepted: the rows' published words rely on
                                        // consecutive numbers, see RowPub)
    A.sync.pub = RowPub{h->row_pub, h->top_pub, A.sync.epoch};
    A.path.top_pub = h->top_pub;
    A.sync.wait_ticks = h->wait_limit_us * (uint64_t)h->wall_khz / 1000ull;
    A.sync.stamps = h->stamps;
    if (h->stamps) {
        // earliest start: all ones, latest end: zero (set by a fill kernel; the launch stays capturable)
        fill_i32_kernel<<<dim3(1), dim3(64), 0, s>>>((int32_t *)h->stamps, -1, 2);
        fill_i32_kernel<<<dim3(1), dim3(64), 0, s>>>((int32_t *)(h->stamps + 1), 0, 2);
    }
    const int ud = h->upper_depth < h->D ? h->upper_depth : h->D;
    A.upper_nodes = h->level_start[ud + 1];
    const void *fn = bf16 ? (const void *)stand_step_kernel<kDtBf16> : (const void *)stand_step_kernel<kDtF32>;
    const size_t smem = step_shared_bytes(h->N, h->D);
    if (h->step_slots == 0) {
        // how many of the kernel's workgroups are resident at once: the rows before the tail fill the device once
        int per_cu = 0, cus = 0;
        HIP_TRY(h, hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, kStepThreads, smem));
        HIP_TRY(h, hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, h->cfg.device));
        h->step_slots = per_cu * cus > 0 ? per_cu * cus : 1;
    }
    const uint32_t rows = (uint32_t)(h->B * h->N), n_up = (uint32_t)(A.upper_nodes * h->B);
    A.shuffle_mul = 1; A.shuffle_add = 0;
    if (h->shuffle) {
        // a multiplier coprime with both group sizes permutes the slots of each group
        uint32_t mul = (h->shuffle * 2654435761u) | 1u;
        mul = mul % 1000003u + 2u;
        while (gcd_u32(mul, n_up ? n_up : 1u) != 1u || gcd_u32(mul, rows - n_up ? rows - n_up : 1u) != 1u) ++mul;
        A.shuffle_mul = mul; A.shuffle_add = h->shuffle;
    }
    const uint32_t row_wgs = rows;  // one row per workgroup
    {
        // By default the rows before the tail leave room, in the first device-full of workgroups, for the first
        // two tail workgroups of every trajectory: those are resident from the start and follow the path the moment
        // the root rows publish (they wait in place meanwhile, which costs less than their later start would:
        // 126.5 against 129.8 us per step at B = 32, 64 nodes); the other tail workgroups take the slots the first
        // rows free.  Never fewer rows than the upper levels have.
        const uint32_t early = (uint32_t)h->B * (uint32_t)(A.G < 2 ? A.G : 2);
        const uint32_t deflt = (uint32_t)h->step_slots > early ? (uint32_t)h->step_slots - early : 1u;
        const uint32_t want = h->rows_first > 0 ? (uint32_t)h->rows_first : deflt;
        const uint32_t first = want > n_up ? want : n_up;
        A.rows_first = (int)(first < row_wgs ? first : row_wgs);
    }
#ifdef STAND_DEBUG_NO_TAIL
    A.G = 0;
#endif
    const dim3 grid(row_wgs + (uint32_t)(h->B * A.G)), block(kStepThreads);
    void *args[] = {&A};
    const bool timed = h->profiling && h->ev_used < h->ev_begin.size();
    if (timed) {
        hipEvent_t e0 = h->ev_begin[h->ev_used], e1 = h->ev_end[h->ev_used];
        h->ev_used++;
        HIP_TRY(h, hipExtLaunchKernel(fn, grid, block, args, smem, s, e0, e1, 0));
    } else {
        HIP_TRY(h, hipLaunchKernel(fn, grid, block, args, smem, s));
    }
    HIP_TRY(h, hipGetLastError());
    h->step_epoch = A.sync.epoch;
    std::swap(h->draft_tok, h->draft_tok2); std::swap(h->draft_has, h->draft_has2);
    std::swap(h->draft_qid, h->draft_qid2); std::swap(h->draft_qmu, h->draft_qmu2);
    h->table_used = true;
    return STAND_OK;
}

extern "C" int stand_set_step_plan(stand_handle *h, int32_t mode, int32_t upper_depth, int32_t tail_groups, int32_t rows_first,
                                   uint32_t shuffle)
{
    if (!h || mode < STAND_STEP_AUTO || mode > STAND_STEP_FUSED || upper_depth < 0 || upper_depth > STAND_MAX_DEPTH ||
        tail_groups < 0 || tail_groups > 8 || rows_first < 0)
        return STAND_EINVAL;
    if (mode == STAND_STEP_FUSED && h->cfg.update_mode != STAND_UPDATE_ACCEPTED_PATH) return STAND_EINVAL;
    h->step_mode = mode; h->upper_depth = upper_depth; h->tail_groups = tail_groups; h->rows_first = rows_first;
    h->shuffle = shuffle;
    h->plan_serial = false;  // (a new plan starts from the one launch; the window in progress is kept)
    return STAND_OK;
}

extern "C" int stand_step_timeline(stand_handle *h, int32_t enable, uint64_t *host_ticks, uint64_t *ticks_per_second)
{
    if (!h) return STAND_EINVAL;
    HIP_TRY(h, hipSetDevice(h->cfg.device));
    if (ticks_per_second) *ticks_per_second = (uint64_t)h->wall_khz * 1000ull;
    const size_t n = 2 + 8 * (size_t)h->B;
    if (host_ticks && h->stamps) {
        HIP_TRY(h, hipDeviceSynchronize());
        HIP_TRY(h, hipMemcpy(host_ticks, h->stamps, n * sizeof(uint64_t), hipMemcpyDeviceToHost));
    } else if (host_ticks) {
        return STAND_ESTATE;
    }
    if (enable && !h->stamps) {
        HIP_TRY(h, hipDeviceSynchronize());
        HIP_TRY(h, dmalloc(&h->stamps, n));
        HIP_TRY(h, hipMemset(h->stamps, 0, n * sizeof(uint64_t)));
    } else if (!enable && h->stamps) {
        HIP_TRY(h, hipDeviceSynchronize());
        (void)hipFree(h->stamps);
        h->stamps = nullptr;
    }
    return STAND_OK;
}

extern "C" int stand_step_is_one_launch(const stand_handle *h) { return h ? (step_fused_wanted(h) ? 1 : 0) : STAND_EINVAL; }

extern "C" int stand_set_wait_limit(stand_handle *h, uint64_t microseconds)
{
    if (!h || microseconds > 60ull * 1000 * 1000) return STAND_EINVAL;
    h->wait_limit_us = microseconds;
    return STAND_OK;
}

extern "C" int stand_step(stand_handle *h, uint64_t step, const void *d_logits, int32_t *d_out_tok, int32_t *d_out_node,
                          int32_t *d_out_len, int32_t *d_next_draft_tok, const int32_t *d_force_tok, void *stream)
{
    if (!h || !d_logits || !d_out_tok || !d_out_node || !d_out_len) return STAND_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    HIP_TRY(h, hipSetDevice(h->cfg.device));
    const int32_t *commit = d_force_tok ? d_force_tok : d_out_tok;
    // The one launch numbers itself (its waits and the words its rows publish carry the launch's number, given as
    // a kernel argument): recorded into a graph it would be replayed with a number that has passed.  While the
    // stream is being captured the separate launches are taken, whatever the plan says; they replay correctly.
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(s, &cap) != hipSuccess) { (void)hipGetLastError(); cap = hipStreamCaptureStatusNone; }
    const bool capturing = cap != hipStreamCaptureStatusNone;
    plan_observe(h, s, capturing);
    if (!capturing && step_fused_wanted(h))
        return launch_step_fused(h, step, d_logits, d_out_tok, d_out_node, d_out_len, d_next_draft_tok, commit, s);
    int rc = launch_row_pass(h, h->vs, step, d_logits, s);
    if (rc) return rc;
    const MergeArgs mg = merge_args(h, commit, nullptr, d_out_len);
    rc = launch_path_pass(h, h->vs, step, d_logits, 0, nullptr, nullptr, d_out_tok, d_out_node, d_out_len, &mg, s);
    if (rc) return rc;
    rc = launch_merge_apply(h, mg, false, s);
    if (rc) return rc;
    // the draft kernel appends the committed tokens to the contexts before it looks anything up
    return launch_draft(h, step + 1, d_next_draft_tok, commit, d_out_len, s);
}

extern "C" int stand_row_results(stand_handle *h, float *d_row_max, float *d_row_sum, int32_t *d_top_idx, float *d_top_p,
                                 void *stream)
{
    if (!h) return STAND_EINVAL;
    HIP_TRY(h, hipSetDevice(h->cfg.device));
    const size_t n = (size_t)h->B * h->N * h->K;
    copy_row_results_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)stream>>>(
        h->B * h->N, h->K, h->vs.row_m, h->vs.row_s, h->vs.top_idx, h->vs.top_p, d_row_max, d_row_sum, d_top_idx, d_top_p);
    HIP_TRY(h, hipGetLastError());
    return STAND_OK;
}

extern "C" int stand_table_export(stand_handle *h, void *host_buf, uint64_t *inout_bytes)
{
    if (!h || !inout_bytes) return STAND_EINVAL;
    HIP_TRY(h, hipSetDevice(h->cfg.device));
    HIP_TRY(h, hipDeviceSynchronize());
    const uint64_t cap = h->cfg.table_capacity;
    const unsigned blocks = (unsigned)((cap + 255) / 256);
    unsigned long long n = 0;
    HIP_TRY(h, hipMemset(h->counter, 0, sizeof(unsigned long long)));
    table_compact_kernel<<<dim3(blocks), dim3(256)>>>(h->table, cap, h->slot_bytes, h->counter, nullptr, 0);
    HIP_TRY(h, hipGetLastError());
    HIP_TRY(h, hipMemcpy(&n, h->counter, sizeof(n), hipMemcpyDeviceToHost));
    const uint64_t need = n * (uint64_t)h->slot_bytes;
    const uint64_t have = *inout_bytes;
    *inout_bytes = need;
    if (!host_buf) return STAND_OK;
    if (have < need) return STAND_EINVAL;
    if (n == 0) return STAND_OK;
    // the compacted copy goes to a buffer the handle keeps (it grows when a later export needs more)
    if (h->export_cap < need) {
        if (h->export_buf) (void)hipFree(h->export_buf);
        h->export_buf = nullptr; h->export_cap = 0;
        HIP_TRY(h, hipMalloc((void **)&h->export_buf, need));
        h->export_cap = need;
    }
    char *dbuf = h->export_buf;
    hipError_t e = hipMemset(h->counter, 0, sizeof(unsigned long long));
    if (e == hipSuccess) {
        table_compact_kernel<<<dim3(blocks), dim3(256)>>>(h->table, cap, h->slot_bytes, h->counter, dbuf, n);
        e = hipGetLastError();
    }
    std::vector<char> tmp(need);
    if (e == hipSuccess) e = hipMemcpy(tmp.data(), dbuf, need, hipMemcpyDeviceToHost);
    HIP_TRY(h, e);
    std::vector<uint64_t> order(n);
    for (uint64_t i = 0; i < n; ++i) order[i] = i;
    const int sb = h->slot_bytes;
    std::sort(order.begin(), order.end(), [&](uint64_t x, uint64_t y) {
        uint64_t fx, fy;
        memcpy(&fx, tmp.data() + x * sb, 8);
        memcpy(&fy, tmp.data() + y * sb, 8);
        return fx < fy;
    });
    for (uint64_t i = 0; i < n; ++i) memcpy((char *)host_buf + i * sb, tmp.data() + order[i] * sb, sb);
    return STAND_OK;
}

extern "C" int stand_table_import(stand_handle *h, const void *host_buf, uint64_t bytes)
{
    if (!h || (!host_buf && bytes) || bytes % (uint64_t)h->slot_bytes) return STAND_EINVAL;
    if (h->table_used) return STAND_ESTATE;
    HIP_TRY(h, hipSetDevice(h->cfg.device));
    const uint64_t n = bytes / h->slot_bytes, cap = h->cfg.table_capacity, mask = cap - 1;
    const int sb = h->slot_bytes, K = h->K;
    if (n > cap) return STAND_EINVAL;
    // place the entries on the host exactly as the device would (linear probing), then upload
    std::vector<char> img;
    try { img.assign((size_t)cap * sb, 0); } catch (...) { return STAND_ENOMEM; }
    for (uint64_t i = 0; i < n; ++i) {
        const char *src = (const char *)host_buf + i * sb;
        uint64_t fp; uint32_t count, order;
        memcpy(&fp, src, 8); memcpy(&count, src + 8, 4); memcpy(&order, src + 12, 4);
        if (fp == 0 || count == 0 || order < 1 || order > STAND_MAX_ORDER) return STAND_EINVAL;
        for (int q = 0; q < K; ++q) {
            int32_t id; memcpy(&id, src + 16 + 4 * q, 4);
            if (id < 0 || id >= h->V) return STAND_EINVAL;
        }
        bool placed = false;
        for (int p = 0; p < h->cfg.max_probe && !placed; ++p) {
            char *dst = img.data() + ((fp + (uint64_t)p) & mask) * sb;
            uint64_t cur; memcpy(&cur, dst, 8);
            if (cur == fp) return STAND_EINVAL;  // duplicate key
            if (cur == 0) { memcpy(dst, src, sb); placed = true; }
        }
        if (!placed) return STAND_EINVAL;
    }
    HIP_TRY(h, hipMemcpy(h->table, img.data(), img.size(), hipMemcpyHostToDevice));
    h->table_used = true;
    return STAND_OK;
}

extern "C" int stand_get_context(stand_handle *h, int32_t b, int32_t *host_tail, int32_t n, int64_t *len_out, void *stream)
{
    if (!h || b < 0 || b >= h->B || n < 0 || n > kMaxOrder || (n > 0 && !host_tail)) return STAND_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    HIP_TRY(h, hipSetDevice(h->cfg.device));
    int32_t tail[kMaxOrder];
    long long len = 0;
    HIP_TRY(h, hipMemcpyAsync(tail, h->ctx_tail + (size_t)b * kMaxOrder, sizeof(tail), hipMemcpyDeviceToHost, s));
    HIP_TRY(h, hipMemcpyAsync(&len, h->ctx_len + b, sizeof(len), hipMemcpyDeviceToHost, s));
    HIP_TRY(h, hipStreamSynchronize(s));
    for (int i = 0; i < n; ++i) host_tail[i] = tail[kMaxOrder - n + i];
    if (len_out) *len_out = len;
    return STAND_OK;
}

extern "C" int stand_get_stats(stand_handle *h, stand_stats *out)
{
    if (!h || !out) return STAND_EINVAL;
    HIP_TRY(h, hipSetDevice(h->cfg.device));
    HIP_TRY(h, hipDeviceSynchronize());
    unsigned long long st[kStatCount];
    HIP_TRY(h, hipMemcpy(st, h->stats, sizeof(st), hipMemcpyDeviceToHost));
    memset(out, 0, sizeof(*out));
    for (int n = 0; n <= STAND_MAX_ORDER; ++n) out->hits[n] = st[kStatHits + n];
    out->misses = st[kStatMisses]; out->inserts = st[kStatInserts]; out->merges = st[kStatMerges];
    out->drops = st[kStatDrops]; out->near_threshold = st[kStatNear]; out->tokens_emitted = st[kStatTokens];
    out->accept_tests = st[kStatTests]; out->filter_mismatch = st[kStatMismatch];
    out->wait_expired = st[kStatWaitExpired]; out->late_paths = st[kStatLatePaths];
    return STAND_OK;
}

extern "C" int stand_set_filter_margin(stand_handle *h, float margin)
{
    if (!h || !(margin >= kFastEps) || !(margin <= 1.0f)) return STAND_EINVAL;
    h->filter_margin = margin;
    return STAND_OK;
}

extern "C" int stand_profile_begin(stand_handle *h, int32_t max_launches)
{
    if (!h || max_launches < 0 || max_launches > (1 << 20)) return STAND_EINVAL;
    HIP_TRY(h, hipSetDevice(h->cfg.device));
    while ((int32_t)h->ev_begin.size() < max_launches) {
        hipEvent_t a, b;
        HIP_TRY(h, hipEventCreate(&a));
        h->ev_begin.push_back(a);
        HIP_TRY(h, hipEventCreate(&b));
        h->ev_end.push_back(b);
    }
    h->ev_used = 0;
    h->profiling = max_launches > 0;
    return STAND_OK;
}

extern "C" int stand_profile_end(stand_handle *h, double *row_pass_ms_total, int32_t *launches)
{
    if (!h || !row_pass_ms_total || !launches) return STAND_EINVAL;
    HIP_TRY(h, hipSetDevice(h->cfg.device));
    HIP_TRY(h, hipDeviceSynchronize());
    double total = 0.0;
    for (size_t i = 0; i < h->ev_used; ++i) {
        float ms = 0.0f;
        HIP_TRY(h, hipEventElapsedTime(&ms, h->ev_begin[i], h->ev_end[i]));
        total += (double)ms;
    }
    *row_pass_ms_total = total;
    *launches = (int32_t)h->ev_used;
    h->profiling = false;
    h->ev_used = 0;
    return STAND_OK;
}

extern "C" int stand_get_record_slots(stand_handle *h, int64_t *host_slots)
{
    if (!h || !host_slots) return STAND_EINVAL;
    HIP_TRY(h, hipSetDevice(h->cfg.device));
    HIP_TRY(h, hipDeviceSynchronize());
    HIP_TRY(h, hipMemcpy(host_slots, h->rec_slot, sizeof(int64_t) * (size_t)h->B * h->R * h->NO, hipMemcpyDeviceToHost));
    return STAND_OK;
}

extern "C" int stand_get_node_counts(stand_handle *h, uint64_t *host_counts)
{
    if (!h || !host_counts) return STAND_EINVAL;
    HIP_TRY(h, hipSetDevice(h->cfg.device));
    HIP_TRY(h, hipDeviceSynchronize());
    HIP_TRY(h, hipMemcpy(host_counts, h->node_count, sizeof(uint64_t) * (size_t)h->N, hipMemcpyDeviceToHost));
    return STAND_OK;
}

extern "C" int stand_reset_node_counts(stand_handle *h)
{
    if (!h) return STAND_EINVAL;
    HIP_TRY(h, hipSetDevice(h->cfg.device));
    HIP_TRY(h, hipDeviceSynchronize());
    HIP_TRY(h, hipMemset(h->node_count, 0, sizeof(uint64_t) * (size_t)h->N));
    return STAND_OK;
}

// ---- draft-tree shapes (host only) -----------------------------------------------------------------
extern "C" int stand_tree_initial(int32_t levels, int32_t *host_parent_out, int32_t capacity, int32_t *n_out)
{
    if (levels < 1 || levels > STAND_MAX_DEPTH || !n_out || capacity < 0 || (capacity > 0 && !host_parent_out))
        return STAND_EINVAL;
    // One level at a time, as arrays: rank[i] of node i among its siblings and sibs[i], the size of its
    // sibling group.  The level's fan-outs are a function of (depth, rank, sibs); the next level is their
    // expansion, and the parents of its nodes are this level's ids repeated fan-out times.
    std::vector<int32_t> parents(1, -1), rank(1, 0), sibs(1, 1), fan;
    int32_t level_first = 0;  // id of the level's first node
    for (int32_t depth = 0; depth < levels; ++depth) {
        const size_t n = rank.size();
        fan.assign(n, 0);
        for (size_t i = 0; i < n; ++i) {
            int32_t f;
            if (depth == 0) f = 8;
            else if (depth == 1) f = std::max(8 - 2 * rank[i], 1);
            else f = std::max((int32_t)std::ceil((double)(sibs[i] - 1) / (0.7 * (double)rank[i] + 1.0)), depth <= 3 ? 2 : 0);
            fan[i] = f;
        }
        fan[0] = std::max(fan[0], 3);
        size_t total = 0;
        for (size_t i = 0; i < n; ++i) total += (size_t)fan[i];
        if (total == 0) break;
        std::vector<int32_t> next_rank, next_sibs;
        next_rank.reserve(total);
        next_sibs.reserve(total);
        for (size_t i = 0; i < n; ++i) {
            parents.insert(parents.end(), (size_t)fan[i], level_first + (int32_t)i);
            for (int32_t r = 0; r < fan[i]; ++r) next_rank.push_back(r);
            next_sibs.insert(next_sibs.end(), (size_t)fan[i], fan[i]);
        }
        level_first += (int32_t)n;
        rank.swap(next_rank);
        sibs.swap(next_sibs);
    }
    *n_out = (int32_t)parents.size();
    if (capacity > 0) {
        if ((size_t)capacity < parents.size()) return STAND_EINVAL;
        std::copy(parents.begin(), parents.end(), host_parent_out);
    }
    return STAND_OK;
}

extern "C" int stand_tree_select(const int32_t *host_parent, const uint64_t *host_counts, int32_t n, int32_t n_keep,
                                 int32_t *host_parent_out, int32_t *host_old_id_out)
{
    if (!host_parent || !host_counts || !host_parent_out || n < 1 || n_keep < 1 || n_keep > n) return STAND_EINVAL;
    if (host_parent[0] != -1) return STAND_EINVAL;
    for (int32_t u = 1; u < n; ++u)
        if (host_parent[u] < 0 || host_parent[u] >= u) return STAND_EINVAL;
    std::vector<int32_t> depth((size_t)n, 0), first_child((size_t)n, -1), nchild((size_t)n, 0);
    for (int32_t u = 1; u < n; ++u) {
        depth[u] = depth[host_parent[u]] + 1;
        if (nchild[host_parent[u]]++ == 0) first_child[host_parent[u]] = u;
        if (u > 1 && (host_parent[u] < host_parent[u - 1])) return STAND_EINVAL;  // children must be contiguous, breadth first
    }
    // Grow the kept set from the root: the candidates are the children of kept nodes, the best
    // candidate is the one with the largest usable count (a node is used at most as often as
    // its parent), then the shallowest, then the lowest id.
    struct Cand { uint64_t count; int32_t depth, id; };
    auto worse = [](const Cand &x, const Cand &y) {
        if (x.count != y.count) return x.count < y.count;
        if (x.depth != y.depth) return x.depth > y.depth;
        return x.id > y.id;
    };
    std::vector<Cand> heap;
    std::vector<char> kept((size_t)n, 0);
    uint64_t top = 0;
    for (int32_t u = 0; u < n; ++u) top = std::max(top, host_counts[u]);
    heap.push_back(Cand{top, 0, 0});
    int32_t taken = 0;
    while (taken < n_keep && !heap.empty()) {
        std::pop_heap(heap.begin(), heap.end(), worse);
        const Cand c = heap.back();
        heap.pop_back();
        kept[(size_t)c.id] = 1;
        ++taken;
        for (int32_t j = 0; j < nchild[c.id]; ++j) {
            const int32_t v = first_child[c.id] + j;
            heap.push_back(Cand{std::min(host_counts[v], c.count), depth[v], v});
            std::push_heap(heap.begin(), heap.end(), worse);
        }
    }
    // breadth-first renumbering of the kept nodes, children in their old rank order
    std::vector<int32_t> queue, new_of((size_t)n, -1);
    queue.push_back(0);
    new_of[0] = 0;
    host_parent_out[0] = -1;
    for (size_t head = 0; head < queue.size(); ++head) {
        const int32_t u = queue[head];
        if (host_old_id_out) host_old_id_out[head] = u;
        for (int32_t j = 0; j < nchild[u]; ++j) {
            const int32_t v = first_child[u] + j;
            if (!kept[(size_t)v]) continue;
            new_of[(size_t)v] = (int32_t)queue.size();
            host_parent_out[queue.size()] = (int32_t)head;
            queue.push_back(v);
        }
    }
    return (int32_t)queue.size() == n_keep ? STAND_OK : STAND_EINVAL;
}

extern "C" int stand_copy_bytes(void *d_dst, const void *d_src, uint64_t bytes, void *stream)
{
    if (!d_dst || !d_src || (bytes & 15u) || (((uintptr_t)d_dst | (uintptr_t)d_src) & 15u)) return STAND_EINVAL;
    const size_t nwords = bytes / 16;
    if (nwords == 0) return STAND_OK;
    const size_t want = (nwords + 255) / 256;
    const unsigned blocks = (unsigned)(want < 16384 ? want : 16384);
    copy_words_kernel<<<dim3(blocks), dim3(256), 0, (hipStream_t)stream>>>((const uint4 *)d_src, (uint4 *)d_dst, nwords);
    return hipGetLastError() == hipSuccess ? STAND_OK : STAND_EHIP;
}

extern "C" int stand_read_rows(const void *d_src, uint64_t row_bytes, uint64_t rows, uint32_t *d_sink, void *stream)
{
    if (!d_src || !d_sink || row_bytes == 0 || (row_bytes & 15u) || ((uintptr_t)d_src & 15u) || rows == 0 ||
        rows > 0x7FFFFFFFull)
        return STAND_EINVAL;
    read_rows_kernel<<<dim3((unsigned)rows), dim3(256), 0, (hipStream_t)stream>>>((const uint4 *)d_src, (size_t)(row_bytes / 16),
                                                                                 d_sink);
    return hipGetLastError() == hipSuccess ? STAND_OK : STAND_EHIP;
}

extern "C" const char *stand_strerror(int code)
{
    switch (code) {
    case STAND_OK: return "ok";
    case STAND_EINVAL: return "invalid argument or configuration";
    case STAND_ENOMEM: return "out of memory";
    case STAND_EHIP: return "HIP runtime error (see stand_last_hip_error)";
    case STAND_ESTATE: return "call not allowed in this state";
    case STAND_ELIMIT: return "request exceeds a fixed limit of the library";
    default: return "unknown error";
    }
}

extern "C" int stand_last_hip_error(const stand_handle *h) { return h ? h->last_hip : 0; }
