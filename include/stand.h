/*
 * stand.h -- C ABI of libstand: the per-step speculation loop of STAND (STochastic Adaptive
 * N-gram Drafting, arxiv 2506.04708) for AMD MI355X (gfx950), with the target model's logits
 * supplied by the caller.
 *
 * One handle owns one n-gram table in device memory that is shared by `max_batch`
 * trajectories, the trajectories' context tails and the pending draft tree of each.
 *
 * Conventions
 *   - Pointers named d_* are DEVICE memory owned by the caller; every output buffer is fully
 *     overwritten.  Pointers named host_* are HOST memory.  Nothing is retained after return
 *     except by stand_create (which copies the tree).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls are
 *     asynchronous on it and ordered by it; the functions documented as synchronising wait
 *     for the stream themselves.
 *   - Every function returns STAND_OK (0) or a negative STAND_E* code.  On STAND_EINVAL
 *     nothing has been launched and no output has been written.
 *   - One host thread per handle at a time.
 *   - Tree layout: node 0 is the root (= the last committed token, whose logits row predicts
 *     the first new token); parent[u] < u; nodes are numbered breadth first with the children
 *     of a node contiguous, in rank order (rank j = j-th draw of the sampling without
 *     replacement).  N = tree_nodes counts the root; D = depth of the deepest node.
 *   - Logits layout: [max_batch][tree_nodes][vocab], row major, vocab contiguous, bf16 bit
 *     patterns (uint16) or float32.  Entries must be finite or -inf, each row's maximum finite.
 *   - Token ids are int32 in [0, vocab); -1 marks "no token" (an invalid tree node, padding).
 */
#ifndef STAND_H
#define STAND_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define STAND_OK 0
#define STAND_EINVAL (-1) /* bad argument or configuration                        */
#define STAND_ENOMEM (-2) /* host or device allocation failed                     */
#define STAND_EHIP (-3)   /* a HIP call failed; stand_last_hip_error() has its code */
#define STAND_ESTATE (-4) /* call order violated (e.g. import into a used table)   */
#define STAND_ELIMIT (-5) /* the request exceeds a fixed limit of the library        */

#define STAND_BF16 0
#define STAND_F32 1

#define STAND_UPDATE_ACCEPTED_PATH 0 /* merge the rows that produced committed tokens (paper Sec. 4.1) */
#define STAND_UPDATE_ALL_NODES 1     /* merge the row of EVERY drafted node of the verified tree, each under  */
                                     /* the context it would have if its path were accepted: records in the   */
                                     /* order b, node, n ascending; commit rows are then ignored by the merge  */
                                     /* (the committed tokens are still appended).  A stress variant for the   */
                                     /* table: thousands of records per step instead of hundreds               */

/* What an update does to an entry that already exists.  The method keeps the running mean of all
 * observations of a context (paper Sec. 4.1).  REPLACE keeps only the newest observation, the
 * policy of the lookup table the paper compares against and argues loses information as
 * trajectories accumulate (Sec. 5.1, discussion of Table 1); the occurrence count is still
 * kept.  Records of one step apply in record order, so the last record of a key wins. */
#define STAND_MERGE_MEAN 0
#define STAND_MERGE_REPLACE 1

/* How the children of a tree node are drawn from its table entry (paper Sec. 3.1 "deterministic
 * or stochastic" drafting, Sec. 4.2, and the ablation of Table 5).  All three keep the output
 * distribution equal to the target's; they differ in how often drafts are accepted. */
#define STAND_DRAFT_GUMBEL_TOPK 0   /* Gumbel-Top-K: score ln mu - ln(-ln U), the c largest (the method) */
#define STAND_DRAFT_MULTINOMIAL 1   /* c sequential draws without replacement, proportional to mu;     */
                                    /* the uniform of draw j is keyed by j; same law as Gumbel-Top-K     */
#define STAND_DRAFT_DETERMINISTIC 2 /* the c largest mu (ties: lower id); in verification the proposal  */
                                    /* of each child is one-hot, so it is accepted with probability r(x) */

/* How stand_step issues its work (results are the same; see stand_set_step_plan). */
#define STAND_STEP_AUTO 0   /* one launch where it pays (769 .. 8192 rows, accepted-path updates, accepted paths */
                            /* that seldom reach below upper_depth: watched while running), else serial        */
#define STAND_STEP_SERIAL 1 /* five dependent launches: rows, exact sums, finish + claims, apply, draft           */
#define STAND_STEP_FUSED 2  /* one launch: the dependent tail runs beside the rows that are still streaming      */

#define STAND_MAX_TOPK 32
#define STAND_MAX_ORDER 8
#define STAND_MAX_NODES 1024
#define STAND_MAX_DEPTH 31
#define STAND_STATIC_SCRATCH_BYTES (8u << 20) /* scratch of stand_verify_static: 8 MiB per GPU */

typedef struct stand_handle stand_handle;

typedef struct {
    int32_t vocab;              /* V >= max(2, topk); a row of logits must stay 128 KiB below 4 GiB    */
                                /* (V <= 2 147 418 112 for bf16, 1 073 709 056 for fp32)               */
    int32_t max_batch;          /* B >= 1 trajectories sharing the table                            */
    int32_t order_min;          /* shortest context length used as a key, >= 1                      */
    int32_t order_max;          /* longest, <= STAND_MAX_ORDER (paper Sec. 4.1: unigram .. 4-gram)   */
    int32_t topk;               /* K ids and probabilities stored per key (paper: 10), <= 32;       */
                                /* must be >= the largest fan-out of the tree                       */
    int32_t tree_nodes;         /* N, root included, <= STAND_MAX_NODES                             */
    const int32_t *tree_parent; /* host, [N], layout above; copied                                  */
    float temperature;          /* T > 0; rows are softmax(logits / T) (paper Sec. 5: 0.6)          */
    uint64_t table_capacity;    /* slots, a power of two >= 16                                      */
    int32_t max_probe;          /* linear-probe limit, >= 1; past it an update is dropped+counted   */
                                /* (which updates of a step are dropped at a nearly full table      */
                                /* depends on the order in which the step's keys claim their slots) */
    uint64_t seed;              /* key of the counter-based uniforms                                */
    int32_t logits_dtype;       /* STAND_BF16 or STAND_F32                                          */
    int32_t update_mode;        /* STAND_UPDATE_*                                                   */
    int32_t device;             /* HIP device ordinal                                               */
    int32_t draft_mode;         /* STAND_DRAFT_*                                                    */
    int32_t merge_policy;       /* STAND_MERGE_*                                                    */
} stand_config;

typedef struct {
    uint64_t hits[STAND_MAX_ORDER + 1]; /* draft lookups answered by order n                          */
    uint64_t misses;                    /* draft lookups that found no order                          */
    uint64_t inserts, merges, drops;    /* table updates: new key / existing key / no slot in reach   */
    uint64_t near_threshold;            /* accept tests decided by the exact normaliser because the   */
                                        /* fast one left them within its error bound                  */
    uint64_t tokens_emitted;
    uint64_t accept_tests;
    uint64_t filter_mismatch;           /* path nodes whose outcome changed under exact arithmetic     */
                                        /* (must stay 0; a self-check of the error bound)              */
    uint64_t wait_expired;              /* one-launch step: bounded waits that ran out (must stay 0;   */
                                        /* the outputs of that step are void, see stand_set_wait_limit) */
    uint64_t late_paths;                /* accepted paths that reached below tree depth upper_depth    */
                                        /* (stand_set_step_plan): what STAND_STEP_AUTO watches          */
} stand_stats;

/* Creates a handle: validates the configuration, copies the tree, allocates and clears the
 * table (capacity * (16 + 8*topk) bytes) and the per-trajectory state on cfg->device.
 * Synchronises the device. */
int stand_create(const stand_config *cfg, stand_handle **out);
int stand_destroy(stand_handle *h);

/* Depth D of the tree given at creation; the width of the out_* arrays below is D + 1. */
int stand_depth(const stand_handle *h);

/* Prompt / prefix of trajectory b (host tokens, n >= 0): replaces its context.  Nothing is
 * merged into the table (no distribution exists for prompt positions) and the pending draft
 * of b is dropped.  Synchronises `stream`. */
int stand_set_context(stand_handle *h, int32_t b, const int32_t *host_tokens, int32_t n, void *stream);

/* Beam copy (tree search: parents copied, table shared): trajectory b continues from the context of
 * host_src_of[b] (B entries in 0 .. B-1, as it was before the call; a trajectory may be the source of
 * several).  Pending drafts are dropped; call stand_draft before the next verify.  Asynchronous on
 * `stream` (the map is copied before the call returns); no host synchronisation. */
int stand_reorder(stand_handle *h, const int32_t *host_src_of, void *stream);

/* Table update (paper Sec. 4.1, "Efficient logit approximation").  For committed token j of
 * trajectory b (j < d_commit_len[b] <= D+1), produced by the distribution of logits row
 * d_commit_row[b][j], and every order n the context is long enough for: the row's top-K
 * (ids, softmax probabilities) is merged into the entry keyed by the n tokens preceding
 * token j -- running mean with weights k/(k+1) and 1/(k+1), absent ids = 0, truncated to the
 * K largest by (probability desc, id asc).  Records apply in the order b, j, n ascending.
 * Afterwards the tokens are appended to the contexts.  d_commit_tok/d_commit_row: [B][D+1]. */
int stand_update(stand_handle *h, uint64_t step, const void *d_logits, const int32_t *d_commit_tok,
                 const int32_t *d_commit_row, const int32_t *d_commit_len, void *stream);

/* Draft (paper Sec. 4.2, "Stochastic tree drafting" and "Gumbel-Top-K sampling").  For every
 * trajectory, walks the tree: a node with a valid token looks up its context (committed
 * context + tokens on the path from the root) from order_max down to order_min, first hit
 * wins; its c children get the c largest of  ln mu_i - ln(-ln U_i)  over the stored ids with
 * mu_i > 0, in rank order.  Fewer candidates than children, or a miss: the remaining
 * children are -1 and so are their subtrees.  Writes d_draft_tok [B][N] (node 0 = last
 * committed token, or -1 for an empty context) and keeps the proposals for stand_verify. */
int stand_draft(stand_handle *h, uint64_t step, int32_t *d_draft_tok, void *stream);

/* Verify (paper Sec. 3.2 applied recursively to the children of a node).  d_logits holds the
 * target model's logits for the tree drafted with the same `step`.  From the root: the
 * children of the current node are tested in rank order, child x accepted iff
 * U < r(x) / w(x) with r the residual target and w the proposal renormalised over the
 * children not yet rejected; on rejection r <- norm(max(0, r - w)).  An accepted child
 * becomes the current node.  When no child is accepted (or there is none) one token is drawn
 * from the residual of the current node -- the position floor(u T / 2^64) in the residual's
 * cumulative integer mass T, u = 64 counter-based random bits of (trajectory, step, node) --
 * and the walk stops.  Each node on the accepted path adds 1 to its acceptance counter
 * (stand_get_node_counts).
 * Outputs: d_out_tok [B][D+1] emitted tokens, d_out_node [B][D+1] the tree node whose logits
 * row produced each of them (root, then the accepted nodes), d_out_len [B] in 1..D+1; unused
 * entries are -1.  Handle state (table, contexts) is not changed. */
int stand_verify(stand_handle *h, uint64_t step, const void *d_logits, int32_t *d_out_tok,
                 int32_t *d_out_node, int32_t *d_out_len, void *stream);

/* stand_verify for callers that cannot allocate device memory or tolerate a library that does: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same
 * results and same error behaviour as stand_verify, but everything the kernels keep between them (the
 * row pass's per-row results, the partial sums, stop records and observations of the path rows) lives in
 * a fixed array of STAND_STATIC_SCRATCH_BYTES that is part of the library's device image -- one copy
 * per GPU, held until the process ends -- instead of the handle's own buffers.  The call allocates and
 * frees nothing (no hipMalloc, hipFree or allocating library routine).
 *   - Limit: stand_static_scratch_need(h) bytes must fit the array (about max_batch * tree_nodes *
 *     (12 * topk + 12) bytes plus the path rows' share: 0.6 MB for 32 x 64 rows with topk 16, 7.5 MB for
 *     128 x 128 rows with topk 32); otherwise STAND_ELIMIT and nothing is launched.
 *   - All handles on one GPU share that GPU's array and a call leaves its contents behind: calls that
 *     overlap on one GPU (different streams or host threads) race; calls ordered by one stream do not.
 *     Nothing in the array needs to be cleared between calls.
 *   - stand_row_results keeps reporting the last stand_verify / stand_step, not this call. */
int stand_verify_static(stand_handle *h, uint64_t step, const void *d_logits, int32_t *d_out_tok,
                        int32_t *d_out_node, int32_t *d_out_len, void *stream);
/* Scratch bytes stand_verify_static needs for this handle's shape (0 for a NULL handle). */
uint64_t stand_static_scratch_need(const stand_handle *h);

/* One speculation step = stand_verify(step) -> stand_update with the emitted tokens and their
 * rows -> stand_draft(step + 1) into d_next_draft_tok [B][N].
 * If d_force_tok ([B][D+1], may be NULL) is given, the tokens committed to the contexts and
 * used as table keys are d_force_tok[b][0 .. out_len[b]) instead of the emitted ones (replay
 * of a recorded trajectory); the emitted tokens are still returned in d_out_tok. */
int stand_step(stand_handle *h, uint64_t step, const void *d_logits, int32_t *d_out_tok,
               int32_t *d_out_node, int32_t *d_out_len, int32_t *d_next_draft_tok,
               const int32_t *d_force_tok, void *stream);

/* How stand_step is issued (paper: the step is verify -> update -> draft, Sec. 3.2, 4.1, 4.2; this only
 * chooses the launch structure, every output is the same bit for bit).
 *   mode         STAND_STEP_AUTO / SERIAL / FUSED.  FUSED is refused (STAND_EINVAL) with
 *                STAND_UPDATE_ALL_NODES, whose records need every drafted row.  AUTO copies one counter
 *                (stand_stats.late_paths) to pinned host memory every 32 steps, without waiting for it,
 *                and takes the serial launches while more than 0.4 paths per step reach below
 *                upper_depth (they would wait for rows that stream late), the one launch again below
 *                0.25; no such copy is made while the stream is being captured, or in the other modes.
 *                While the stream is being captured (HIP graphs) stand_step always issues the five
 *                launches: the one launch carries its own number as an argument and cannot be replayed.
 *   upper_depth  FUSED: the rows of tree nodes up to this depth take the first places in the launch
 *                (default 2: paths that end above depth 3 never wait for a late row; deeper paths are
 *                still correct, the tail then waits for the rows it needs).  0 .. STAND_MAX_DEPTH.
 *   tail_groups  FUSED: workgroups per trajectory that share the exact sums of the path rows, 1 .. 8;
 *                0 = chosen from the batch size.
 *   rows_first   FUSED: number of row workgroups placed before the tail's workgroups (at least the
 *                upper levels' rows); 0 = as many as the device holds at once less two tail workgroups
 *                per trajectory, which are then resident from the start and follow the path as soon as
 *                the root rows are done; the other tail workgroups start when the first rows end.
 *   shuffle      non-zero: the order in which row workgroups take rows is permuted (seeded by the value);
 *                a test that results do not depend on the workgroup -> work mapping. */
int stand_set_step_plan(stand_handle *h, int32_t mode, int32_t upper_depth, int32_t tail_groups, int32_t rows_first,
                        uint32_t shuffle);

/* 1 if stand_step on this handle is currently issued as one launch, 0 if as five (see stand_set_step_plan). */
int stand_step_is_one_launch(const stand_handle *h);

/* Bound, in microseconds, of every wait inside the one-launch step (default 200 000).  A wait that runs
 * out is counted in stand_stats.wait_expired; every kernel still ends normally, but the step's outputs
 * for the affected trajectories are void (out_len 0, tokens -1) and the table must be considered invalid.
 * With a healthy device no wait comes near the default.  0 makes every wait that is not satisfied at once
 * expire (for tests of this path). */
int stand_set_wait_limit(stand_handle *h, uint64_t microseconds);

/* Measurement aid: where the time of the one-launch step goes.  enable != 0 makes later one-launch steps
 * record readings of the device's constant clock (allocates 16 + 64 * max_batch bytes once; enable == 0
 * frees them).  host_ticks, if not NULL, receives the readings of the last such step ([2 + 8 * max_batch]:
 * earliest start and latest end of a row workgroup, then per trajectory: tail workgroup started, path
 * known, exact sums of all its workgroups in, its claims made, its rows finished, all trajectories' claims
 * in, all records applied, draft written); STAND_ESTATE if recording was not enabled.  *ticks_per_second,
 * if not NULL, receives the clock's rate.  Synchronises the device. */
int stand_step_timeline(stand_handle *h, int32_t enable, uint64_t *host_ticks, uint64_t *ticks_per_second);

/* Per-row results of the last stand_verify / stand_step, for inspection: for each of the B*N
 * rows the maximum logit, the softmax normaliser (fast single-pass value, relative error
 * below 1e-5), and the K largest entries (ids exact; probabilities from the fast normaliser).
 * Any pointer may be NULL.  d_row_max, d_row_sum: [B*N] float; d_top_idx: [B*N][K] int32;
 * d_top_p: [B*N][K] float. */
int stand_row_results(stand_handle *h, float *d_row_max, float *d_row_sum, int32_t *d_top_idx,
                      float *d_top_p, void *stream);

/* Table export: entries sorted by key fingerprint, each
 *   uint64 fingerprint, uint32 count, uint32 order, int32 ids[K], float mu[K]   (16 + 8K bytes).
 * On entry *inout_bytes is the size of host_buf; on return the bytes needed/written.
 * host_buf == NULL only queries the size.  Synchronises the device. */
int stand_table_export(stand_handle *h, void *host_buf, uint64_t *inout_bytes);
/* Loads entries in the export format into an EMPTY table (STAND_ESTATE otherwise). */
int stand_table_import(stand_handle *h, const void *host_buf, uint64_t bytes);

/* Copies the last `n` context tokens of trajectory b to host (n <= order_max kept on device)
 * and returns the context length through *len_out.  Synchronises `stream`. */
int stand_get_context(stand_handle *h, int32_t b, int32_t *host_tail, int32_t n, int64_t *len_out, void *stream);

/* Table slot of every merge record of the last stand_update / stand_step, for inspection: host_slots
 * [max_batch * R * orders] with R = depth + 1 (or tree_nodes with STAND_UPDATE_ALL_NODES), record
 * (b, position or node, order) at index (b * R + position) * orders + (order - order_min); -1 for a record
 * that did not exist in that update (position beyond the committed tokens, context shorter than the order,
 * undrafted node) AND for a record that was dropped because no slot was in reach (paper Sec. 4.1 has an
 * unbounded table; see max_probe).  Synchronises the device. */
int stand_get_record_slots(stand_handle *h, int64_t *host_slots);

/* Counters since creation.  Synchronises the device. */
int stand_get_stats(stand_handle *h, stand_stats *out);

/* Timing of the row pass (the kernel that streams all logits; paper Sec. 4.1 softmax + top-k):
 * after stand_profile_begin, each of the next max_launches row-pass launches made by
 * stand_verify / stand_step is bracketed by a pair of HIP events on the caller's stream.
 * stand_profile_end synchronises the device, returns the summed event time in milliseconds
 * and the number of launches measured, and switches the timing off. */
/* Accept tests are first decided with a fast normaliser of the row.  Its relative error is bounded from
 * the shape of the launch (2^-23 per addition a lane performs: vocab / (8 or 4 elements * 64 lanes *
 * waves per row), plus the combination of lanes and waves) and never assumed below 5e-5.  A test whose margin
 * is smaller than the assumed error is decided again with the exact normaliser (counted in
 * stand_stats.near_threshold), and every node on an accepted path is replayed with exact
 * probabilities afterwards (stand_stats.filter_mismatch counts disagreements; it must stay 0), so
 * results never depend on this value.  `margin` in [5e-5, 1] replaces the 5e-5 floor for later calls:
 * a larger value only sends more tests to the exact path (1 sends practically all of them).
 * STAND_EINVAL outside the range. */
int stand_set_filter_margin(stand_handle *h, float margin);

int stand_profile_begin(stand_handle *h, int32_t max_launches);
int stand_profile_end(stand_handle *h, double *row_pass_ms_total, int32_t *launches);

/* Inputs of the target model's verify pass for the pending drafts (paper Sec. 3.2: the drafted
 * tree is scored in one pass with tree attention).  d_mask[b][u][v] (uint8, [B][N][N]) = 1 iff
 * node v lies on the path root -> u (u included) and u carries a drafted token, else 0;
 * d_pos[b][u] (int64, [B][N]) = position of node u in trajectory b's sequence, i.e.
 * (committed tokens - 1) + depth(u) with the root = the last committed token; -1 for nodes
 * without a drafted token.  Reflects the last stand_draft / stand_step.  The rows of the KV
 * cache to keep after verification are those of d_out_node[b][0 .. d_out_len[b]) of
 * stand_verify / stand_step; no separate output is needed for them. */
int stand_tree_packing(stand_handle *h, uint8_t *d_mask, int64_t *d_pos, void *stream);

/* ---- data-driven draft tree (paper Sec. 4.3 and appendix "Initial tree for optimization") ----
 *
 * The paper starts from a large heuristic tree, runs speculative decoding on sample data while
 * counting which nodes lie on accepted paths, keeps the most often accepted nodes and re-packs
 * them into the static tree used afterwards.  The three host-side steps of that procedure:
 *
 * stand_tree_initial: the initial tree of the appendix (Alg. 1) with `levels` levels below the
 *   root (the paper: 20, giving 625 nodes).  Fan-out by depth and by rank r among the siblings:
 *   root 8; depth 1: max(8 - 2r, 1); deeper: ceil((siblings - 1) / (0.7 r + 1)), at least 2 at
 *   depths 2 and 3; the first node of each level at least 3.  Writes the node count to *n_out
 *   and, if capacity > 0, parent[] (layout of stand_config.tree_parent) to host_parent_out;
 *   STAND_EINVAL if capacity is positive but too small.  Host memory only, no device needed.
 *
 * stand_get_node_counts / stand_reset_node_counts: every stand_verify / stand_step adds 1 to
 *   counts[u] for each node u on each trajectory's accepted path (the root is on every path).
 *   host_counts: [tree_nodes].  Both synchronise the device.
 *
 * stand_tree_select: keeps n_keep of the n nodes of `host_parent` -- ranked by (usable count
 *   descending, depth ascending, id ascending), where a node's usable count is the smallest
 *   count on its way to the root, so the kept set is closed under parents -- and re-packs them
 *   breadth first with siblings in their old rank order.  Writes parent[] of the new tree to
 *   host_parent_out[n_keep] and, if not NULL, the old id of every new node to
 *   host_old_id_out[n_keep].  STAND_EINVAL if the input is not in the tree layout above. */
int stand_tree_initial(int32_t levels, int32_t *host_parent_out, int32_t capacity, int32_t *n_out);
int stand_get_node_counts(stand_handle *h, uint64_t *host_counts);
int stand_reset_node_counts(stand_handle *h);
int stand_tree_select(const int32_t *host_parent, const uint64_t *host_counts, int32_t n, int32_t n_keep,
                      int32_t *host_parent_out, int32_t *host_old_id_out);

/* Measurement aid, not part of the method: copies `bytes` (a multiple of 16, both pointers
 * 16-byte aligned, device memory, non-overlapping) with a plain grid-stride kernel on `stream`.
 * Its HBM traffic is known (bytes read + bytes written), so profiler byte counters read for
 * the kernels above can be scaled by what they read for this one.  STAND_EINVAL on a bad
 * size or alignment. */
int stand_copy_bytes(void *d_dst, const void *d_src, uint64_t bytes, void *stream);

/* Measurement aid, not part of the method: reads `rows` consecutive rows of `row_bytes` bytes
 * (a multiple of 16; d_src 16-byte aligned, device memory) with one 256-thread workgroup per
 * row, the launch shape of the row pass, doing nothing with the data but a checksum.  Its
 * duration is the floor of any kernel that fetches the logits once on this device.  d_sink
 * (device, 4 * rows words) receives one word per wave.  STAND_EINVAL on a bad size or
 * alignment. */
int stand_read_rows(const void *d_src, uint64_t row_bytes, uint64_t rows, uint32_t *d_sink, void *stream);

const char *stand_strerror(int code);
int stand_last_hip_error(const stand_handle *h);

#ifdef __cplusplus
}
#endif
#endif /* STAND_H */
