"""Seeded synthetic inputs for the STAND speculation step: draft-tree shapes, token streams
shaped like reasoning traces with repeated spans, and verify-pass logits.

This module holds none of the method's arithmetic (no softmax, top-k, hashing of keys,
sampling or acceptance): it only produces the bytes that the library and its checker are
both fed.  It needs numpy only.
"""
import numpy as np

BASE_SEED = 0x5354414E44

# Workload shapes (paper Sec. 5: temperature 0.6, orders up to 4-grams, top-10; vocabulary
# sizes are those of the model families used there).
CONFIGS = {
    "cfg1": dict(B=1, V=32000, dtype="f32", N=16, D=4, caps=[4, 2, 1, 1], order_min=1, order_max=3, K=10,
                 T=0.6, steps=64, capacity=4096, rho=0.4, seed=BASE_SEED + 0),
    "cfg2": dict(B=1, V=152064, dtype="bf16", N=32, D=6, caps=[4, 2, 2, 1], order_min=1, order_max=4, K=10,
                 T=0.6, steps=2048, capacity=1 << 20, rho=0.5, seed=BASE_SEED + 1),
    "cfg3": dict(B=32, V=152064, dtype="bf16", N=64, D=8, caps=[8, 4, 2, 1], order_min=1, order_max=4, K=16,
                 T=0.6, steps=4096, capacity=1 << 22, rho=0.5, seed=BASE_SEED + 2),
    # best-of-N: all trajectories start from one 512-token prompt, then diverge; 60 % of the repeated spans are
    # copies from ANOTHER trajectory's history
    "cfg4": dict(B=64, V=128256, dtype="bf16", N=48, D=7, caps=[6, 3, 2, 1], order_min=1, order_max=4, K=10,
                 T=1.0, steps=8192, capacity=1 << 23, rho=0.6, cross=0.6, shared_prefix=512, prompt_len=512,
                 seed=BASE_SEED + 3),
    # tree search: every 64 steps half of the beams are pruned and the survivors are expanded (each beam
    # continues from the context of a surviving parent; the table is shared and kept)
    "cfg5": dict(B=128, V=152064, dtype="bf16", N=128, D=10, caps=[8, 4, 2, 1], order_min=1, order_max=5, K=32,
                 T=0.8, steps=16384, capacity=1 << 24, rho=0.5, reorder_every=64, seed=BASE_SEED + 4),
}


# ---- draft-tree shapes ------------------------------------------------------------------
def make_tree(N, D, caps):
    """Static draft tree with N nodes (root included) and depth D.

    Candidates are the nodes of the complete tree whose fan-out at depth d is caps[d] (last
    value repeated).  The root, all its children and the leftmost chain down to depth D are
    taken first; then the remaining candidate with the largest prior prod(0.9 * 0.7**rank)
    over its path is added (ties: shallower, then smaller parent path, then lower rank; a
    child of rank j only after its sibling of rank j-1) until N nodes are chosen.  Nodes are
    numbered breadth first, siblings contiguous in rank order.  Returns parent[N].
    """
    def cap(d):
        return caps[d] if d < len(caps) else caps[-1]

    def score(path):
        s = 1.0
        for r in path:
            s *= 0.9 * 0.7 ** r
        return s

    sel = {()}
    for r in range(cap(0)):
        sel.add((r,))
    for d in range(1, D + 1):
        sel.add(tuple([0] * d))
    if len(sel) > N:
        raise ValueError("N too small for this depth and root fan-out")
    while len(sel) < N:
        best = None
        for p in sel:
            d = len(p)
            if d >= D:
                continue
            for r in range(cap(d)):
                c = p + (r,)
                if c in sel:
                    continue
                key = (-score(c), len(c), p, r)
                if best is None or key < best[0]:
                    best = (key, c)
                break
        if best is None:
            raise ValueError("candidate tree exhausted before N nodes")
        sel.add(best[1])
    ids = {(): 0}
    parent = [-1]
    frontier = [()]
    while frontier:
        nxt = []
        for p in frontier:
            for c in sorted(q for q in sel if len(q) == len(p) + 1 and q[:-1] == p):
                ids[c] = len(parent)
                parent.append(ids[p])
                nxt.append(c)
        frontier = nxt
    return np.asarray(parent, dtype=np.int32)


def tree_info(parent):
    """depth[N], nchild[N], first_child[N] (-1 if none) and the maximum depth."""
    parent = np.asarray(parent, dtype=np.int32)
    N = parent.shape[0]
    depth = np.zeros(N, np.int32)
    nchild = np.zeros(N, np.int32)
    first = np.full(N, -1, np.int32)
    for u in range(1, N):
        depth[u] = depth[parent[u]] + 1
        if nchild[parent[u]] == 0:
            first[parent[u]] = u
        nchild[parent[u]] += 1
    return depth, nchild, first, int(depth.max())


# ---- integer hashing for the generators (splitmix-style; not the library's key hash) ------
def _mix(x):
    x = np.asarray(x, dtype=np.uint64)
    with np.errstate(over="ignore"):
        x = (x ^ (x >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        x = (x ^ (x >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        x = x ^ (x >> np.uint64(31))
    return x


def _h(*parts):
    acc = np.uint64(0x243F6A8885A308D3)
    for p in parts:
        with np.errstate(over="ignore"):
            acc = _mix(acc ^ (np.asarray(p, dtype=np.uint64) + np.uint64(0x9E3779B97F4A7C15)))
    return acc


# ---- token streams ----------------------------------------------------------------------
def successors(seed, token, V):
    """The 4 successors of a token in the sparse order-1 Markov source."""
    return np.asarray([int(_h(seed, token, j) % np.uint64(V)) for j in range(4)], dtype=np.int64)


_SUCC_P = np.asarray([0.55, 0.25, 0.15, 0.05])


def token_streams(seed, B, V, length, rho, cross=0.0, shared_prefix=0):
    """B token streams of `length` tokens.

    Each stream is a sequence of spans of length uniform in 8..32.  With probability rho a
    span is a copy of an earlier span (start uniform in the trajectory's own history, or,
    with probability `cross`, in another trajectory's history); otherwise it continues the
    sparse Markov source (4 successors per token with probabilities .55/.25/.15/.05).
    The first `shared_prefix` tokens are common to all trajectories.
    """
    rng = np.random.Generator(np.random.Philox(key=int(seed) & (2 ** 64 - 1)))
    out = np.zeros((B, length), np.int32)
    pos = np.zeros(B, np.int64)
    first = int(rng.integers(V))
    for b in range(B):
        out[b, 0] = first if shared_prefix else int(rng.integers(V))
        pos[b] = 1
    if shared_prefix:
        while pos[0] < min(shared_prefix, length):
            t = pos[0]
            succ = successors(seed, int(out[0, t - 1]), V)
            out[0, t] = succ[rng.choice(4, p=_SUCC_P)]
            pos[0] += 1
        for b in range(1, B):
            out[b, : pos[0]] = out[0, : pos[0]]
            pos[b] = pos[0]
    # round-robin over trajectories so that cross-trajectory copies see comparable histories
    while (pos < length).any():
        for b in range(B):
            if pos[b] >= length:
                continue
            span = int(rng.integers(8, 33))
            span = min(span, length - pos[b])
            if rng.random() < rho and pos[b] > 40:
                src_b = b
                if cross > 0 and B > 1 and rng.random() < cross:
                    src_b = int(rng.integers(B - 1))
                    src_b += src_b >= b
                hist = pos[src_b]
                if hist > span:
                    start = int(rng.integers(0, hist - span + 1))
                    out[b, pos[b]: pos[b] + span] = out[src_b, start: start + span]
                    pos[b] += span
                    continue
            for _ in range(span):
                t = pos[b]
                succ = successors(seed, int(out[b, t - 1]), V)
                out[b, t] = succ[rng.choice(4, p=_SUCC_P)]
                pos[b] += 1
    return out


# ---- logits -----------------------------------------------------------------------------
def f32_to_bf16_bits(x):
    """Round-to-nearest-even conversion of float32 values to bf16 bit patterns (uint16)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b):
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def peaked_tokens(seed, step, b, parent, depth, first_child, nchild, draft_tok, stream_next, V, max_peaks=4):
    """For every tree node of trajectory b: the 1..max_peaks token ids that receive the +8 peak.

    Order of preference: the stream's next token when the node's path matches the stream,
    then the node's drafted children in rank order, then hash-chosen fillers.  stream_next
    is the stream from the root's position on: stream_next[0] is the token after the root.
    Returns an int64 array [N, 4] padded with -1.
    """
    N = parent.shape[0]
    out = np.full((N, 4), -1, np.int64)
    on_stream = np.zeros(N, bool)
    on_stream[0] = True
    for u in range(1, N):
        d = depth[u]
        on_stream[u] = (on_stream[parent[u]] and draft_tok[u] >= 0 and d - 1 < len(stream_next)
                        and int(draft_tok[u]) == int(stream_next[d - 1]))
    for u in range(N):
        r = 1 + int(_h(seed, step, b, u, 77) % np.uint64(max_peaks))
        cand = []
        d = depth[u]
        if on_stream[u] and d < len(stream_next):
            cand.append(int(stream_next[d]))
        for j in range(nchild[u]):
            t = int(draft_tok[first_child[u] + j])
            if t >= 0 and t not in cand:
                cand.append(t)
        j = 0
        while len(cand) < r:
            t = int(_h(seed, step, b, u, 1000 + j) % np.uint64(V))
            j += 1
            if t not in cand:
                cand.append(t)
        out[u, :r] = cand[:r]
    return out


def peaked_tokens_batch(seed, step, parent, depth, first_child, nchild, draft_tok, stream_next, V, max_peaks=4):
    """peaked_tokens for all B trajectories at once (same results, array operations instead of loops over the
    nodes of every trajectory): draft_tok [B, N]; stream_next [B, L] with L >= D + 1, padded with -1 where a
    stream ends.  Returns int64 [B, N, 4] padded with -1, or None if the fixed number of fillers it draws did
    not give enough distinct tokens."""
    draft_tok = np.asarray(draft_tok, np.int64)
    stream_next = np.asarray(stream_next, np.int64)
    B, N = draft_tok.shape
    L = stream_next.shape[1]
    on_stream = np.zeros((B, N), bool)
    on_stream[:, 0] = True
    for u in range(1, N):            # parents come first in the numbering
        d = int(depth[u])
        nxt = stream_next[:, d - 1] if d - 1 < L else np.full(B, -1, np.int64)
        on_stream[:, u] = on_stream[:, parent[u]] & (draft_tok[:, u] >= 0) & (nxt >= 0) & (draft_tok[:, u] == nxt)
    bb = np.arange(B, dtype=np.uint64)[:, None]
    uu = np.arange(N, dtype=np.uint64)[None, :]
    r = 1 + (_h(seed, step, bb, uu, 77) % np.uint64(max_peaks)).astype(np.int64)          # [B, N]
    maxc = int(nchild.max()) if N > 1 else 0
    nfill = max_peaks + 6                                                               # spare fillers for duplicates
    cand = np.full((B, N, 1 + maxc + nfill), -1, np.int64)
    dn = np.minimum(depth, L - 1)
    sn = stream_next[:, dn]                                                             # [B, N]: stream token after node u's path
    cand[:, :, 0] = np.where(on_stream & (depth[None, :] < L) & (sn >= 0), sn, -1)
    for j in range(maxc):
        has = nchild > j
        idx = np.where(has, first_child + j, 0)
        cand[:, :, 1 + j] = np.where(has[None, :], draft_tok[:, idx], -1)
    for j in range(nfill):
        cand[:, :, 1 + maxc + j] = (_h(seed, step, bb, uu, 1000 + j) % np.uint64(V)).astype(np.int64)
    # drop negative entries and later duplicates, keep the order, take the first r
    C = cand.shape[2]
    keep = cand >= 0
    for i in range(1, C):
        keep[:, :, i] &= ~((cand[:, :, :i] == cand[:, :, i:i + 1]) & (cand[:, :, :i] >= 0)).any(axis=2)
    rank = np.cumsum(keep, axis=2) - 1                                                  # position among the kept
    out = np.full((B, N, 4), -1, np.int64)
    sel = keep & (rank < r[:, :, None])
    bi, ui, ci = np.nonzero(sel)
    out[bi, ui, rank[bi, ui, ci]] = cand[bi, ui, ci]
    if not (np.sum(out >= 0, axis=2) == r).all():
        return None                  # too many duplicate fillers (tiny vocabularies): the caller takes the loops
    return out


def logits_step(seed, step, B, N, V, dtype, peaks, sigma2=3.0, peak=8.0, scale=1.0):
    """Verify-pass logits [B, N, V] of one step: i.i.d. N(0, sigma2) noise plus `peak` on the
    tokens listed in peaks[B, N, 4] (-1 = none), all multiplied by `scale` (1: the recipe; larger values
    give the large logits of stress cases).  dtype "f32" -> float32, "bf16" -> uint16 bit patterns
    (rounded to nearest even)."""
    rng = np.random.Generator(np.random.Philox(key=[int(seed) & (2 ** 64 - 1), int(step)]))
    x = rng.standard_normal((B, N, V), dtype=np.float32)
    x *= np.float32(np.sqrt(sigma2))
    for b in range(B):
        for u in range(N):
            for t in peaks[b][u]:
                if t >= 0:
                    x[b, u, int(t)] += np.float32(peak)
    if scale != 1.0:
        x *= np.float32(scale)
    if dtype == "f32":
        return x
    return f32_to_bf16_bits(x)


class Workload:
    """Open-loop replay driver state: the exogenous streams and each trajectory's position.

    The verify result sets the pace (how many tokens are committed); the tokens committed are
    the stream's.  Logits of a step peak on the stream's continuation, on the drafted
    children and on fillers, so acceptance paths of every depth occur.
    """

    def __init__(self, name=None, **override):
        cfg = dict(CONFIGS[name]) if name else {}
        cfg.update(override)
        self.cfg = cfg
        self.B, self.V, self.N, self.D, self.K = cfg["B"], cfg["V"], cfg["N"], cfg["D"], cfg["K"]
        self.dtype, self.T, self.seed = cfg["dtype"], cfg["T"], cfg["seed"]
        self.W = self.D + 1
        # a given parent[] (e.g. a tree produced by the tree optimisation) overrides the shape recipe
        self.parent = (np.asarray(cfg["parent"], np.int32) if cfg.get("parent") is not None
                       else make_tree(cfg["N"], cfg["D"], cfg["caps"]))
        self.depth, self.nchild, self.first_child, dmax = tree_info(self.parent)
        assert dmax == self.D
        self.prompt_len = cfg.get("prompt_len", 16)
        horizon = cfg.get("stream_len", self.prompt_len + (self.D + 1) * cfg.get("run_steps", 64) + self.D + 2)
        self.streams = token_streams(self.seed, self.B, self.V, horizon, cfg["rho"],
                                     cross=cfg.get("cross", 0.0), shared_prefix=cfg.get("shared_prefix", 0))
        self.pos = np.full(self.B, self.prompt_len - 1, np.int64)  # index of the root token in the stream

    def prompt(self, b):
        return self.streams[b, : self.prompt_len]

    def reorder_map(self, step):
        """Beam re-parenting due BEFORE the verification of `step` (tree-search workloads), or None: a seeded
        half of the beams survives, beam b continues from the context of survivor b mod (B / 2) -- a map with
        duplicates.  Each beam keeps its own exogenous stream, so copies of one parent diverge afterwards."""
        every = self.cfg.get("reorder_every", 0)
        if not every or step == 0 or step % every or self.B < 2:
            return None
        rng = np.random.Generator(np.random.Philox(key=[int(self.seed) & (2 ** 64 - 1), 0x7265 + int(step)]))
        survivors = rng.permutation(self.B)[: self.B // 2]
        return survivors[np.arange(self.B) % len(survivors)].astype(np.int32)

    def peaks(self, step, draft_tok):
        L = self.D + 2
        nxt = np.full((self.B, L), -1, np.int64)
        for b in range(self.B):
            t = self.streams[b, self.pos[b] + 1: self.pos[b] + 1 + L]
            nxt[b, : len(t)] = t
        out = peaked_tokens_batch(self.seed, step, self.parent, self.depth, self.first_child, self.nchild,
                                  draft_tok, nxt, self.V, self.cfg.get("max_peaks", 4))
        return out if out is not None else self.peaks_by_loops(step, draft_tok)

    def peaks_by_loops(self, step, draft_tok):
        """The same by the per-trajectory function (kept as the definition; tests compare the two)."""
        out = np.full((self.B, self.N, 4), -1, np.int64)
        for b in range(self.B):
            nxt = self.streams[b, self.pos[b] + 1: self.pos[b] + self.D + 3]
            out[b] = peaked_tokens(self.seed, step, b, self.parent, self.depth, self.first_child, self.nchild,
                                   draft_tok[b], nxt, self.V, self.cfg.get("max_peaks", 4))
        return out

    def logits(self, step, draft_tok):
        return logits_step(self.seed, step, self.B, self.N, self.V, self.dtype, self.peaks(step, draft_tok),
                           scale=self.cfg.get("logit_scale", 1.0))

    def commit(self, out_len):
        """Tokens to commit after a verify that emitted out_len[b] tokens: the stream's next ones."""
        W = self.D + 1
        tok = np.full((self.B, W), -1, np.int32)
        for b in range(self.B):
            n = int(out_len[b])
            tok[b, :n] = self.streams[b, self.pos[b] + 1: self.pos[b] + 1 + n]
            self.pos[b] += n
        return tok
