"""ctypes front end of the CPU oracle (oracle/stand_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by the
cpu_baseline leg of bench.py.  The product package never imports it.

The functions here marshal arguments; all arithmetic is in the C file.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "stand_oracle.c")
_LIB = os.path.join(_HERE, "libstand_oracle.so")

MAX_K = 32
MAX_ORDER = 8
DT_BF16 = 0
DT_F32 = 1
STREAM_DRAFT, STREAM_ACCEPT, STREAM_BONUS = 0, 1, 2
DRAFT_GUMBEL_TOPK, DRAFT_MULTINOMIAL, DRAFT_DETERMINISTIC = 0, 1, 2
UPDATE_ACCEPTED_PATH, UPDATE_ALL_NODES = 0, 1
MERGE_MEAN, MERGE_REPLACE = 0, 1


def build(force=False):
    """Compile the oracle with gcc (no fast-math, no contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fPIC", "-shared", "-Wall", "-Wextra",
             "-o", _LIB, _SRC, "-lm"])
    return _LIB


class _Config(C.Structure):
    _fields_ = [
        ("vocab", C.c_int32), ("max_batch", C.c_int32),
        ("order_min", C.c_int32), ("order_max", C.c_int32),
        ("topk", C.c_int32), ("tree_nodes", C.c_int32),
        ("tree_parent", C.POINTER(C.c_int32)),
        ("temperature", C.c_float),
        ("table_capacity", C.c_uint64),
        ("max_probe", C.c_int32),
        ("seed", C.c_uint64),
        ("logits_dtype", C.c_int32),
        ("update_mode", C.c_int32),
        ("draft_mode", C.c_int32),
        ("merge_policy", C.c_int32),
    ]


class Stats(C.Structure):
    _fields_ = [
        ("hits", C.c_uint64 * (MAX_ORDER + 1)),
        ("misses", C.c_uint64),
        ("inserts", C.c_uint64), ("merges", C.c_uint64), ("drops", C.c_uint64),
        ("near_threshold", C.c_uint64),
        ("tokens_emitted", C.c_uint64),
        ("fp_collisions", C.c_uint64),
        ("accept_tests", C.c_uint64),
    ]


class NodeState(C.Structure):
    _fields_ = [("r", C.c_float * MAX_K), ("w", C.c_float * MAX_K), ("rho", C.c_float),
                ("rounds", C.c_int), ("near_threshold", C.c_int)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        L.so_uniform.restype = C.c_float
        L.so_uniform.argtypes = [C.c_uint64, C.c_uint32, C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32]
        L.so_philox.argtypes = [C.c_uint64] + [C.c_uint32] * 4 + [C.c_void_p]
        L.so_exp2.restype = C.c_float
        L.so_exp2.argtypes = [C.c_float]
        L.so_log.restype = C.c_float
        L.so_log.argtypes = [C.c_float]
        L.so_scale.restype = C.c_float
        L.so_scale.argtypes = [C.c_float]
        L.so_row_softmax.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_float, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.so_topk.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
        L.so_row_obs.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_float, C.c_int] + [C.c_void_p] * 4
        L.so_merge.argtypes = [C.c_uint32, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.so_fingerprint.restype = C.c_uint64
        L.so_fingerprint.argtypes = [C.c_int, C.c_void_p]
        L.so_gumbel_topk.restype = C.c_int
        L.so_gumbel_topk.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
        L.so_verify_node.restype = C.c_int
        L.so_verify_node.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.POINTER(NodeState), C.c_int]
        L.so_multinomial_wor.restype = C.c_int
        L.so_multinomial_wor.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
        L.so_top_c.restype = C.c_int
        L.so_top_c.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p]
        L.so_residual_dense.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.POINTER(NodeState), C.c_void_p]
        L.so_uniform_u64.restype = C.c_uint64
        L.so_uniform_u64.argtypes = [C.c_uint64, C.c_uint32, C.c_uint64, C.c_uint32, C.c_uint32]
        L.so_row_masses.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_float, C.c_void_p]
        L.so_residual_draw.restype = C.c_int32
        L.so_residual_draw.argtypes = [C.c_void_p, C.c_int, C.c_uint64, C.c_int, C.c_void_p, C.POINTER(NodeState), C.c_uint64]
        L.so_create.restype = C.c_void_p
        L.so_create.argtypes = [C.POINTER(_Config)]
        L.so_destroy.argtypes = [C.c_void_p]
        L.so_depth.restype = C.c_int32
        L.so_depth.argtypes = [C.c_void_p]
        L.so_set_context.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_int]
        L.so_reorder.argtypes = [C.c_void_p, C.c_void_p]
        L.so_context_len.restype = C.c_int64
        L.so_context_len.argtypes = [C.c_void_p, C.c_int]
        L.so_context_tail.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p]
        L.so_table_put.restype = C.c_int
        L.so_table_put.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_uint32, C.c_void_p, C.c_void_p]
        L.so_lookup.restype = C.c_int
        L.so_lookup.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p]
        L.so_draft.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p]
        L.so_verify.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.so_update.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.so_step.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p] + [C.c_void_p] * 4
        L.so_update_drops.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.so_table_size.restype = C.c_int64
        L.so_table_size.argtypes = [C.c_void_p]
        L.so_table_export.restype = C.c_int64
        L.so_table_export.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64]
        L.so_get_stats.argtypes = [C.c_void_p, C.POINTER(Stats)]
        L.so_get_node_counts.argtypes = [C.c_void_p, C.c_void_p]
        L.so_tree_packing.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        L.so_reset_node_counts.argtypes = [C.c_void_p]
        L.so_mc_draft.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_uint64, C.c_uint64, C.c_int, C.c_void_p]
        L.so_mc_node.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_int, C.c_uint64, C.c_uint64, C.c_int,
                                 C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.so_mc_draw.argtypes = [C.c_void_p, C.c_int, C.c_uint64, C.c_int, C.c_void_p, C.c_void_p, C.c_float,
                                 C.c_uint64, C.c_uint64, C.c_void_p]
        _lib = L
    return _lib


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _dtype_code(row):
    if row.dtype == np.float32:
        return DT_F32
    if row.dtype == np.uint16:
        return DT_BF16
    raise TypeError("logits must be float32 or uint16 (bf16 bit patterns)")


# ---- stateless pieces -------------------------------------------------------------------
def uniform(seed, b, step, node, token, stream):
    return float(lib().so_uniform(seed, b, step, node, token, stream))


def philox(seed, c0, c1, c2, c3):
    out = np.zeros(4, np.uint32)
    lib().so_philox(seed, c0, c1, c2, c3, _p(out))
    return out


def exp2(y):
    return float(lib().so_exp2(np.float32(y)))


def log(x):
    return float(lib().so_log(np.float32(x)))


def row_softmax(row, temperature, want_p=True):
    row = np.ascontiguousarray(row)
    V = row.shape[0]
    p = np.empty(V, np.float32) if want_p else None
    m = C.c_float()
    s = C.c_float()
    S = C.c_uint64()
    lib().so_row_softmax(_p(row), _dtype_code(row), V, temperature, _p(p) if want_p else None,
                         C.byref(m), C.byref(s), C.byref(S))
    return p, m.value, s.value, S.value


def topk(vals, k):
    vals = _f32(vals)
    idx = np.empty(k, np.int32)
    val = np.empty(k, np.float32)
    lib().so_topk(_p(vals), vals.shape[0], k, _p(idx), _p(val))
    return idx, val


def row_obs(row, temperature, K):
    row = np.ascontiguousarray(row)
    idx = np.empty(K, np.int32)
    p = np.empty(K, np.float32)
    m = C.c_float()
    s = C.c_float()
    lib().so_row_obs(_p(row), _dtype_code(row), row.shape[0], temperature, K, _p(idx), _p(p), C.byref(m), C.byref(s))
    return idx, p, m.value, s.value


def merge(count, ids, mu, obs_ids, obs_p):
    ids, obs_ids = _i32(ids), _i32(obs_ids)
    mu, obs_p = _f32(mu), _f32(obs_p)
    K = ids.shape[0]
    ids2 = np.empty(K, np.int32)
    mu2 = np.empty(K, np.float32)
    lib().so_merge(count, _p(ids), _p(mu), K, _p(obs_ids), _p(obs_p), _p(ids2), _p(mu2))
    return ids2, mu2


def fingerprint(tokens):
    t = _i32(tokens)
    return int(lib().so_fingerprint(t.shape[0], _p(t)))


def gumbel_topk(ids, mu, c, U):
    ids, mu, U = _i32(ids), _f32(mu), _f32(U)
    out = np.full(c, -1, np.int32)
    n = lib().so_gumbel_topk(_p(ids), _p(mu), ids.shape[0], c, _p(U), _p(out))
    return out[:n]


def multinomial_wor(ids, mu, c, U):
    ids, mu, U = _i32(ids), _f32(mu), _f32(U)
    out = np.full(c, -1, np.int32)
    n = lib().so_multinomial_wor(_p(ids), _p(mu), ids.shape[0], c, _p(U), _p(out))
    return out[:n]


def top_c(ids, mu, c):
    ids, mu = _i32(ids), _f32(mu)
    out = np.full(c, -1, np.int32)
    n = lib().so_top_c(_p(ids), _p(mu), ids.shape[0], c, _p(out))
    return out[:n]


def verify_node(p, ids, mu, child_tok, omega, onehot=False):
    p, ids, mu = _f32(p), _i32(ids), _f32(mu)
    child_tok, omega = _i32(child_tok), _f32(omega)
    st = NodeState()
    acc = lib().so_verify_node(_p(p), ids.shape[0], _p(ids), _p(mu), child_tok.shape[0], _p(child_tok), _p(omega), C.byref(st), int(onehot))
    return acc, st


def residual_dense(p, ids, st):
    p, ids = _f32(p), _i32(ids)
    r = np.empty_like(p)
    lib().so_residual_dense(_p(p), p.shape[0], ids.shape[0], _p(ids), C.byref(st) if st is not None else None, _p(r))
    return r


def uniform_u64(seed, b, step, node, stream):
    return int(lib().so_uniform_u64(seed, b, step, node, stream))


def row_masses(row, temperature):
    row = np.ascontiguousarray(row)
    F = np.empty(row.shape[0], np.uint64)
    lib().so_row_masses(_p(row), _dtype_code(row), row.shape[0], temperature, _p(F))
    return F


def residual_draw(F, S, ids, st, u):
    """st: NodeState or None (no proposal); ids may be empty when st is None."""
    F = np.ascontiguousarray(F, np.uint64)
    ids = _i32(ids)
    return int(lib().so_residual_draw(_p(F), F.shape[0], int(S), ids.shape[0], _p(ids),
                                      C.byref(st) if st is not None else None, int(u)))


def mc_gumbel_topk(ids, mu, c, trials, seed, mode=DRAFT_GUMBEL_TOPK):
    ids, mu = _i32(ids), _f32(mu)
    K = ids.shape[0]
    counts = np.zeros(K ** c, np.uint64)
    lib().so_mc_draft(_p(ids), _p(mu), K, c, trials, seed, mode, _p(counts))
    return counts


def mc_node(p, ids, mu, c, trials, seed, mode=DRAFT_GUMBEL_TOPK):
    p, ids, mu = _f32(p), _i32(ids), _f32(mu)
    counts = np.zeros(p.shape[0], np.uint64)
    acc = C.c_uint64()
    near = C.c_uint64()
    err = C.c_double()
    mn = C.c_double()
    lib().so_mc_node(_p(p), p.shape[0], ids.shape[0], _p(ids), _p(mu), c, trials, seed, mode, _p(counts),
                     C.byref(acc), C.byref(near), C.byref(err), C.byref(mn))
    return counts, acc.value, near.value, err.value, mn.value


def mc_draw(F, S, ids, r, rho, trials, seed):
    F = np.ascontiguousarray(F, np.uint64)
    ids, r = _i32(ids), _f32(r)
    counts = np.zeros(F.shape[0], np.uint64)
    lib().so_mc_draw(_p(F), F.shape[0], int(S), ids.shape[0], _p(ids), _p(r), float(rho), trials, seed, _p(counts))
    return counts


# ---- stateful oracle --------------------------------------------------------------------
class Oracle:
    """One shared n-gram table + B trajectories, driven step by step."""

    def __init__(self, vocab, max_batch, order_min, order_max, topk, tree_parent, temperature,
                 table_capacity, max_probe, seed, logits_dtype, update_mode=0, draft_mode=DRAFT_GUMBEL_TOPK,
                 merge_policy=MERGE_MEAN):
        self._parent = _i32(tree_parent)
        cfg = _Config(vocab, max_batch, order_min, order_max, topk, self._parent.shape[0],
                      self._parent.ctypes.data_as(C.POINTER(C.c_int32)), temperature, table_capacity,
                      max_probe, seed, logits_dtype, update_mode, draft_mode, merge_policy)
        self.h = lib().so_create(C.byref(cfg))
        self.B, self.N, self.K, self.V = max_batch, self._parent.shape[0], topk, vocab
        self.D = int(lib().so_depth(self.h))
        self.W = self.D + 1
        self.dtype = logits_dtype

    def close(self):
        if self.h:
            lib().so_destroy(self.h)
            self.h = None

    def __del__(self):
        self.close()

    def _check_logits(self, logits):
        want = np.float32 if self.dtype == DT_F32 else np.uint16
        assert logits.dtype == want and logits.flags.c_contiguous
        assert logits.size == self.B * self.N * self.V

    def set_context(self, b, tokens):
        t = _i32(tokens)
        lib().so_set_context(self.h, b, _p(t), t.shape[0])

    def reorder(self, src_of):
        s = _i32(src_of)
        lib().so_reorder(self.h, _p(s))

    def context_len(self, b):
        return int(lib().so_context_len(self.h, b))

    def context_tail(self, b, n):
        out = np.empty(n, np.int32)
        lib().so_context_tail(self.h, b, n, _p(out))
        return out

    def table_put(self, tokens, count, ids, mu):
        t, ids, mu = _i32(tokens), _i32(ids), _f32(mu)
        return lib().so_table_put(self.h, t.shape[0], _p(t), count, _p(ids), _p(mu))

    def lookup(self, ctx):
        c = _i32(ctx)
        ids = np.empty(self.K, np.int32)
        mu = np.empty(self.K, np.float32)
        cnt = C.c_uint32()
        n = lib().so_lookup(self.h, _p(c), c.shape[0], _p(ids), _p(mu), C.byref(cnt))
        return n, ids, mu, cnt.value

    def draft(self, step):
        out = np.empty((self.B, self.N), np.int32)
        lib().so_draft(self.h, step, _p(out))
        return out

    def verify(self, step, logits):
        self._check_logits(logits)
        tok = np.empty((self.B, self.W), np.int32)
        node = np.empty((self.B, self.W), np.int32)
        ln = np.empty(self.B, np.int32)
        lib().so_verify(self.h, step, _p(logits), _p(tok), _p(node), _p(ln))
        return tok, node, ln

    def update(self, step, logits, commit_tok, commit_row, commit_len, drops=None):
        """drops: optional uint8 flags, one per record (b, position or node, order): these records are dropped and
        all others applied (the capacity model is then off), see so_update_drops."""
        self._check_logits(logits)
        ct, cr, cl = _i32(commit_tok), _i32(commit_row), _i32(commit_len)
        assert ct.shape == (self.B, self.W) and cr.shape == (self.B, self.W) and cl.shape == (self.B,)
        if drops is None:
            lib().so_update(self.h, step, _p(logits), _p(ct), _p(cr), _p(cl))
        else:
            d = np.ascontiguousarray(drops, dtype=np.uint8).reshape(-1)
            lib().so_update_drops(self.h, step, _p(logits), _p(ct), _p(cr), _p(cl), _p(d))

    def step(self, step, logits):
        self._check_logits(logits)
        tok = np.empty((self.B, self.W), np.int32)
        node = np.empty((self.B, self.W), np.int32)
        ln = np.empty(self.B, np.int32)
        nxt = np.empty((self.B, self.N), np.int32)
        lib().so_step(self.h, step, _p(logits), _p(tok), _p(node), _p(ln), _p(nxt))
        return tok, node, ln, nxt

    def table_export(self):
        n = int(lib().so_table_size(self.h))
        es = 16 + 8 * self.K
        buf = np.zeros(max(n, 1) * es, np.uint8)
        got = lib().so_table_export(self.h, _p(buf), buf.shape[0])
        assert got == n
        return parse_table_export(buf[: n * es], self.K)

    def stats(self):
        s = Stats()
        lib().so_get_stats(self.h, C.byref(s))
        return s

    def node_counts(self):
        out = np.zeros(self.N, np.uint64)
        lib().so_get_node_counts(self.h, _p(out))
        return out

    def tree_packing(self):
        mask = np.zeros((self.B, self.N, self.N), np.uint8)
        pos = np.zeros((self.B, self.N), np.int64)
        lib().so_tree_packing(self.h, _p(mask), _p(pos))
        return mask, pos

    def reset_node_counts(self):
        lib().so_reset_node_counts(self.h)


def parse_table_export(buf, K):
    """Split an exported table (entries sorted by fingerprint) into arrays."""
    es = 16 + 8 * K
    n = buf.shape[0] // es
    rec = np.frombuffer(buf.tobytes(), dtype=np.dtype([
        ("fp", "<u8"), ("count", "<u4"), ("order", "<u4"), ("ids", "<i4", (K,)), ("mu", "<f4", (K,))]), count=n)
    return rec


# ---- data-driven draft tree (Sec. 4.3, App. "Initial tree for optimization") -----------------------
def tree_initial(levels=20):
    """The large initial tree of the tree optimisation (appendix "Initial tree for optimization", Alg. 1), as parent[].

    Level by level, on whole levels at once.  A level is described by two arrays: each node's rank r among its
    siblings and its number of siblings s (itself included).  Its fan-outs follow from them -- depth 0: 8;
    depth 1: max(8 - 2r, 1); deeper: ceil((s - 1) / (0.7 r + 1)), at least 2 at depths 2 and 3; the first node of
    a level at least 3 -- and the next level is their expansion: fan-out f contributes ranks 0..f-1 with s = f,
    and the parents' ids repeat f times.  Ids are handed out level after level, so the numbering is breadth first
    with the children of a node contiguous in rank order.  levels = 20 gives the paper's 625 nodes of depth 20.
    """
    parent = [np.array([-1], np.int64)]
    rank, sibs = np.zeros(1, np.int64), np.ones(1, np.int64)
    first_id = 0
    for depth in range(levels):
        if depth == 0:
            fan = np.full(1, 8, np.int64)
        elif depth == 1:
            fan = np.maximum(8 - 2 * rank, 1)
        else:
            fan = np.ceil((sibs - 1) / (0.7 * rank + 1.0)).astype(np.int64)
            if depth <= 3:
                fan = np.maximum(fan, 2)
        fan[0] = max(int(fan[0]), 3)
        total = int(fan.sum())
        if total == 0:
            break
        ids = first_id + np.arange(len(fan), dtype=np.int64)
        parent.append(np.repeat(ids, fan))
        starts = np.repeat(np.cumsum(fan) - fan, fan)
        rank = np.arange(total, dtype=np.int64) - starts
        sibs = np.repeat(fan, fan)
        first_id += len(fan)
    return np.concatenate(parent).astype(np.int32)


def tree_select(parent, counts, n_keep):
    """Keeps the n_keep most often accepted nodes of a tree and re-packs them into a tree of that size
    (paper Sec. 4.3; there n_keep = 80).

    A node can only be used if all its ancestors are, so a node counts as often as the least
    counted node on its way to the root; nodes are ranked by (that count descending, depth
    ascending, id ascending) and the first n_keep are kept.  They are renumbered by (depth, old
    id), which is again breadth first with siblings contiguous in their old rank order.
    Returns (new parent[], old id of every new node).
    """
    parent = np.asarray(parent, np.int64)
    counts = np.asarray(counts, np.uint64)
    n = parent.shape[0]
    assert 1 <= n_keep <= n
    depth = np.zeros(n, np.int64)
    eff = [int(c) for c in counts]
    eff[0] = max(eff)                       # the root is on every path
    for u in range(1, n):
        depth[u] = depth[parent[u]] + 1
        eff[u] = min(eff[u], eff[parent[u]])
    order = sorted(range(n), key=lambda u: (-eff[u], depth[u], u))
    kept = sorted(order[:n_keep], key=lambda u: (depth[u], u))
    new_id = {u: i for i, u in enumerate(kept)}
    new_parent = np.array([-1 if u == 0 else new_id[int(parent[u])] for u in kept], np.int32)
    return new_parent, np.asarray(kept, np.int32)
