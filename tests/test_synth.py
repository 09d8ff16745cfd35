"""Input generators (no method arithmetic): the array form of the peaked-token recipe equals its definition by
loops, and the workloads have the structure the configurations name."""
import numpy as np

from paper_2506_04708_amd import synth


def _random_drafts(w, r):
    d = np.full((w.B, w.N), -1, np.int64)
    for b in range(w.B):
        d[b, 0] = w.streams[b, w.pos[b]]
        for u in range(1, w.N):
            if d[b, w.parent[u]] >= 0 and r.random() < 0.8:
                d[b, u] = w.streams[b, w.pos[b] + w.depth[u]] if r.random() < 0.5 else r.integers(w.V)
    return d


def test_peaked_tokens_array_form_equals_the_loops():
    r = np.random.default_rng(0)
    for name, over in [("cfg1", dict(V=40, B=3)), ("cfg3", dict(V=5000, B=8)), ("cfg5", dict(V=300, B=4)),
                       ("cfg3", dict(V=48, B=4, max_peaks=1)), ("cfg1", dict(V=33, B=2))]:
        w = synth.Workload(name, run_steps=20, **over)
        for step in range(5):
            d = _random_drafts(w, r)
            assert np.array_equal(w.peaks(step, d), w.peaks_by_loops(step, d)), (name, step)
            w.pos += r.integers(1, 3, size=w.B)
        # near the end of a stream the continuation is shorter than the tree is deep
        w.pos[:] = w.streams.shape[1] - 3
        d = _random_drafts(w, r) if False else np.full((w.B, w.N), -1, np.int64)
        d[:, 0] = 1
        assert np.array_equal(w.peaks(7, d), w.peaks_by_loops(7, d))
