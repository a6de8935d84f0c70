"""The seeded input generators that both the oracle and the library read (CPU only): what they promise
about shape, validity and reproducibility.  They hold none of the method's arithmetic."""
import numpy as np

import workloads as wl


def test_drifting_stream_is_valid_reproducible_and_moves():
    T, E, K, n = 512, 24, 3, 5
    a = list(wl.drifting_topk_stream(T, E, K, n, seed=7, skew=1.2, drift=0.3))
    b = list(wl.drifting_topk_stream(T, E, K, n, seed=7, skew=1.2, drift=0.3))
    c = list(wl.drifting_topk_stream(T, E, K, n, seed=8, skew=1.2, drift=0.3))
    assert len(a) == n
    for x, y in zip(a, b):
        assert x.shape == (T, K) and x.dtype == np.int32
        assert np.array_equal(x, y)                                   # a function of its arguments
        assert x.min() >= 0 and x.max() < E
        assert all(len(set(row)) == K for row in x.tolist())          # distinct experts per token
    assert any(not np.array_equal(x, z) for x, z in zip(a, c))
    loads = [np.bincount(x.ravel(), minlength=E) for x in a]
    assert all(int(l.sum()) == T * K for l in loads)
    assert loads[0].max() > 2 * loads[0].mean()                       # skewed
    assert np.abs(loads[-1] - loads[0]).sum() > np.abs(loads[1] - loads[0]).sum() * 0.5 > 0      # and drifting


def test_zipf_loads_and_random_topk():
    load = wl.zipf_loads(32, 10000, 1.3, seed=3)
    assert load.sum() == 10000 and load.min() >= 0 and len(load) == 32
    srt = np.sort(load)[::-1]
    assert srt[0] > 5 * srt[8]                                        # i^(-1.3): the 9th is 17 times lighter
    assert np.array_equal(load, wl.zipf_loads(32, 10000, 1.3, seed=3))
    idx = wl.random_topk(300, 10, 4, seed=1, skew=1.5)
    assert idx.shape == (300, 4) and idx.dtype == np.int32
    assert all(len(set(r)) == 4 for r in idx.tolist()) and idx.min() >= 0 and idx.max() < 10


def test_placements_have_the_shapes_the_paper_gives():
    """Appendix B: Example 1 a cycle (every rank two experts, every expert two ranks), Example 2 the 4 x 4
    torus (16 ranks, 32 experts, degree 4), Example 3 K_{4,4} (8 ranks, 16 experts), Example 4's recipe for
    8 ranks (28 + 4 experts)."""
    for place, E, G, per_rank in ((wl.placement_cycle(8), 8, 8, 2), (wl.placement_torus4x4(), 32, 16, 4),
                                  (wl.placement_z2xz4(), 16, 8, 4), (wl.placement_complete_plus_matching(8), 32, 8, 8)):
        assert place.shape == (E, G) and place.dtype == np.uint8
        assert (place.sum(axis=1) == 2).all()                         # an expert is an edge: two ranks
        assert (place.sum(axis=0) == per_rank).all()                  # regular: every rank the same degree
    k44 = wl.placement_z2xz4()
    side = {g: None for g in range(8)}
    # bipartite: colour ranks along edges, no edge inside a side
    side[0] = 0
    for _ in range(8):
        for e in range(16):
            a, b = np.nonzero(k44[e])[0]
            if side[a] is not None and side[b] is None: side[b] = 1 - side[a]
            if side[b] is not None and side[a] is None: side[a] = 1 - side[b]
    assert all(side[np.nonzero(k44[e])[0][0]] != side[np.nonzero(k44[e])[0][1]] for e in range(16))
    assert sorted(side.values()) == [0] * 4 + [1] * 4
    home = wl.placement_home(32, 8)
    assert (home.sum(axis=1) == 1).all() and (home.sum(axis=0) == 4).all()
    assert wl.placement_full(5, 3).all()
