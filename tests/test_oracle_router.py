"""Pins for oracle/router.py (CPU only)."""
import numpy as np

from oracle import router


def test_topk_against_python_sort_and_invariants():
    rng = np.random.default_rng(0)
    for (T, E, K) in [(7, 5, 1), (33, 8, 2), (20, 16, 8), (5, 4, 4)]:
        logits = rng.standard_normal((T, E))
        logits[0, :] = 0.25                       # a full tie: lowest indices win, in order
        idx, w = router.topk_from_logits(logits, K)
        for t in range(T):
            want = sorted(range(E), key=lambda e: (-logits[t, e], e))[:K]
            assert idx[t].tolist() == want
            assert len(set(idx[t].tolist())) == K
        assert (idx >= 0).all() and (idx < E).all()
        assert (w > 0).all() and np.allclose(w.sum(axis=1), 1.0, atol=1e-15)
        # softmax over the selected logits: ratios of weights are exp of logit differences
        sel = np.take_along_axis(logits, idx.astype(np.int64), axis=1)
        assert np.allclose(np.log(w[:, :1] / w), sel[:, :1] - sel, atol=1e-12)
        i2, w2 = router.topk_from_logits_fast(logits, K)
        assert (i2 == idx).all() and np.allclose(w2, w, rtol=0, atol=1e-15)


def test_logits_match_a_hand_computation():
    x = np.array([[1.0, 2.0], [0.5, -1.0]])
    w = np.array([[1.0, 0.0, 2.0], [0.0, 1.0, -1.0]])
    b = np.array([0.0, 10.0, 0.5])
    got = router.router_logits(x, w, b)
    assert np.array_equal(got, np.array([[1.0, 12.0, 0.5], [0.5, 9.0, 2.5]]))
    assert np.array_equal(router.router_logits(x, w, None), got - b[None, :])


def test_kth_gap():
    logits = np.array([[3.0, 1.0, 2.5, 0.0]])
    assert router.kth_gap(logits, 1)[0] == 0.5
    assert router.kth_gap(logits, 2)[0] == 1.5
    assert np.isinf(router.kth_gap(logits, 4)[0])
