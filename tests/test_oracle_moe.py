"""Pins for oracle/moe.py (CPU only): library routines, special cases, finite
differences and autograd of an independently written dense layer."""
import numpy as np
import torch

import workloads as wl
from oracle import moe, router, sched


def tiny_layer(seed=0, T=24, d=8, f=12, E=5, K=2):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((T, d))
    W = [(rng.standard_normal((d, f)) * 0.3, rng.standard_normal((d, f)) * 0.3,
          rng.standard_normal((f, d)) * 0.3) for _ in range(E)]
    logits = rng.standard_normal((T, E))
    idx, w = router.topk_from_logits(logits, K)
    return x, W, idx, w


def test_single_expert_is_a_plain_swiglu_mlp():
    """K=1, E=1, G=1: the layer is one dense MLP; compare with torch's own
    silu and matmul."""
    x, W, _, _ = tiny_layer(E=1, K=1)
    idx = np.zeros((x.shape[0], 1), dtype=np.int32)
    w = np.ones((x.shape[0], 1))
    got = moe.dense_reference(x, idx, w, lambda e: W[e])
    xt = torch.from_numpy(x)
    Wg, Wu, Wd = (torch.from_numpy(a) for a in W[0])
    want = (torch.nn.functional.silu(xt @ Wg) * (xt @ Wu)) @ Wd
    assert np.allclose(got, want.numpy(), rtol=1e-13, atol=1e-14)


def test_zero_gate_weights_give_zero_output():
    x, W, idx, w = tiny_layer()
    W0 = [(np.zeros_like(a), b, c) for (a, b, c) in W]
    assert not moe.dense_reference(x, idx, w, lambda e: W0[e]).any()


def test_scheduled_path_equals_dense_reference():
    """Section 3: any replica computes a token equivalently, so the scheduled
    layer equals the unscheduled per-token definition."""
    x, W, idx, w = tiny_layer(T=32, E=8)
    ref = moe.dense_reference(x, idx, w, lambda e: W[e])
    ref2 = moe.dense_reference_by_expert(x, idx, w, lambda e: W[e])
    assert np.allclose(ref, ref2, rtol=1e-13, atol=1e-15)
    sub = moe.dense_reference_by_expert(x, idx, w, lambda e: W[e], tokens=np.array([5, 0, 17]))
    assert np.allclose(sub, ref[[5, 0, 17]], rtol=1e-13, atol=1e-15)
    for place in (None, wl.placement_complete_plus_matching(4), wl.placement_home(8, 4)):
        s = sched.schedule(idx, 8, 4, place)
        xp = moe.permute(x, s["pair_of_row"], idx.shape[1])
        yp = moe.grouped_ffn(xp, s["seg_off"], lambda e: W[e])
        out = moe.combine(yp, s["row_of_pair"], w)
        assert np.abs(out - ref).max() <= 1e-12 * np.abs(ref).max()


def torch_dense_layer(x, Wg, Wu, Wd, idx, w):
    """Independent dense formulation: every expert on every token, masked."""
    T, d = x.shape
    E = Wg.shape[0]
    out = torch.zeros_like(x)
    for e in range(E):
        y = (torch.nn.functional.silu(x @ Wg[e]) * (x @ Wu[e])) @ Wd[e]
        coef = torch.zeros(T, dtype=x.dtype)
        for k in range(idx.shape[1]):
            coef = coef + torch.where(torch.from_numpy(idx[:, k] == e), w[:, k], torch.zeros(T, dtype=x.dtype))
        out = out + coef[:, None] * y
    return out


def test_backward_against_autograd_and_finite_differences():
    x, W, idx, w = tiny_layer(seed=3, T=16, d=6, f=10, E=4, K=2)
    rng = np.random.default_rng(7)
    d_out = rng.standard_normal(x.shape)
    g = moe.backward_dense(x, idx, w, lambda e: W[e], d_out)

    xt = torch.from_numpy(x).requires_grad_()
    wt = torch.from_numpy(w).requires_grad_()
    Wg = torch.from_numpy(np.stack([a for a, _, _ in W])).requires_grad_()
    Wu = torch.from_numpy(np.stack([b for _, b, _ in W])).requires_grad_()
    Wd = torch.from_numpy(np.stack([c for _, _, c in W])).requires_grad_()
    out = torch_dense_layer(xt, Wg, Wu, Wd, idx, wt)
    assert np.allclose(out.detach().numpy(), moe.dense_reference(x, idx, w, lambda e: W[e]), rtol=1e-12, atol=1e-14)
    (out * torch.from_numpy(d_out)).sum().backward()
    assert np.allclose(g["d_x"], xt.grad.numpy(), rtol=1e-10, atol=1e-12)
    assert np.allclose(g["d_topk_w"], wt.grad.numpy(), rtol=1e-10, atol=1e-12)
    for e in range(4):
        if e in g["d_w_gate"]:
            assert np.allclose(g["d_w_gate"][e], Wg.grad[e].numpy(), rtol=1e-10, atol=1e-12)
            assert np.allclose(g["d_w_up"][e], Wu.grad[e].numpy(), rtol=1e-10, atol=1e-12)
            assert np.allclose(g["d_w_down"][e], Wd.grad[e].numpy(), rtol=1e-10, atol=1e-12)
        else:
            assert not Wg.grad[e].any()

    # central finite differences on a few coordinates
    eps = 1e-6
    base = lambda xx, ww, WW: moe.layer_loss(xx, idx, ww, lambda e: WW[e], d_out)
    for (t, j) in [(0, 0), (5, 3), (15, 5)]:
        xp = x.copy(); xp[t, j] += eps
        xm = x.copy(); xm[t, j] -= eps
        fd = (base(xp, w, W) - base(xm, w, W)) / (2 * eps)
        assert abs(fd - g["d_x"][t, j]) <= 1e-6 * max(1.0, abs(fd))
    for (t, k) in [(1, 0), (9, 1)]:
        wp = w.copy(); wp[t, k] += eps
        wm = w.copy(); wm[t, k] -= eps
        fd = (base(x, wp, W) - base(x, wm, W)) / (2 * eps)
        assert abs(fd - g["d_topk_w"][t, k]) <= 1e-6 * max(1.0, abs(fd))
    e = int(idx[0, 0])
    for which, key, (i, j) in [(0, "d_w_gate", (2, 4)), (1, "d_w_up", (0, 9)), (2, "d_w_down", (7, 1))]:
        Wp = [list(t3) for t3 in W]; Wm = [list(t3) for t3 in W]
        Wp[e][which] = W[e][which].copy(); Wp[e][which][i, j] += eps
        Wm[e][which] = W[e][which].copy(); Wm[e][which][i, j] -= eps
        fd = (base(x, w, Wp) - base(x, w, Wm)) / (2 * eps)
        assert abs(fd - g[key][e][i, j]) <= 1e-6 * max(1.0, abs(fd))


def test_workload_generator_shapes_and_determinism():
    cfg = wl.CONFIGS["cfg1_tiny_f32"]
    a = wl.make_inputs(cfg)
    b = wl.make_inputs(cfg)
    assert a.x.shape == (256, 128) and a.w_gate.shape == (8, 128, 256) and a.w_down.shape == (8, 256, 128)
    assert torch.equal(a.x, b.x) and torch.equal(a.w_up, b.w_up) and torch.equal(a.bias, b.bias)
    assert abs(float(a.w_gate.std()) - 0.02) < 1e-3 and abs(float(a.x.std()) - 1.0) < 2e-2
    g, u, dn = wl.expert_weights(cfg, 3)
    assert torch.equal(g, a.w_gate[3]) and torch.equal(dn, a.w_down[3])
    c5 = wl.scaled(wl.CONFIGS["cfg5_train"], T=64, d=32, f=64)
    i5 = wl.make_inputs(c5)
    assert i5.bias[0] == 4.0 and not i5.bias[1:].any() and i5.d_out.shape == (64, 32)
    assert i5.x.dtype == torch.bfloat16


def test_weight_grad_columns_match_the_full_gradients():
    x, W, idx, w = tiny_layer(seed=5, T=20, d=6, f=9, E=3, K=2)
    d_out = np.random.default_rng(1).standard_normal(x.shape)
    g = moe.backward_dense(x, idx, w, lambda e: W[e], d_out)
    for e in g["d_w_gate"]:
        tt, kk = np.nonzero(idx == e)
        cols = moe.weight_grad_columns(x[tt], w[tt, kk][:, None] * d_out[tt], *W[e], cols=[0, 4, 8])
        for j, (cg, cu, cd) in cols.items():
            assert np.allclose(cg, g["d_w_gate"][e][:, j], rtol=1e-12, atol=1e-14)
            assert np.allclose(cu, g["d_w_up"][e][:, j], rtol=1e-12, atol=1e-14)
            assert np.allclose(cd, g["d_w_down"][e][j, :], rtol=1e-12, atol=1e-14)
