"""GPU parity of the backward pass against the oracle's closed-form gradients."""
import numpy as np
import pytest
import torch

import paper_2511_16947_amd as fm
import workloads as wl
from oracle import moe
from gpu_common import GpuLayer, check_schedule_against_oracle, max_rel_err, max_rel_err_rows, to64, weights_of_factory

pytestmark = pytest.mark.gpu
DEV = "cuda"
TOL = 2e-2


class GpuBackward:
    def __init__(self, layer: GpuLayer):
        s, dev = layer.shape, layer.inp.x.device
        self.layer = layer
        self.ws = fm.alloc_workspace(s, fm.WS_BACKWARD, dev)
        self.d_x = torch.full((s.T, s.d), float("nan"), dtype=s.torch_dtype, device=dev)
        self.d_topk_w = torch.full((s.T, s.K), float("nan"), dtype=torch.float32, device=dev)
        self.d_wg = torch.full((s.E, s.d, s.f), float("nan"), dtype=torch.float32, device=dev)
        self.d_wu = torch.full((s.E, s.d, s.f), float("nan"), dtype=torch.float32, device=dev)
        self.d_wd = torch.full((s.E, s.f, s.d), float("nan"), dtype=torch.float32, device=dev)

    def run(self, accumulate=False, rank=-1):
        L, i = self.layer, self.layer.inp
        fm.fine_backward(L.shape, rank, i.d_out, L.x_perm, L.y_perm, L.act_save, i.w_gate, i.w_up, i.w_down,
                         L.sb.row_of_pair, L.sb.pair_of_row, L.sb.seg_off, L.topk_w, self.d_x, self.d_topk_w,
                         self.d_wg, self.d_wu, self.d_wd, accumulate, self.ws)
        torch.cuda.synchronize()


def small_train_cfgs():
    c5 = wl.CONFIGS["cfg5_train"]
    return [
        wl.scaled(c5, name="cfg5_small", T=2048, d=128, f=256),
        wl.scaled(c5, name="cfg5_ragged", T=1024, d=192, f=320, E=16, K=2, G=4, bias_kind="scaled_z", bias_scale=1.5),
        wl.scaled(c5, name="cfg5_topk4", T=512, d=256, f=128, E=32, K=4, G=8, bias_kind="scaled_z", bias_scale=2.0),
        # one long segment per expert (K = 1, two experts, one rank): whole 256-row tiles and a ragged
        # tail in the data-gradient kernels, a long contraction in the weight gradients
        wl.scaled(c5, name="cfg5_long", T=1200, d=128, f=192, E=8, K=1, G=1, bias_kind="one_hot", bias_scale=3.0),
        # weight matrices of 320 x 448: the 8-wave weight-gradient kernel (256 x 256 tiles stored straight from
        # the accumulators) with ragged last row and column tiles
        wl.scaled(c5, name="cfg5_wgrad_ragged", T=1024, d=320, f=448, E=4, K=2, G=2, bias_kind="scaled_z", bias_scale=1.0),
    ]


@pytest.mark.parametrize("cfg", small_train_cfgs(), ids=lambda c: c.name)
@pytest.mark.parametrize("tile", [0, 1, 2, 3])
@pytest.mark.parametrize("saved", [False, True, "with_h"])
def test_backward_elementwise(cfg, tile, saved):
    """saved: the pre-activations are recomputed by the backward pass (False), kept by the forward pass (True),
    or kept together with H (FINE_FLAG_ACT_SAVE_H)."""
    print("backward case", cfg.name, "tile", tile, "act_save", saved, flush=True)
    inp = wl.make_inputs(cfg, DEV)
    with_h = saved == "with_h"
    layer = GpuLayer(cfg, inp, fm.FLAG_LOCALITY | (tile << 8) | (fm.FLAG_ACT_SAVE_H if with_h else 0))
    if saved:
        layer.act_save = torch.full((cfg.P * (3 if with_h else 2) * cfg.f,), float("nan"), dtype=torch.bfloat16, device=DEV)
    layer.forward()
    if with_h:
        # behind the pre-activations lies H = silu(A) * B of every row
        ab = layer.act_save[:cfg.P * 2 * cfg.f].view(cfg.P, 2 * cfg.f).double()
        a, b = ab[:, :cfg.f], ab[:, cfg.f:]
        h = layer.act_save[cfg.P * 2 * cfg.f:].view(cfg.P, cfg.f).double()
        assert max_rel_err(h.cpu().numpy(), (a / (1.0 + torch.exp(-a)) * b).cpu().numpy()) <= TOL
    bwd = GpuBackward(layer)
    bwd.run()

    idx = layer.topk_idx.cpu().numpy()
    w = to64(layer.topk_w)
    check_schedule_against_oracle(layer.sb, idx, cfg.E, cfg.G)
    g = moe.backward_dense(to64(inp.x), idx, w, weights_of_factory(inp), to64(inp.d_out))
    assert max_rel_err(to64(bwd.d_x), g["d_x"]) <= TOL
    assert max_rel_err(to64(bwd.d_topk_w), g["d_topk_w"]) <= TOL
    for e in range(cfg.E):
        for got, key in ((bwd.d_wg, "d_w_gate"), (bwd.d_wu, "d_w_up"), (bwd.d_wd, "d_w_down")):
            if e in g[key]:
                assert max_rel_err(to64(got[e]), g[key][e]) <= TOL, (key, e)
            else:
                assert not got[e].any(), (key, e)          # experts without tokens: exact zeros

    if tile in (0, 3) and not saved:
        # accumulate adds to what is there
        before = bwd.d_wd.clone()
        bwd.run(accumulate=True)
        assert max_rel_err(to64(bwd.d_wd), 2.0 * to64(before)) <= 1e-6
        assert max_rel_err_rows(to64(bwd.d_wd).reshape(-1, cfg.d), 2.0 * to64(before).reshape(-1, cfg.d)) <= 1e-6


@pytest.mark.parametrize("tile", [0, 3])
def test_backward_under_a_restricted_placement(tile):
    """Scheduling only relocates work (Section 3): under a restricted placement, where an expert's
    rows sit on several ranks in other proportions, the gradients are those of the dense
    definition all the same, and the weight gradients of an expert are summed over its replicas."""
    cfg = wl.scaled(wl.CONFIGS["cfg5_train"], name="cfg5_placed", T=1024, d=128, f=256, E=16, K=2, G=8,
                    bias_kind="scaled_z", bias_scale=1.5)
    inp = wl.make_inputs(cfg, DEV)
    place = wl.placement_z2xz4()                        # Appendix B Example 3: 16 experts on 8 ranks, two replicas each
    layer = GpuLayer(cfg, inp, fm.FLAG_LOCALITY | (tile << 8))
    layer.act_save = torch.empty(cfg.P, 2 * cfg.f, dtype=torch.bfloat16, device=DEV)
    layer.forward(place=torch.from_numpy(place).to(DEV))
    bwd = GpuBackward(layer)
    bwd.run()
    idx = layer.topk_idx.cpu().numpy()
    want = check_schedule_against_oracle(layer.sb, idx, cfg.E, cfg.G, place)
    seg = want["seg_off"]
    assert ((np.diff(seg, axis=1) > 0).sum(axis=0) == 2).any()       # some expert really runs on both of its ranks
    g = moe.backward_dense(to64(inp.x), idx, to64(layer.topk_w), weights_of_factory(inp), to64(inp.d_out))
    assert max_rel_err(to64(bwd.d_x), g["d_x"]) <= TOL
    assert max_rel_err(to64(bwd.d_topk_w), g["d_topk_w"]) <= TOL
    for e in range(cfg.E):
        for got, key in ((bwd.d_wg, "d_w_gate"), (bwd.d_wu, "d_w_up"), (bwd.d_wd, "d_w_down")):
            if e in g[key]:
                assert max_rel_err(to64(got[e]), g[key][e]) <= TOL, (key, e)
            else:
                assert not got[e].any(), (key, e)


@pytest.mark.parametrize("tile", [0, 3])
@pytest.mark.parametrize("saved", [False, True, "with_h"])
def test_backward_rank_by_rank(tile, saved):
    """One fine_backward call per rank in ascending order (rank 0 overwriting the weight gradients,
    the others adding to them) against one call for all ranks: d_x and d_topk_w bit-equal, the weight
    gradients equal up to fp32 summation order and within tolerance of the oracle.  Under a
    restricted placement, so that experts really are split over ranks."""
    cfg = wl.scaled(wl.CONFIGS["cfg5_train"], name="cfg5_ranks", T=1024, d=128, f=256, E=16, K=2, G=8,
                    bias_kind="scaled_z", bias_scale=1.5)
    inp = wl.make_inputs(cfg, DEV)
    place = torch.from_numpy(wl.placement_z2xz4()).to(DEV)
    with_h = saved == "with_h"
    layer = GpuLayer(cfg, inp, fm.FLAG_LOCALITY | (tile << 8) | (fm.FLAG_ACT_SAVE_H if with_h else 0))
    if saved:
        layer.act_save = torch.empty(cfg.P * (3 if with_h else 2) * cfg.f, dtype=torch.bfloat16, device=DEV)
    layer.forward(place=place)
    whole = GpuBackward(layer)
    whole.run()
    parts = GpuBackward(layer)
    for r in range(cfg.G):
        parts.run(accumulate=(r > 0), rank=r)
    assert torch.equal(parts.d_x.view(torch.int16), whole.d_x.view(torch.int16))
    assert torch.equal(parts.d_topk_w, whole.d_topk_w)
    idx = layer.topk_idx.cpu().numpy()
    g = moe.backward_dense(to64(inp.x), idx, to64(layer.topk_w), weights_of_factory(inp), to64(inp.d_out))
    for got, ref, key in ((parts.d_wg, whole.d_wg, "d_w_gate"), (parts.d_wu, whole.d_wu, "d_w_up"),
                          (parts.d_wd, whole.d_wd, "d_w_down")):
        assert max_rel_err(to64(got), to64(ref)) <= 1e-5, key
        for e in range(cfg.E):
            if e in g[key]:
                assert max_rel_err(to64(got[e]), g[key][e]) <= TOL, (key, e)
            else:
                assert not got[e].any(), (key, e)
    # a rank out of range is an argument error
    with pytest.raises(fm.FineError):
        parts.run(rank=cfg.G)


def test_backward_full_size_cfg5():
    """The training workload at full size, per-rank forward calls as bench.py issues them: every
    element of d_x and d_topk_w, and every element of the three weight gradients of five experts
    (the hottest, whose rows are split over many ranks, the two next, a median one and the least
    loaded), tensor-wide and row by row; the other experts' gradients must be finite."""
    cfg = wl.CONFIGS["cfg5_train"]
    print("full-size backward cfg5", flush=True)
    inp = wl.make_inputs(cfg, DEV)
    layer = GpuLayer(cfg, inp, fm.FLAG_LOCALITY | fm.FLAG_ACT_SAVE_H)      # as bench.py runs it: H kept by the forward pass
    layer.act_save = torch.empty(cfg.P * 3 * cfg.f, dtype=torch.bfloat16, device=DEV)
    layer.forward(per_rank=True)
    bwd = GpuBackward(layer)
    bwd.run()
    print("  backward done", flush=True)
    idx = layer.topk_idx.cpu().numpy()
    w = to64(layer.topk_w)
    want = check_schedule_against_oracle(layer.sb, idx, cfg.E, cfg.G)
    assert not torch.isnan(bwd.d_wg).any() and not torch.isnan(bwd.d_wu).any() and not torch.isnan(bwd.d_wd).any()
    load = want["load"]
    order = np.argsort(-load, kind="stable")
    nonempty = order[load[order] > 0]
    experts = sorted({int(nonempty[0]), int(nonempty[1]), int(nonempty[2]), int(nonempty[len(nonempty) // 2]),
                      int(nonempty[-1])})
    g = moe.backward_dense(to64(inp.x), idx, w, weights_of_factory(inp), to64(inp.d_out), weight_grad_experts=experts)
    print("  oracle done", flush=True)
    for name, got, ref in (("d_x", to64(bwd.d_x), g["d_x"]), ("d_topk_w", to64(bwd.d_topk_w), g["d_topk_w"])):
        e_all = max_rel_err(got, ref)
        e_row = max_rel_err_rows(got, ref) if name == "d_x" else e_all
        print("  %s: every element, max-rel-err %.3e, worst row %.3e" % (name, e_all, e_row), flush=True)
        assert e_all <= TOL and e_row <= TOL
    for e in experts:
        for got, key in ((bwd.d_wg, "d_w_gate"), (bwd.d_wu, "d_w_up"), (bwd.d_wd, "d_w_down")):
            ge, ref = to64(got[e]), g[key][e]
            e_all, e_row = max_rel_err(ge, ref), max_rel_err_rows(ge, ref)
            print("  expert %d (%d rows) %s: max-rel-err %.3e, worst row %.3e" % (e, load[e], key, e_all, e_row), flush=True)
            assert e_all <= TOL and e_row <= TOL, (key, e)


def test_a_training_step_can_be_captured_in_a_graph():
    """Forward pass (keeping the pre-activations and H) and backward pass of a small layer whose GEMMs cut tiles along
    k, captured in one HIP graph: every replay, with eager work and synchronisations in between, gives the bits of
    the eager run (the partial-sum counters and work queues are cleared and waited for inside the kernels)."""
    cfg = wl.scaled(wl.CONFIGS["cfg5_train"], name="graph_train", T=512, d=256, f=2560, E=4, K=2, G=2,
                    bias_kind="scaled_z", bias_scale=1.0)
    inp = wl.make_inputs(cfg, DEV)
    layer = GpuLayer(cfg, inp, fm.FLAG_LOCALITY | (3 << 8) | fm.FLAG_ACT_SAVE_H)
    layer.act_save = torch.empty(cfg.P * 3 * cfg.f, dtype=torch.bfloat16, device=DEV)
    layer.forward(per_rank=True)                           # eager; also sets every kernel attribute before the capture
    bwd = GpuBackward(layer)
    bwd.run()
    want = [t.clone() for t in (layer.out, bwd.d_x, bwd.d_topk_w, bwd.d_wg, bwd.d_wu, bwd.d_wd)]
    g = moe.backward_dense(to64(inp.x), layer.topk_idx.cpu().numpy(), to64(layer.topk_w), weights_of_factory(inp),
                           to64(inp.d_out))
    assert max_rel_err(to64(bwd.d_x), g["d_x"]) <= TOL

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    L, i = layer, inp
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            layer.topk()
            layer.sched(None)
            layer.permute()
            for r in range(cfg.G):
                layer.ffn(r)
            layer.combine()
            fm.fine_backward(L.shape, -1, i.d_out, L.x_perm, L.y_perm, L.act_save, i.w_gate, i.w_up, i.w_down,
                             L.sb.row_of_pair, L.sb.pair_of_row, L.sb.seg_off, L.topk_w, bwd.d_x, bwd.d_topk_w,
                             bwd.d_wg, bwd.d_wu, bwd.d_wd, False, bwd.ws)
    torch.cuda.current_stream().wait_stream(side)
    for n in range(3):
        for t in (layer.out, bwd.d_x, bwd.d_topk_w, bwd.d_wg, bwd.d_wu, bwd.d_wd, layer.act_save):
            t.fill_(float("nan"))
        layer.topk()                                       # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip((layer.out, bwd.d_x, bwd.d_topk_w, bwd.d_wg, bwd.d_wu, bwd.d_wd), want):
            assert torch.equal(got.view(torch.int32 if got.dtype == torch.float32 else torch.int16),
                               ref.view(torch.int32 if ref.dtype == torch.float32 else torch.int16)), n
