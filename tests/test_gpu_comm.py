"""GPU parity of communication-aware scheduling (Appendix A.1, Eq. 4; fine_sched_comm) against the
oracle: every output bit-exact, and a layer run on such a schedule still computes the dense
definition."""
import numpy as np
import pytest
import torch

import paper_2511_16947_amd as fm
import workloads as wl
from oracle import comm, moe, sched
from gpu_common import GpuLayer, max_rel_err, to64, tol_for, weights_of_factory

pytestmark = pytest.mark.gpu
DEV = "cuda"
OUT = ("load", "input_eg", "x_eg", "pair_dst", "row_of_pair", "pair_of_row", "seg_off", "rank_off")
KEY = dict(load="load", input_eg="input", x_eg="x", pair_dst="pair_dst", row_of_pair="row_of_pair",
           pair_of_row="pair_of_row", seg_off="seg_off", rank_off="rank_off")


def run_comm(shape, idx_dev, place_dev, a, b, rpn):
    sb = fm.SchedBuffers(shape, DEV)
    for name in OUT:
        getattr(sb, name).fill_(-5)
    cc = torch.full((2,), -5, dtype=torch.int32, device=DEV)
    fm.fine_sched_comm(shape, idx_dev, place_dev, a, b, rpn, sb.load, sb.input_eg, sb.x_eg, cc, sb.pair_dst,
                       sb.row_of_pair, sb.pair_of_row, sb.seg_off, sb.rank_off, sb.ws)
    torch.cuda.synchronize()
    return sb, cc.cpu().numpy()


def check(sb, cc, idx, E, G, place, a, b, rpn, locality):
    want = comm.schedule(idx, E, G, place, a, b, rpn, locality)
    assert (int(cc[0]), int(cc[1])) == (want["comp"], -1 if want["comm"] is None else want["comm"])
    for name in OUT:
        got = getattr(sb, name).cpu().numpy().astype(np.int64)
        w = np.asarray(want[KEY[name]]).astype(np.int64)
        assert np.array_equal(got, w), "%s differs (first at %s)" % (name, np.argwhere(got != w)[:3].tolist())
    return want


@pytest.mark.parametrize("locality", [True, False])
@pytest.mark.parametrize("rpn", [0, 2, 4])
def test_comm_aware_schedules_bit_exact(rpn, locality):
    rng = np.random.default_rng(100 + rpn)
    flags = fm.FLAG_LOCALITY if locality else 0
    for trial in range(10):
        E, G = int(rng.integers(2, 40)), int(rng.choice([2, 4, 6, 8, 12, 16]))
        K = int(rng.integers(1, min(E, 4) + 1))
        T = G * int(rng.integers(4, 60))
        if trial % 3 == 0:
            place = None
        else:
            place = np.zeros((E, G), dtype=np.uint8)
            for e in range(E):
                place[e, rng.choice(G, size=int(rng.integers(1, min(G, 4) + 1)), replace=False)] = 1
        a, b = [(0, 1), (1, 10), (1, 1), (5, 2)][trial % 4]
        idx = wl.random_topk(T, E, K, seed=trial, skew=float(rng.uniform(0, 2.5)))
        print("comm-aware case", trial, E, G, K, T, "alpha", a, b, "rpn", rpn, flush=True)
        shape = fm.Shape(T, 64, 64, E, K, G, fm.FINE_BF16, flags)
        sb, cc = run_comm(shape, torch.from_numpy(idx).to(DEV), None if place is None else torch.from_numpy(place).to(DEV),
                          a, b, rpn)
        want = check(sb, cc, idx, E, G, place, a, b, rpn, locality)
        if a == 0 and rpn <= 1:      # Eq. 1 and Algorithm 1: fine_sched's result
            ref = fm.SchedBuffers(shape, DEV)
            ref.run(shape, torch.from_numpy(idx).to(DEV), None if place is None else torch.from_numpy(place).to(DEV))
            torch.cuda.synchronize()
            for name in OUT:
                assert torch.equal(getattr(sb, name), getattr(ref, name)), name
            assert int(ref.max_load.cpu()[0]) == int(cc[0])


def test_comm_aware_full_size_schedules():
    """The two largest routing tables (256 experts on 32 ranks, top-8; 64 experts on 16 ranks with one
    expert holding half of the pairs) under a two-replica placement, alpha_1 = 0.1 and alpha_2 = 1 of
    Appendix C.2, nodes of 8 ranks."""
    for name, a, b in (("cfg4_dsv3", 1, 10), ("cfg5_train", 1, 1)):
        cfg = wl.CONFIGS[name]
        inp = wl.make_inputs(cfg, DEV, with_weights=False)
        shape = fm.shape_of(cfg)
        idx_dev = torch.empty(cfg.T, cfg.K, dtype=torch.int32, device=DEV)
        w = torch.empty(cfg.T, cfg.K, dtype=torch.float32, device=DEV)
        fm.fine_topk(shape, inp.x, inp.w_router, inp.bias, idx_dev, w, fm.alloc_workspace(shape, fm.WS_TOPK, DEV))
        place = wl.placement_circulant(cfg.E, cfg.G)
        print("comm-aware full-size case", name, flush=True)
        sb, cc = run_comm(shape, idx_dev, torch.from_numpy(place).to(DEV), a, b, 8)
        want = check(sb, cc, idx_dev.cpu().numpy(), cfg.E, cfg.G, place, a, b, 8, True)
        # against Eq. 1's schedule on the same table: comp no smaller, comm no larger
        ref = sched.schedule(idx_dev.cpu().numpy(), cfg.E, cfg.G, place)
        comp1, comm1, _, _ = comm.volumes(ref["x"], ref["input"], place)
        print("  Eq. 1: comp %d comm %d;  Eq. 4: comp %d comm %d" % (comp1, comm1, want["comp"], want["comm"]), flush=True)
        assert want["comp"] >= comp1 and want["comm"] <= comm1


def test_comm_aware_reports_an_expert_without_replica_and_bad_arguments():
    T, E, K, G = 64, 4, 1, 4
    idx = wl.random_topk(T, E, K, seed=0, skew=0.0)
    place = wl.placement_full(E, G)
    place[2, :] = 0
    shape = fm.Shape(T, 64, 64, E, K, G)
    sb, cc = run_comm(shape, torch.from_numpy(idx).to(DEV), torch.from_numpy(place).to(DEV), 1, 1, 2)
    assert cc.tolist() == [-1, -1] and not sb.x_eg.any()
    ident = torch.arange(T * K, dtype=torch.int32, device=DEV)
    assert bool((sb.pair_dst == -1).all().cpu()) and torch.equal(sb.row_of_pair, ident) and torch.equal(sb.pair_of_row, ident)
    with pytest.raises(fm.FineError):
        run_comm(shape, torch.from_numpy(idx).to(DEV), None, -1, 1, 0)
    with pytest.raises(fm.FineError):
        run_comm(shape, torch.from_numpy(idx).to(DEV), None, 1, 0, 0)


def test_layer_on_a_comm_aware_schedule_computes_the_dense_definition():
    cfg = wl.scaled(wl.CONFIGS["cfg2_mixtral"], name="cfg2_comm", T=1024, d=256, f=512, E=16, K=2, G=8)
    inp = wl.make_inputs(cfg, DEV)
    layer = GpuLayer(cfg, inp)
    layer.topk()
    place = wl.placement_z2xz4()
    cc = torch.empty(2, dtype=torch.int32, device=DEV)
    sb = layer.sb
    fm.fine_sched_comm(layer.shape, layer.topk_idx, torch.from_numpy(place).to(DEV), 1, 1, 4, sb.load, sb.input_eg, sb.x_eg,
                       cc, sb.pair_dst, sb.row_of_pair, sb.pair_of_row, sb.seg_off, sb.rank_off, sb.ws)
    layer.permute()
    for r in range(cfg.G):
        layer.ffn(r)
    layer.combine()
    torch.cuda.synchronize()
    idx = layer.topk_idx.cpu().numpy()
    check(sb, cc.cpu().numpy(), idx, cfg.E, cfg.G, place, 1, 1, 4, True)
    ref = moe.dense_reference_by_expert(to64(inp.x), idx, to64(layer.topk_w), weights_of_factory(inp))
    assert max_rel_err(to64(layer.out), ref) <= tol_for(cfg)
