"""GPU parity of the warm-started scheduler (Section 4.1: across micro-batches the placement
stays and the loads change, so the solver may start from the previous solution).  Whatever it
starts from, every output must be the oracle's canonical schedule, bit for bit."""
import numpy as np
import pytest
import torch

import paper_2511_16947_amd as fm
import workloads as wl
from oracle import placement as opl
from gpu_common import check_schedule_against_oracle

pytestmark = pytest.mark.gpu
DEV = "cuda"


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def searched_placement(load, G, slots, n=64, seed=3):
    return opl.search(load, G, slots, n, seed)[3]


STREAMS = [
    # name, placement, E, G, K, T, micro-batches, drift
    ("cycle8", lambda load: wl.placement_cycle(8), 8, 8, 2, 2048, 6, 0.10),
    ("k8plus4", lambda load: wl.placement_complete_plus_matching(8), 32, 8, 2, 2048, 6, 0.05),
    ("torus16", lambda load: wl.placement_torus4x4(), 32, 16, 2, 2048, 5, 0.05),
    ("circ256x32_top8", lambda load: wl.placement_circulant(256, 32), 256, 32, 8, 2048, 4, 0.05),
    ("searched_64x16_5slots", lambda load: searched_placement(load, 16, 5), 64, 16, 4, 2048, 6, 0.10),
    ("searched_32x8_fast_drift", lambda load: searched_placement(load, 8, 6), 32, 8, 2, 1024, 6, 0.60),
]


@pytest.mark.parametrize("case", STREAMS, ids=lambda c: c[0])
def test_a_warm_started_stream_gives_the_canonical_schedule_every_time(case):
    name, mk, E, G, K, T, n, drift = case
    batches = list(wl.drifting_topk_stream(T, E, K, n, seed=len(name), skew=1.2, drift=drift))
    place = mk(np.bincount(batches[0].ravel(), minlength=E))
    shape = fm.Shape(T, 64, 64, E, K, G, fm.FINE_BF16, fm.FLAG_LOCALITY)
    sb = fm.SchedBuffers(shape, DEV)
    place_d = dev(place)
    loads = []
    for i, idx in enumerate(batches):
        print("stream", name, "micro-batch", i, flush=True)
        sb.run(shape, dev(idx), place_d, warm=i > 0)       # the first call has nothing to start from
        torch.cuda.synchronize()
        want = check_schedule_against_oracle(sb, idx, E, G, place, True)
        loads.append(np.asarray(want["load"]))
    assert any((a != b).any() for a, b in zip(loads, loads[1:])), "the stream's loads never moved"


def test_any_starting_point_gives_the_same_schedule():
    """x_prev only says where the search starts: zeros, another placement's solution, random
    numbers (negative and huge ones too), or the answer itself all end in the same bits."""
    E, G, K, T = 48, 12, 3, 1536
    idx = wl.random_topk(T, E, K, seed=5, skew=1.4)
    load = np.bincount(idx.ravel(), minlength=E)
    place = searched_placement(load, G, 6)
    shape = fm.Shape(T, 64, 64, E, K, G, fm.FINE_BF16, fm.FLAG_LOCALITY)
    sb = fm.SchedBuffers(shape, DEV)
    idx_d, place_d = dev(idx), dev(place)
    sb.run(shape, idx_d, place_d)
    torch.cuda.synchronize()
    want = check_schedule_against_oracle(sb, idx, E, G, place, True)
    answer = sb.x_eg.clone()
    rng = np.random.default_rng(9)
    other = np.asarray(want["x"]).astype(np.int32)[:, ::-1]            # a solution laid over other ranks
    starts = {
        "zeros": np.zeros((E, G), np.int32),
        "the answer": answer.cpu().numpy(),
        "other ranks": other,
        "random": rng.integers(0, 1000, (E, G), dtype=np.int32),
        "negative and huge": rng.integers(-2**31, 2**31 - 1, (E, G), dtype=np.int64).astype(np.int32),
        "everything on the last replica": np.where(np.cumsum(place[:, ::-1], axis=1)[:, ::-1] == 1, place, 0).astype(np.int32) * 7,
    }
    for name, prev in starts.items():
        print("start from", name, flush=True)
        sb.x_eg.fill_(-5)
        fm.fine_sched_warm(shape, idx_d, place_d, dev(prev), sb.load, sb.input_eg, sb.x_eg, sb.max_load, sb.pair_dst,
                           sb.row_of_pair, sb.pair_of_row, sb.seg_off, sb.rank_off, sb.ws)
        torch.cuda.synchronize()
        check_schedule_against_oracle(sb, idx, E, G, place, True)


def test_warm_start_without_a_placement_is_the_closed_form():
    E, G, K, T = 16, 4, 2, 512
    idx = wl.random_topk(T, E, K, seed=2, skew=1.0)
    shape = fm.Shape(T, 64, 64, E, K, G, fm.FINE_BF16, fm.FLAG_LOCALITY)
    sb = fm.SchedBuffers(shape, DEV)
    sb.x_eg.fill_(123)
    sb.run(shape, dev(idx), None, warm=True)
    torch.cuda.synchronize()
    check_schedule_against_oracle(sb, idx, E, G, None, True)


def test_warm_start_still_reports_an_expert_without_replica():
    E, G, K, T = 8, 4, 2, 256
    idx = wl.random_topk(T, E, K, seed=4, skew=0.5)
    place = wl.placement_circulant(E, G)
    place[3, :] = 0
    shape = fm.Shape(T, 64, 64, E, K, G, fm.FINE_BF16, fm.FLAG_LOCALITY)
    sb = fm.SchedBuffers(shape, DEV)
    sb.x_eg.fill_(9)
    sb.run(shape, dev(idx), dev(place), warm=True)
    torch.cuda.synchronize()
    assert int(sb.max_load.cpu()[0]) == -1
    assert int(sb.x_eg.abs().sum().cpu()) == 0
    assert bool((sb.pair_dst == -1).all().cpu())
    ident = torch.arange(T * K, dtype=torch.int32, device=sb.row_of_pair.device)
    assert torch.equal(sb.row_of_pair, ident) and torch.equal(sb.pair_of_row, ident)
    assert not sb.seg_off.any() and not sb.rank_off.any()


def test_scheduling_on_a_second_stream_gives_the_in_line_results():
    """Section 4.4 hides the scheduling behind other work.  Micro-batch i+1 is gated and scheduled
    (warm-started) on a second stream while micro-batch i runs permute, expert FFN and combine on the
    first, two buffer sets taking turns; every micro-batch's output must have the bits of the run
    that does everything in line on one stream, and its schedule must be the oracle's."""
    cfg = wl.LayerConfig("stream_overlap", 1024, 256, 512, 16, 2, 4, "bf16", 21, "scaled_z", 1.0)
    n = 5
    inp = wl.make_inputs(cfg, DEV)
    s = fm.shape_of(cfg, fm.FLAG_LOCALITY)
    gen = torch.Generator().manual_seed(77)
    biases = [(inp.bias + (0.2 * i) * torch.randn(cfg.E, generator=gen).to(DEV)).contiguous() for i in range(n)]
    place_np = wl.placement_circulant(cfg.E, cfg.G)
    place = dev(place_np)
    topk_idx = [torch.empty(s.T, s.K, dtype=torch.int32, device=DEV) for _ in range(2)]
    topk_w = [torch.empty(s.T, s.K, dtype=torch.float32, device=DEV) for _ in range(2)]
    sbs = [fm.SchedBuffers(s, DEV) for _ in range(2)]
    x_perm = torch.empty(s.P, s.d, dtype=s.torch_dtype, device=DEV)
    y_perm = torch.empty(s.P, s.d, dtype=s.torch_dtype, device=DEV)
    outs = [torch.empty(s.T, s.d, dtype=s.torch_dtype, device=DEV) for _ in range(n)]
    ws_ffn = fm.alloc_workspace(s, fm.WS_FFN, DEV)
    ws_topk = fm.alloc_workspace(s, fm.WS_TOPK, DEV)       # one: the gate calls follow each other on the side stream

    def gate_and_schedule(i):
        b, sb = i & 1, sbs[i & 1]
        fm.fine_topk(s, inp.x, inp.w_router, biases[i], topk_idx[b], topk_w[b], ws_topk)
        fm.fine_sched_warm(s, topk_idx[b], place, sbs[b ^ 1].x_eg if i > 0 else None, sb.load, sb.input_eg, sb.x_eg,
                           sb.max_load, sb.pair_dst, sb.row_of_pair, sb.pair_of_row, sb.seg_off, sb.rank_off, sb.ws)

    def compute(i):
        b, sb = i & 1, sbs[i & 1]
        fm.fine_permute(s, inp.x, sb.pair_of_row, x_perm)
        for r in range(s.G):
            fm.fine_grouped_ffn(s, r, x_perm, inp.w_gate, inp.w_up, inp.w_down, sb.seg_off, y_perm, None, ws_ffn)
        fm.fine_combine(s, y_perm, sb.row_of_pair, topk_w[b], outs[i])

    # in line, one stream; the schedules are checked against the oracle on the way
    want, want_x = [], []
    for i in range(n):
        gate_and_schedule(i)
        compute(i)
        torch.cuda.synchronize()
        check_schedule_against_oracle(sbs[i & 1], topk_idx[i & 1].cpu().numpy(), cfg.E, cfg.G, place_np, True)
        want.append(outs[i].clone())
        want_x.append(sbs[i & 1].x_eg.clone())
        outs[i].zero_()
    assert any(not torch.equal(a, b) for a, b in zip(want_x, want_x[1:])), "the stream's schedules never moved"

    main = torch.cuda.current_stream()
    side = torch.cuda.Stream()
    scheduled = [torch.cuda.Event() for _ in range(n)]
    computed = [torch.cuda.Event() for _ in range(n)]
    for rep in range(2):
        print("two-stream pass", rep, flush=True)
        side.wait_stream(main)
        with torch.cuda.stream(side):
            gate_and_schedule(0)
            scheduled[0].record(side)
        for i in range(n):
            if i + 1 < n:
                with torch.cuda.stream(side):
                    if i >= 1:
                        side.wait_event(computed[i - 1])      # buffer set (i+1)&1 was micro-batch i-1's
                    gate_and_schedule(i + 1)
                    scheduled[i + 1].record(side)
            main.wait_event(scheduled[i])
            compute(i)
            computed[i].record(main)
        main.wait_stream(side)
        torch.cuda.synchronize()
        for i in range(n):
            assert torch.equal(outs[i].view(torch.int16), want[i].view(torch.int16)), (rep, i)
            outs[i].zero_()
