"""fine_sched_static (the scheduler for callers that cannot allocate: its tables live in a static
array of the library's device image) against fine_sched, through the C ABI: every output
bit-equal, on two calls in a row of which the second is the smaller problem, so that what the
first call left in the shared array must not matter."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2511_16947_amd as fm
import workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda"

OUTPUTS = ("load", "input_eg", "x_eg", "max_load", "pair_dst", "row_of_pair", "pair_of_row", "seg_off", "rank_off")


def run_both(T, E, K, G, seed, skew, place):
    shape = fm.Shape(T, 64, 64, E, K, G)
    idx = torch.from_numpy(wl.random_topk(T, E, K, seed=seed, skew=skew)).to(DEV)
    pl = None if place is None else torch.from_numpy(place).to(DEV)
    a, b = fm.SchedBuffers(shape, DEV), fm.SchedBuffers(shape, DEV)
    for name in OUTPUTS:                         # stale contents must be overwritten
        getattr(a, name).fill_(-7)
        getattr(b, name).fill_(-9)
    a.run(shape, idx, pl)
    fm.fine_sched_static(shape, idx, pl, b.load, b.input_eg, b.x_eg, b.max_load, b.pair_dst, b.row_of_pair,
                         b.pair_of_row, b.seg_off, b.rank_off)
    torch.cuda.synchronize()
    for name in OUTPUTS:
        assert torch.equal(getattr(a, name), getattr(b, name)), name
    assert int(a.max_load.cpu()[0]) > 0
    return b


def test_static_scratch_scheduler_matches_fine_sched_on_two_calls_in_a_row():
    # the larger problem first (256 experts on 32 ranks: 2.3 MiB of the 4 MiB array) ...
    print("no-alloc case 1: T=4096 E=256 K=8 G=32, restricted placement", flush=True)
    run_both(4096, 256, 8, 32, seed=3, skew=1.0, place=wl.placement_circulant(256, 32))
    # ... then a smaller one on the same array, every expert on every rank
    print("no-alloc case 2: T=512 E=16 K=2 G=8, full placement", flush=True)
    run_both(512, 16, 2, 8, seed=5, skew=1.5, place=None)
    # and the large one again without a placement
    print("no-alloc case 3: T=4096 E=256 K=8 G=32, full placement", flush=True)
    run_both(4096, 256, 8, 32, seed=4, skew=0.5, place=None)


def test_static_scratch_scheduler_rejects_what_does_not_fit():
    lib = fm.load_library()
    # 1024 experts on 64 ranks: the transfer tables alone take 32 MiB
    big = fm.Shape(64 * 64, 64, 64, 1024, 2, 64)
    assert fm.fine_workspace_bytes(big, fm.WS_SCHED) > (4 << 20)
    one = torch.zeros(16, dtype=torch.int32, device=DEV)
    p = ctypes.c_void_p(one.data_ptr())
    cs = big.c()
    rc = lib.fine_sched_static(ctypes.byref(cs), p, None, p, p, p, p, p, p, p, p, p, None)
    assert rc == fm.FINE_WORKSPACE_TOO_SMALL
    bad = fm.Shape(250, 64, 64, 8, 2, 4).c()            # G does not divide T: as fine_sched
    assert lib.fine_sched_static(ctypes.byref(bad), p, None, p, p, p, p, p, p, p, p, p, None) == fm.FINE_INVALID_ARG
    ok = fm.Shape(256, 64, 64, 8, 2, 4).c()
    assert lib.fine_sched_static(ctypes.byref(ok), None, None, p, p, p, p, p, p, p, p, p, None) == fm.FINE_INVALID_ARG
    torch.cuda.synchronize()
