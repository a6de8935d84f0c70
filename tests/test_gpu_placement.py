"""GPU parity of the scheduler under restricted placements (the LP of Eq. 1 proper):
every output bit-exact against the oracle's canonical solver."""
import numpy as np
import pytest
import torch

import paper_2511_16947_amd as fm
import workloads as wl
from oracle import sched
from gpu_common import check_schedule_against_oracle
from test_oracle_sched import read_golden

pytestmark = pytest.mark.gpu
DEV = "cuda"


def topk_from_loads(load, seed):
    """K = 1 routing table with exactly the given expert loads, tokens shuffled."""
    idx = np.repeat(np.arange(len(load), dtype=np.int32), np.asarray(load, dtype=np.int64))
    np.random.default_rng(seed).shuffle(idx)
    return idx.reshape(-1, 1)


def run_case(idx, E, G, place, locality=True):
    T, K = idx.shape
    shape = fm.Shape(T, 64, 64, E, K, G, fm.FINE_BF16, fm.FLAG_LOCALITY if locality else 0)
    sb = fm.SchedBuffers(shape, DEV)
    sb.run(shape, torch.from_numpy(idx).to(DEV), torch.from_numpy(np.ascontiguousarray(place)).to(DEV))
    torch.cuda.synchronize()
    return sb, check_schedule_against_oracle(sb, idx, E, G, place, locality)


def test_worked_example_of_section3_on_the_gpu():
    place, load, mstar, xs = read_golden("worked_example_sec3.txt")
    idx = topk_from_loads(load, seed=0)
    sb, want = run_case(idx, 4, 4, place)
    assert int(sb.max_load.cpu()[0]) == mstar == 8
    assert np.array_equal(sb.x_eg.cpu().numpy(), xs)


def test_tie_break_example_on_the_gpu():
    place, load, mstar, xs = read_golden("tie_break_example.txt")
    sb, _ = run_case(topk_from_loads(load, seed=1), 2, 2, place)
    assert np.array_equal(sb.x_eg.cpu().numpy(), xs)


PLACED = [
    ("cycle8_cfg2like", lambda: wl.placement_cycle(8), 8, 8, 2, 8192, 1.0),
    ("k8plus4_zipf05", lambda: wl.placement_complete_plus_matching(8), 32, 8, 2, 4096, 0.5),
    ("k8plus4_zipf20", lambda: wl.placement_complete_plus_matching(8), 32, 8, 2, 4096, 2.0),
    ("torus16", lambda: wl.placement_torus4x4(), 32, 16, 2, 2048, 1.2),
    ("k44", lambda: wl.placement_z2xz4(), 16, 8, 4, 1024, 1.5),
    ("circ128x8_top8", lambda: wl.placement_circulant(128, 8), 128, 8, 8, 1024, 1.3),
    ("circ256x32_top8", lambda: wl.placement_circulant(256, 32), 256, 32, 8, 4096, 1.0),
    ("circ64x16", lambda: wl.placement_circulant(64, 16), 64, 16, 2, 4096, 2.5),
    ("home_vanilla_ep", lambda: wl.placement_home(32, 8), 32, 8, 2, 1024, 1.0),
    ("full_mask_equals_closed_form", lambda: wl.placement_full(16, 4), 16, 4, 2, 512, 1.5),
]


@pytest.mark.parametrize("locality", [True, False])
@pytest.mark.parametrize("case", PLACED, ids=lambda c: c[0])
def test_restricted_placements_bit_exact(case, locality):
    name, mk, E, G, K, T, skew = case
    place = mk()
    assert place.shape == (E, G)
    idx = wl.random_topk(T, E, K, seed=len(name), skew=skew)
    print("placement case", name, "locality", locality, flush=True)
    sb, want = run_case(idx, E, G, place, locality)
    rows = np.diff(want["rank_off"])
    assert rows.max() == want["max_load"]


def test_random_placements_with_varied_replica_counts():
    rng = np.random.default_rng(42)
    for trial in range(12):
        E = int(rng.integers(2, 40)); G = int(rng.choice([2, 3, 4, 6, 8, 12]))
        K = int(rng.integers(1, min(E, 4) + 1))
        T = G * int(rng.integers(4, 60))
        place = np.zeros((E, G), dtype=np.uint8)
        for e in range(E):
            place[e, rng.choice(G, size=int(rng.integers(1, min(G, 4) + 1)), replace=False)] = 1
        idx = wl.random_topk(T, E, K, seed=trial, skew=float(rng.uniform(0, 2.5)))
        print("random placement trial", trial, E, G, K, T, flush=True)
        run_case(idx, E, G, place)


def test_full_mask_gives_the_same_schedule_as_no_mask():
    T, E, K, G = 2048, 64, 2, 16
    idx = wl.random_topk(T, E, K, seed=5, skew=1.7)
    shape = fm.Shape(T, 64, 64, E, K, G)
    a, b = fm.SchedBuffers(shape, DEV), fm.SchedBuffers(shape, DEV)
    t = torch.from_numpy(idx).to(DEV)
    a.run(shape, t, None)
    b.run(shape, t, torch.ones(E, G, dtype=torch.uint8, device=DEV))
    torch.cuda.synchronize()
    for name in ("x_eg", "max_load", "pair_dst", "row_of_pair", "pair_of_row", "seg_off", "rank_off"):
        assert torch.equal(getattr(a, name), getattr(b, name)), name


def test_expert_without_replica_is_reported():
    T, E, K, G = 64, 4, 1, 4
    idx = wl.random_topk(T, E, K, seed=0, skew=0.0)
    place = wl.placement_full(E, G)
    place[2, :] = 0
    shape = fm.Shape(T, 64, 64, E, K, G)
    sb = fm.SchedBuffers(shape, DEV)
    sb.run(shape, torch.from_numpy(idx).to(DEV), torch.from_numpy(place).to(DEV))
    torch.cuda.synchronize()
    assert int(sb.max_load.cpu()[0]) == -1
    assert not sb.x_eg.any()
    # nothing is scheduled, and what the movement and FFN entry points would read stays in bounds
    assert bool((sb.pair_dst == -1).all().cpu())
    ident = torch.arange(T * K, dtype=torch.int32, device=DEV)
    assert torch.equal(sb.row_of_pair, ident) and torch.equal(sb.pair_of_row, ident)
    assert not sb.seg_off.any() and not sb.rank_off.any()
    layer_shape = fm.Shape(T, 64, 64, E, K, G, fm.FINE_BF16, fm.FLAG_LOCALITY)
    x = torch.randn(T, 64, device=DEV).bfloat16()
    x_perm = torch.zeros(T * K, 64, dtype=torch.bfloat16, device=DEV)
    out = torch.zeros(T, 64, dtype=torch.bfloat16, device=DEV)
    fm.fine_permute(layer_shape, x, sb.pair_of_row, x_perm)
    fm.fine_combine(layer_shape, x_perm, sb.row_of_pair, torch.ones(T, K, device=DEV), out)
    torch.cuda.synchronize()
    assert torch.equal(out, x)
