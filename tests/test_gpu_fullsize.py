"""Full-size forward parity on the four bf16 workloads, in the launch configuration
bench.py times (one fine_grouped_ffn call per logical rank) and in one call for all ranks:
schedules bit-exact on the whole routing table, and EVERY element of y_perm and of out
against the oracle, tensor-wide and row by row."""
import numpy as np
import pytest
import torch

import paper_2511_16947_amd as fm
import workloads as wl
from oracle import moe
from gpu_common import (GpuLayer, check_router, check_schedule_against_oracle, max_rel_err, max_rel_err_rows, to64,
                        tol_for, weights_of_factory)

pytestmark = pytest.mark.gpu
DEV = "cuda"

FULL = ["cfg2_mixtral", "cfg3_finegrained", "cfg4_dsv3", "cfg5_train"]

# The oracle's expert output of every pair, FFN_{e(p)}(x[t(p)]) in fp64, computed once per workload:
# it does not depend on the schedule (Section 3: any replica computes a token equivalently, which
# tests/test_oracle_moe.py pins on the CPU), so the test under a restricted placement reads it too.
_PAIR_REF = {}


def pair_reference(cfg, inp, idx, want):
    """[P,d] fp64: the oracle's grouped FFN over the oracle's own schedule `want` (one expert's fp64
    weights at a time), re-indexed by pair (0.5 to 1.9 GB per workload, kept for the other test of the same workload)."""
    key = cfg.name
    if key in _PAIR_REF and np.array_equal(_PAIR_REF[key][0], idx):
        return _PAIR_REF[key][1]
    x_perm = moe.permute(to64(inp.x), want["pair_of_row"], cfg.K)
    y = moe.grouped_ffn(x_perm, want["seg_off"], weights_of_factory(inp))
    ref = y[want["row_of_pair"]]
    _PAIR_REF[key] = (idx.copy(), ref)
    return ref


def check_every_element(cfg, layer, want, ref_pair, w):
    tol = tol_for(cfg)
    ref_y = ref_pair[want["pair_of_row"]]
    got_y = to64(layer.y_perm)
    e_all, e_row = max_rel_err(got_y, ref_y), max_rel_err_rows(got_y, ref_y)
    print("  y_perm: every element, max-rel-err %.3e, worst row %.3e" % (e_all, e_row), flush=True)
    assert e_all <= tol and e_row <= tol
    del got_y
    ref_out = moe.combine(ref_y, want["row_of_pair"], w)
    got_out = to64(layer.out)
    e_all, e_row = max_rel_err(got_out, ref_out), max_rel_err_rows(got_out, ref_out)
    print("  out: every element, max-rel-err %.3e, worst row %.3e" % (e_all, e_row), flush=True)
    assert e_all <= tol and e_row <= tol
    return ref_out


@pytest.mark.parametrize("name", FULL)
def test_full_size_forward(name):
    cfg = wl.CONFIGS[name]
    print("full-size case", name, flush=True)
    inp = wl.make_inputs(cfg, DEV)
    layer = GpuLayer(cfg, inp)
    layer.y_perm.fill_(float("nan"))
    layer.out.fill_(float("nan"))
    layer.forward(per_rank=True)
    print("  forward done", flush=True)

    check_router(cfg, inp, layer.topk_idx, layer.topk_w)
    idx = layer.topk_idx.cpu().numpy()
    w = to64(layer.topk_w)
    want = check_schedule_against_oracle(layer.sb, idx, cfg.E, cfg.G)
    print("  schedule bit-exact", flush=True)
    rows = np.diff(want["rank_off"])
    assert rows.max() == rows.min() == cfg.P // cfg.G            # complete balance (G divides P)

    # permute is exact
    por = torch.from_numpy(want["pair_of_row"].astype(np.int64)).to(DEV)
    assert torch.equal(layer.x_perm, inp.x[por // cfg.K])

    ref_pair = pair_reference(cfg, inp, idx, want)
    print("  oracle done", flush=True)
    ref_out = check_every_element(cfg, layer, want, ref_pair, w)

    # the same rows in ONE call for all ranks (thousands of tiles of every length in one launch, handed out to the
    # blocks as they become free): every element again, twice, bit-equal between the two runs
    layer.y_perm.fill_(float("nan"))
    layer.out.fill_(float("nan"))
    layer.ffn(-1)
    layer.combine()
    torch.cuda.synchronize()
    print("  one call for all ranks:", flush=True)
    check_every_element(cfg, layer, want, ref_pair, w)
    first = layer.y_perm.clone()
    layer.y_perm.fill_(float("nan"))
    layer.ffn(-1)
    torch.cuda.synchronize()
    assert torch.equal(layer.y_perm.view(torch.int16), first.view(torch.int16))
    del first

    # the scheduled reference is the dense per-token definition (sampled tokens, hottest expert included)
    rng = np.random.default_rng(123)
    hot = int(np.argmax(want["load"]))
    tokens = rng.choice(cfg.T, size=8, replace=False)
    hot_tok = np.nonzero((idx == hot).any(axis=1))[0][:2]
    tokens = np.unique(np.concatenate([tokens, hot_tok, [0, cfg.T - 1]]))
    x64 = np.zeros((cfg.T, cfg.d))
    x64[tokens] = to64(inp.x[torch.from_numpy(tokens).to(DEV)])
    dense = moe.dense_reference_by_expert(x64, idx, w, weights_of_factory(inp), tokens=tokens)
    assert max_rel_err(ref_out[tokens], dense) <= 1e-12


@pytest.mark.parametrize("name", FULL)
def test_full_size_forward_under_a_searched_placement(name):
    """The bench's secondary measurement: the same per-rank calls under the restricted placement that
    fine_replica_counts + fine_place_search build from the gate's loads (bench.py's slot count and
    seed).  Placement against the oracle's search on sampled candidates, schedule bit-exact on the
    whole routing table, every element of y_perm and out against the oracle."""
    from oracle import placement
    cfg = wl.CONFIGS[name]
    print("full-size case under a searched placement", name, flush=True)
    inp = wl.make_inputs(cfg, DEV)
    layer = GpuLayer(cfg, inp)
    layer.topk()
    layer.sched()
    E, G, n = cfg.E, cfg.G, 4096
    slots = -(-5 * E // (4 * G))
    counts = torch.empty(E, dtype=torch.int32, device=DEV)
    m_num = torch.empty(n, dtype=torch.int64, device=DEV)
    m_den = torch.empty(n, dtype=torch.int32, device=DEV)
    best = torch.empty(1, dtype=torch.int32, device=DEV)
    place = torch.empty(E, G, dtype=torch.uint8, device=DEV)
    fm.fine_replica_counts(layer.shape, layer.sb.load, slots, counts)
    fm.fine_place_search(layer.shape, layer.sb.load, counts, slots, n, 0, m_num, m_den, best, place)
    torch.cuda.synchronize()
    load = layer.sb.load.cpu().numpy().astype(np.int64)
    want_counts = placement.replica_counts(load, G, slots)
    assert np.array_equal(counts.cpu().numpy(), want_counts)
    b = int(best.cpu()[0])
    scores = list(zip(m_num.cpu().tolist(), m_den.cpu().tolist()))
    assert all(num * scores[b][1] >= scores[b][0] * den for num, den in scores)        # nobody beats the choice
    assert all(num * scores[b][1] > scores[b][0] * den for num, den in scores[:b])      # earlier ones are worse
    for c in sorted({0, b, n - 1}):
        p = placement.draw_placement(want_counts, G, slots, 0, c)
        m = placement.max_density(load, p)
        assert (m.numerator, m.denominator) == scores[c], c
        if c == b:
            assert np.array_equal(place.cpu().numpy(), p)
    place_np = place.cpu().numpy()
    assert (place_np.sum(axis=0) <= slots).all()
    print("  placement matches the oracle's search", flush=True)

    # the reference of every pair, from the oracle's schedule under the full placement
    idx = layer.topk_idx.cpu().numpy()
    ref_pair = pair_reference(cfg, inp, idx, check_schedule_against_oracle(layer.sb, idx, E, G))
    print("  oracle done", flush=True)

    layer.y_perm.fill_(float("nan"))
    layer.out.fill_(float("nan"))
    layer.forward(place=place, per_rank=True)
    assert np.array_equal(layer.topk_idx.cpu().numpy(), idx)
    w = to64(layer.topk_w)
    want = check_schedule_against_oracle(layer.sb, idx, E, G, place_np)
    print("  schedule bit-exact", flush=True)
    rows = np.diff(want["rank_off"])
    assert rows.max() == int(want["max_load"]) == -(-scores[b][0] // scores[b][1])
    # a rank computes only experts it holds
    seg = want["seg_off"]
    for g in range(G):
        present = np.nonzero(np.diff(seg[g]) > 0)[0]
        assert place_np[present, g].all() and len(present) <= slots
    check_every_element(cfg, layer, want, ref_pair, w)
