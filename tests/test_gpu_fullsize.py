"""Full-size forward parity on the four bf16 workloads, in the launch configuration
bench.py times (one fine_grouped_ffn call per logical rank): schedules bit-exact on
the whole routing table, outputs on sampled tokens and sampled rows the oracle computes
one by one, plus properties that hold at any size."""
import numpy as np
import pytest
import torch

import paper_2511_16947_amd as fm
import workloads as wl
from oracle import moe
from gpu_common import (GpuLayer, check_router, check_schedule_against_oracle, max_rel_err, to64, tol_for,
                        weights_of_factory)

pytestmark = pytest.mark.gpu
DEV = "cuda"

FULL = [("cfg2_mixtral", 24), ("cfg3_finegrained", 12), ("cfg4_dsv3", 6), ("cfg5_train", 24)]


@pytest.mark.parametrize("name,n_tokens", FULL)
def test_full_size_forward(name, n_tokens):
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

    # every row and every output element was written
    assert not torch.isnan(layer.y_perm.float()).any()
    assert not torch.isnan(layer.out.float()).any()
    # permute is exact
    por = torch.from_numpy(want["pair_of_row"].astype(np.int64)).to(DEV)
    assert torch.equal(layer.x_perm, inp.x[por // cfg.K])

    # sampled tokens: the dense per-token definition
    rng = np.random.default_rng(123)
    hot = int(np.argmax(want["load"]))
    tokens = rng.choice(cfg.T, size=n_tokens, replace=False)
    hot_tok = np.nonzero((idx == hot).any(axis=1))[0][:2]          # make sure the hottest expert is sampled
    tokens = np.unique(np.concatenate([tokens, hot_tok, [0, cfg.T - 1]]))
    weights_of = weights_of_factory(inp)
    x64 = np.zeros((cfg.T, cfg.d))
    x64[tokens] = to64(inp.x[torch.from_numpy(tokens).to(DEV)])
    ref = moe.dense_reference_by_expert(x64, idx, w, weights_of, tokens=tokens)
    got = to64(layer.out[torch.from_numpy(tokens).to(DEV)])
    tol = tol_for(cfg)
    err = max_rel_err(got, ref)
    print("  sampled tokens max-rel-err %.3e" % err, flush=True)
    assert err <= tol

    # sampled rows of y_perm, including the first and last row of some segments
    seg = want["seg_off"]
    cand = [0, cfg.P - 1]
    for g in (0, cfg.G // 2, cfg.G - 1):
        for e in np.nonzero(np.diff(seg[g]) > 0)[0][:2]:
            cand += [int(seg[g, e]), int(seg[g, e + 1] - 1)]
    cand = np.unique(np.array(cand))
    pairs = want["pair_of_row"][cand]
    for r, p in zip(cand, pairs):
        e = int(idx.reshape(-1)[p])
        xr = to64(inp.x[int(p) // cfg.K]).reshape(1, -1)
        yr = moe.ffn_rows(xr, *weights_of(e))[0]
        assert max_rel_err(to64(layer.y_perm[int(r)]), yr) <= tol, (r, e)


@pytest.mark.parametrize("name,n_tokens", [("cfg2_mixtral", 16), ("cfg5_train", 16)])
def test_full_size_forward_under_a_searched_placement(name, n_tokens):
    """The bench's secondary measurement: the same per-rank calls under the restricted placement that
    fine_replica_counts + fine_place_search build from the gate's loads (bench.py's slot count and
    seed).  Placement against the oracle's search on sampled candidates, schedule bit-exact on the
    whole routing table, sampled outputs against the dense definition."""
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

    layer.y_perm.fill_(float("nan"))
    layer.out.fill_(float("nan"))
    layer.forward(place=place, per_rank=True)
    idx = layer.topk_idx.cpu().numpy()
    w = to64(layer.topk_w)
    want = check_schedule_against_oracle(layer.sb, idx, E, G, place_np)
    print("  schedule bit-exact", flush=True)
    rows = np.diff(want["rank_off"])
    assert rows.max() == int(want["max_load"]) == -(-scores[b][0] // scores[b][1])
    assert not torch.isnan(layer.out.float()).any()
    # a rank computes only experts it holds
    seg = want["seg_off"]
    for g in range(G):
        present = np.nonzero(np.diff(seg[g]) > 0)[0]
        assert place_np[present, g].all() and len(present) <= slots
    rng = np.random.default_rng(7)
    tokens = np.unique(np.concatenate([rng.choice(cfg.T, size=n_tokens, replace=False), [0, cfg.T - 1]]))
    x64 = np.zeros((cfg.T, cfg.d))
    x64[tokens] = to64(inp.x[torch.from_numpy(tokens).to(DEV)])
    ref = moe.dense_reference_by_expert(x64, idx, w, weights_of_factory(inp), tokens=tokens)
    err = max_rel_err(to64(layer.out[torch.from_numpy(tokens).to(DEV)]), ref)
    print("  sampled tokens max-rel-err %.3e" % err, flush=True)
    assert err <= tol_for(cfg)
