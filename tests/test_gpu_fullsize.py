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
