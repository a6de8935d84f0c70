"""GPU parity of the forward hot path against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import paper_2511_16947_amd as fm
import workloads as wl
from oracle import moe, router, sched
from gpu_common import (GpuLayer, check_router, check_schedule_against_oracle, max_rel_err, max_rel_err_rows, to64, tol_for,
                        weights_of_factory)

pytestmark = pytest.mark.gpu
DEV = "cuda"


# ------------------------------------------------------------------ scheduler

SCHED_CASES = [
    # T, E, K, G, skew
    (256, 8, 2, 4, 1.0),
    (96, 5, 3, 4, 1.5),        # T/G = 24: source blocks straddle 64-token words
    (640, 128, 8, 8, 1.2),     # many experts, several words per source
    (2048, 256, 8, 32, 1.0),
    (4096, 64, 2, 16, 2.0),
    (64, 1, 1, 1, 0.0),        # degenerate: one expert, one rank
    (64, 3, 3, 64, 0.0),       # one token per rank, every token picks every expert
    (1000, 7, 1, 8, 3.0),      # P not divisible by 64, heavy skew
]


@pytest.mark.parametrize("locality", [True, False])
@pytest.mark.parametrize("case", SCHED_CASES)
def test_sched_full_placement_bit_exact(case, locality):
    T, E, K, G, skew = case
    idx = wl.random_topk(T, E, K, seed=T + E, skew=skew)
    shape = fm.Shape(T, 64, 64, E, K, G, fm.FINE_BF16, fm.FLAG_LOCALITY if locality else 0)
    sb = fm.SchedBuffers(shape, DEV)
    print("sched case", case, "locality", locality, flush=True)
    sb.run(shape, torch.from_numpy(idx).to(DEV))
    torch.cuda.synchronize()
    want = check_schedule_against_oracle(sb, idx, E, G, None, locality)
    rows = np.diff(want["rank_off"])
    assert rows.max() == -(-T * K // G)                  # the balance criterion: max load = ceil(P/G)


def test_sched_is_deterministic_across_runs():
    T, E, K, G = 4096, 128, 8, 8
    idx = torch.from_numpy(wl.random_topk(T, E, K, seed=1, skew=1.3)).to(DEV)
    shape = fm.Shape(T, 64, 64, E, K, G)
    a, b = fm.SchedBuffers(shape, DEV), fm.SchedBuffers(shape, DEV)
    a.run(shape, idx)
    b.run(shape, idx)
    torch.cuda.synchronize()
    for name in ("x_eg", "pair_dst", "row_of_pair", "pair_of_row", "seg_off"):
        assert torch.equal(getattr(a, name), getattr(b, name))


# ------------------------------------------------------------------ gate alone

ROUTER_CASES = [
    # T, d, E, K, dtype        which kernel takes it
    (1000, 256, 8, 2, "bf16"),     # MFMA, waves split k; T not a multiple of 32
    (33, 64, 32, 32, "bf16"),      # one k-step only (three waves idle), K = E at its limit
    (257, 448, 64, 6, "bf16"),     # two expert tiles, k-steps not a multiple of 4
    (300, 192, 128, 8, "bf16"),    # MFMA, block shares the slab; T not a multiple of 128
    (129, 128, 256, 8, "bf16"),    # eight expert tiles
    (700, 1024, 256, 8, "bf16"),   # few token tiles, long k: blocks share a tile, 2 parts of k (with the workspace)
    (130, 1600, 96, 4, "bf16"),    # 3 parts of 9, 9, 7 steps; E = 96: the fourth wave of a block has no experts
    (40, 4608, 160, 5, "bf16"),    # 8 parts of 9 steps; E = 160 on the 256-expert kernel: waves 2 and 3 partly or wholly idle
    (64, 128, 24, 1, "bf16"),      # E a multiple of 8 but not of 32, K = 1
    (200, 128, 12, 3, "bf16"),     # E not a multiple of 8: lane-per-expert kernel
    (77, 50, 5, 2, "f32"),         # fp32
]


@pytest.mark.parametrize("case", ROUTER_CASES, ids=lambda c: "T%d_d%d_E%d_K%d_%s" % c)
def test_router_topk(case):
    T, d, E, K, dtype = case
    cfg = wl.LayerConfig("router_case", T, d, 64, E, K, 1, dtype, 11, "scaled_z", 0.5)
    inp = wl.make_inputs(cfg, DEV, with_weights=False)
    shape = fm.shape_of(cfg)
    idx = torch.full((T, K), -1, dtype=torch.int32, device=DEV)
    w = torch.full((T, K), -1.0, dtype=torch.float32, device=DEV)
    # without and with the workspace (which lets blocks share a token tile when tokens are few)
    for ws in (None, fm.alloc_workspace(shape, fm.WS_TOPK, DEV)):
        print("router case", case, "workspace", None if ws is None else ws.numel(), flush=True)
        idx.fill_(-1)
        w.fill_(-1.0)
        fm.fine_topk(shape, inp.x, inp.w_router, inp.bias, idx, w, ws)
        torch.cuda.synchronize()
        check_router(cfg, inp, idx, w)
        got = idx.cpu().numpy()
        assert got.min() >= 0 and got.max() < E
        assert np.allclose(to64(w).sum(axis=1), 1.0, atol=1e-5)


# ------------------------------------------------------------------ whole layer, small

def small_cfgs():
    c = wl.CONFIGS
    return [
        c["cfg1_tiny_f32"],
        wl.scaled(c["cfg2_mixtral"], name="cfg2_small", T=1024, d=256, f=448),      # ragged n tile (448 = 3.5 x 128)
        wl.scaled(c["cfg3_finegrained"], name="cfg3_small", T=512, d=128, f=192),
        wl.scaled(c["cfg4_dsv3"], name="cfg4_small", T=512, d=192, f=128),
        wl.scaled(c["cfg5_train"], name="cfg5_small", T=2048, d=128, f=256),
        wl.scaled(c["cfg1_tiny_f32"], name="f32_odd", T=60, d=50, f=70, E=5, K=3, G=3),  # nothing a multiple of a tile
        # bf16 with every edge at once: d narrower than a column tile, f = 2.5 column tiles, ragged
        # segments on 3 ranks, E not a multiple of 8 (lane-per-expert gate)
        wl.LayerConfig("bf16_odd", 201, 192, 320, 3, 2, 3, "bf16", 9, "scaled_z", 1.0),
        # one expert, one rank, one token tile: a single segment of 96 rows
        wl.LayerConfig("bf16_single", 96, 64, 64, 8, 1, 1, "bf16", 10, "one_hot", 50.0),
    ]


@pytest.mark.parametrize("cfg", small_cfgs(), ids=lambda c: c.name)
@pytest.mark.parametrize("tile", [0, 1, 2, 3, "simple"])
def test_layer_forward_elementwise(cfg, tile):
    if cfg.dtype == "f32" and tile != 0:
        pytest.skip("tile variants are for the bf16 MFMA kernels")
    flags = fm.FLAG_LOCALITY
    if tile == "simple":
        flags |= fm.FLAG_SIMPLE_FFN
    else:
        flags |= tile << 8
    print("layer case", cfg.name, "tile", tile, flush=True)
    inp = wl.make_inputs(cfg, DEV)
    layer = GpuLayer(cfg, inp, flags)
    layer.forward()

    check_router(cfg, inp, layer.topk_idx, layer.topk_w)
    idx = layer.topk_idx.cpu().numpy()
    w = to64(layer.topk_w)
    want = check_schedule_against_oracle(layer.sb, idx, cfg.E, cfg.G)

    # permute: pure data movement, bit exact
    xp = layer.x_perm.cpu()
    assert torch.equal(xp, inp.x.cpu()[torch.from_numpy(want["pair_of_row"].astype(np.int64) // cfg.K)])

    # expert computation and combine against the unscheduled dense definition, given the
    # library's own routing (indices and fp32 weights)
    weights_of = weights_of_factory(inp)
    ref_out = moe.dense_reference_by_expert(to64(inp.x), idx, w, weights_of)
    ref_y = moe.grouped_ffn(moe.permute(to64(inp.x), want["pair_of_row"], cfg.K), want["seg_off"], weights_of)
    tol = tol_for(cfg)
    assert max_rel_err(to64(layer.y_perm), ref_y) <= tol
    assert max_rel_err(to64(layer.out), ref_out) <= tol

    # per-rank calls: the same rows; a launch cuts the k range of its last tiles by how many
    # tiles it has, so fp32 sums may be taken in another order than in the all-ranks call
    y_all = layer.y_perm.clone()
    layer.y_perm.zero_()
    for r in range(cfg.G):
        layer.ffn(r)
    torch.cuda.synchronize()
    assert max_rel_err(to64(layer.y_perm), ref_y) <= tol
    assert max_rel_err(to64(layer.y_perm), to64(y_all)) <= (1e-5 if cfg.dtype == "f32" else 2.0 ** -7)

    # the same call again gives the same bits (partial sums are added in a fixed order)
    y_first = layer.y_perm.clone()
    layer.y_perm.zero_()
    for r in range(cfg.G):
        layer.ffn(r)
    torch.cuda.synchronize()
    assert torch.equal(layer.y_perm, y_first)


@pytest.mark.parametrize("tile", [2, 3])
def test_tiles_cut_along_k(tile):
    """Few tiles and a long k range in GEMM 2 (f = 80 x 64): the launch cuts every tile's k range
    over many blocks and adds the partial sums up.  Element by element against the oracle, and
    bit-stable from run to run."""
    cfg = wl.LayerConfig("k_cut", 256, 256, 5120, 2, 2, 1, "bf16", 7, "scaled_z", 0.5)
    inp = wl.make_inputs(cfg, DEV)
    layer = GpuLayer(cfg, inp, fm.FLAG_LOCALITY | (tile << 8))
    print("k-cut case tile", tile, flush=True)
    layer.forward()
    idx = layer.topk_idx.cpu().numpy()
    want = sched.schedule(idx, cfg.E, cfg.G)
    weights_of = weights_of_factory(inp)
    ref_y = moe.grouped_ffn(moe.permute(to64(inp.x), want["pair_of_row"], cfg.K), want["seg_off"], weights_of)
    assert max_rel_err(to64(layer.y_perm), ref_y) <= tol_for(cfg)
    first = layer.y_perm.clone()
    for _ in range(3):
        layer.y_perm.zero_()
        layer.ffn(-1)
        torch.cuda.synchronize()
        assert torch.equal(layer.y_perm, first)


@pytest.mark.parametrize("tile,d,f,T,parts", [(3, 1024, 1024, 256, 2), (3, 1024, 1024, 250, 2),
                                              (2, 2048, 2048, 256, 4), (2, 2048, 2048, 232, 4)])
def test_a_small_rest_of_tiles_is_cut_into_few_parts(tile, d, f, T, parts):
    """Fewer tiles than blocks and a k range too short for the cut over the whole grid (16 k-tiles
    on the 256-row tile, 32 on the 128-row tile): every tile of the rest is cut into `parts` parts,
    part p of tile t on block t + p * rest, in both GEMMs.  Every element and every row against
    the oracle, whole and ragged row tiles, and bit-stable from run to run."""
    cfg = wl.LayerConfig("few_parts", T, d, f, 2, 2, 1, "bf16", 11, "scaled_z", 0.5)
    # both GEMMs take the branch: rest tiles * parts fit the grid of 256 blocks, parts divide the
    # k-tiles, at least 8 k-tiles per part, and the whole-grid cut does not pay
    bm = 256 if tile == 3 else 128
    for kd, n_out, bnc in ((d, f, 128), (f, d, 256)):
        nk, rest = kd // 64, 2 * -(-T // bm) * (n_out // bnc)
        assert rest * parts <= 256 and nk % parts == 0 and nk // parts >= 8 and (parts == 4 or rest * 4 > 256 or nk // 4 < 8)
        assert nk * (256 - rest) <= (16 if tile == 3 else 32) * 256
    inp = wl.make_inputs(cfg, DEV)
    layer = GpuLayer(cfg, inp, fm.FLAG_LOCALITY | (tile << 8))
    print("few-parts case tile", tile, "T", T, flush=True)
    layer.y_perm.fill_(float("nan"))
    layer.forward()
    idx = layer.topk_idx.cpu().numpy()
    want = check_schedule_against_oracle(layer.sb, idx, cfg.E, cfg.G)
    weights_of = weights_of_factory(inp)
    ref_y = moe.grouped_ffn(moe.permute(to64(inp.x), want["pair_of_row"], cfg.K), want["seg_off"], weights_of)
    got = to64(layer.y_perm)
    assert max_rel_err(got, ref_y) <= tol_for(cfg)
    assert max_rel_err_rows(got, ref_y) <= tol_for(cfg)
    ref_out = moe.combine(ref_y, want["row_of_pair"], to64(layer.topk_w))
    assert max_rel_err_rows(to64(layer.out), ref_out) <= tol_for(cfg)
    first = layer.y_perm.clone()
    for _ in range(3):
        layer.y_perm.zero_()
        layer.ffn(-1)
        torch.cuda.synchronize()
        assert torch.equal(layer.y_perm, first)


@pytest.mark.parametrize("T", [1280, 1200])
def test_a_rest_above_half_a_round_is_cut_in_groups(T):
    """160 tiles of 50 k-tiles on 256 blocks in GEMM 1 (five row tiles, the last one whole or ragged, 32 column
    tiles): groups of two tiles share three parts, every tile is the sum of two parts.  GEMM 2 (65 tiles of 64
    k-tiles) takes the even cut over the whole grid.  Every element and every row against the oracle, and
    bit-stable from run to run."""
    cfg = wl.LayerConfig("groups", T, 3200, 4096, 1, 1, 1, "bf16", 17, "scaled_z", 0.5)
    inp = wl.make_inputs(cfg, DEV)
    layer = GpuLayer(cfg, inp, fm.FLAG_LOCALITY | (3 << 8))
    print("grouped-cut case T", T, flush=True)
    layer.y_perm.fill_(float("nan"))
    layer.forward()
    idx = layer.topk_idx.cpu().numpy()
    want = check_schedule_against_oracle(layer.sb, idx, cfg.E, cfg.G)
    rest, nk = -(-T // 256) * (cfg.f // 128), cfg.d // 64
    q = -(-rest // (256 - rest))
    assert 128 < rest < 256 and nk > 16 * (q + 1)      # the case is what it says
    weights_of = weights_of_factory(inp)
    ref_y = moe.grouped_ffn(moe.permute(to64(inp.x), want["pair_of_row"], cfg.K), want["seg_off"], weights_of)
    got = to64(layer.y_perm)
    assert max_rel_err(got, ref_y) <= tol_for(cfg)
    assert max_rel_err_rows(got, ref_y) <= tol_for(cfg)
    first = layer.y_perm.clone()
    for _ in range(3):
        layer.y_perm.zero_()
        layer.ffn(-1)
        torch.cuda.synchronize()
        assert torch.equal(layer.y_perm, first)


@pytest.mark.parametrize("d,f,both", [(5632, 2816, True), (1024, 2560, False)])
def test_units_of_a_long_launch_are_handed_out_from_queues(d, f, both):
    """More than two rounds of tiles in one launch (26 row tiles: 572 tiles in both GEMMs on 256 blocks with the
    rest cut along k over the whole grid; or 520 tiles in GEMM 1 with its 16 k-tiles and a rest of 8 tiles cut into
    two parts each): from the second round on the blocks take their tiles, and the parts of the rest, from the
    per-XCD queues, whoever is free first.  Every element and every row against the oracle, ragged row
    tiles of several lengths among whole ones, the call for all ranks and the calls rank by rank,
    and bit-stable from run to run (which block computes a tile must not matter)."""
    cfg = wl.LayerConfig("queues", 2688, d, f, 8, 2, 2, "bf16", 13, "scaled_z", 1.0)
    inp = wl.make_inputs(cfg, DEV)
    layer = GpuLayer(cfg, inp, fm.FLAG_LOCALITY | (3 << 8))
    print("queue case d", d, "f", f, flush=True)
    layer.y_perm.fill_(float("nan"))
    layer.forward()
    idx = layer.topk_idx.cpu().numpy()
    want = check_schedule_against_oracle(layer.sb, idx, cfg.E, cfg.G)
    seg = np.diff(want["seg_off"], axis=1)
    row_tiles = int((-(-seg // 256)).sum())
    assert row_tiles * (cfg.f // 128) > 512 and (not both or row_tiles * (cfg.d // 256) > 512)      # the case is what it says
    if not both:      # few parts: a rest of at most 128 tiles, 16 k-tiles
        assert cfg.d == 1024 and 0 < row_tiles * (cfg.f // 128) - 512 <= 128
    assert ((seg % 256) != 0).sum() >= 4
    weights_of = weights_of_factory(inp)
    ref_y = moe.grouped_ffn(moe.permute(to64(inp.x), want["pair_of_row"], cfg.K), want["seg_off"], weights_of)
    got = to64(layer.y_perm)
    assert max_rel_err(got, ref_y) <= tol_for(cfg)
    assert max_rel_err_rows(got, ref_y) <= tol_for(cfg)
    first = layer.y_perm.clone()
    for _ in range(3):
        layer.y_perm.zero_()
        layer.ffn(-1)
        torch.cuda.synchronize()
        assert torch.equal(layer.y_perm, first)
    # rank by rank the tiles that are cut along k are other ones: equal within rounding, not bit by bit
    layer.y_perm.fill_(float("nan"))
    for r in range(cfg.G):
        layer.ffn(r)
    torch.cuda.synchronize()
    assert max_rel_err_rows(to64(layer.y_perm), ref_y) <= tol_for(cfg)


def test_act_save_holds_the_preactivations():
    cfg = wl.scaled(wl.CONFIGS["cfg2_mixtral"], name="cfg2_small", T=512, d=128, f=256)
    inp = wl.make_inputs(cfg, DEV)
    layer = GpuLayer(cfg, inp)
    layer.act_save = torch.empty(cfg.P, 2 * cfg.f, dtype=torch.bfloat16, device=DEV)
    layer.forward()
    want = sched.schedule(layer.topk_idx.cpu().numpy(), cfg.E, cfg.G)
    xp = moe.permute(to64(inp.x), want["pair_of_row"], cfg.K)
    got = to64(layer.act_save)
    for g in range(cfg.G):
        for e in range(cfg.E):
            lo, hi = want["seg_off"][g, e], want["seg_off"][g, e + 1]
            if hi > lo:
                a = xp[lo:hi] @ to64(inp.w_gate[e])
                b = xp[lo:hi] @ to64(inp.w_up[e])
                assert max_rel_err(got[lo:hi, :cfg.f], a) <= 2e-2
                assert max_rel_err(got[lo:hi, cfg.f:], b) <= 2e-2


def test_bad_arguments_return_errors():
    s = fm.Shape(256, 128, 256, 8, 2, 4, fm.FINE_BF16)
    x = torch.zeros(256, 128, dtype=torch.bfloat16, device=DEV)
    idx = torch.zeros(512, dtype=torch.int32, device=DEV)
    xp = torch.zeros(512, 128, dtype=torch.bfloat16, device=DEV)
    with pytest.raises(fm.FineError) as ei:
        fm.fine_permute(s, x, idx, None)
    assert ei.value.code == fm.FINE_INVALID_ARG
    with pytest.raises(fm.FineError) as ei:
        fm.fine_grouped_ffn(s, 7, xp, xp, xp, xp, idx, xp, None, torch.zeros(1024, dtype=torch.uint8, device=DEV))
    assert ei.value.code == fm.FINE_INVALID_ARG      # rank out of range
    with pytest.raises(fm.FineError) as ei:
        fm.fine_grouped_ffn(s, 0, xp, xp, xp, xp, idx, xp, None, torch.zeros(1024, dtype=torch.uint8, device=DEV))
    assert ei.value.code == fm.FINE_WORKSPACE_TOO_SMALL


def test_a_step_with_the_split_gate_can_be_captured_in_a_graph():
    """128 experts and 512 tokens: the gate runs as two kernels (blocks share token tiles over parts of
    k, partial logits in the workspace, then the selection).  Captured and replayed with eager work in
    between, every replay must give the eager bits."""
    cfg = wl.LayerConfig("graph_split_gate", 512, 1024, 128, 128, 4, 4, "bf16", 13, "scaled_z", 1.0)
    assert fm.fine_workspace_bytes(fm.shape_of(cfg), fm.WS_TOPK) > 256
    inp = wl.make_inputs(cfg, DEV)
    layer = GpuLayer(cfg, inp, fm.FLAG_LOCALITY)
    layer.forward(per_rank=True)
    want_idx, want_w, want_out = layer.topk_idx.clone(), layer.topk_w.clone(), layer.out.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            layer.topk()
            layer.sched()
            layer.permute()
            for r in range(cfg.G):
                layer.ffn(r)
            layer.combine()
    torch.cuda.current_stream().wait_stream(side)
    for i in range(3):
        layer.out.zero_()
        layer.topk_idx.fill_(-1)
        layer.ws_topk.fill_(0x7f)                           # stale partial logits must not matter
        layer.permute()                                      # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(layer.topk_idx, want_idx), i
        assert torch.equal(layer.topk_w, want_w), i
        assert torch.equal(layer.out.view(torch.int16), want_out.view(torch.int16)), i


@pytest.mark.parametrize("restricted", [False, True])
def test_a_step_can_be_captured_in_a_graph(restricted):
    """The library allocates nothing, synchronises nothing and clears its own counters in kernels,
    so a whole forward step is captured in a HIP graph as it is.  Every replay, with eager work and
    synchronisations in between, must give the bits of the eager run."""
    cfg = wl.LayerConfig("graph_k_cut", 512, 256, 2560, 4, 2, 2, "bf16", 11, "scaled_z", 1.0)
    inp = wl.make_inputs(cfg, DEV)
    layer = GpuLayer(cfg, inp, fm.FLAG_LOCALITY | (3 << 8))
    place = None
    if restricted:
        place = torch.from_numpy(np.array([[1, 0], [1, 1], [0, 1], [1, 1]], dtype=np.uint8)).to(DEV)
    layer.forward(place=place, per_rank=True)             # eager; also sets every kernel attribute before the capture
    want_out, want_y = layer.out.clone(), layer.y_perm.clone()
    want_rows = layer.sb.row_of_pair.clone()

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            layer.topk()
            layer.sched(place)
            layer.permute()
            for r in range(cfg.G):
                layer.ffn(r)
            layer.combine()
    torch.cuda.current_stream().wait_stream(side)
    for i in range(4):
        layer.out.zero_()
        layer.y_perm.zero_()
        layer.sb.row_of_pair.fill_(-7)
        layer.topk()                                       # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(layer.sb.row_of_pair, want_rows), i
        assert torch.equal(layer.y_perm.view(torch.int16), want_y.view(torch.int16)), i
        assert torch.equal(layer.out.view(torch.int16), want_out.view(torch.int16)), i
