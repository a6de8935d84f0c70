"""Helpers shared by the GPU parity tests (not collected by pytest)."""
import numpy as np
import torch

import paper_2511_16947_amd as fm
import workloads as wl
from oracle import moe, router, sched


def to64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu", torch.float64).numpy()


def max_rel_err(got: np.ndarray, want: np.ndarray) -> float:
    """max |got - want| / max |want| over the tensor (element-wise ratios are
    meaningless near zeros)."""
    denom = float(np.abs(want).max())
    if denom == 0.0:
        return float(np.abs(got).max())
    return float(np.abs(got - want).max() / denom)


def max_rel_err_rows(got: np.ndarray, want: np.ndarray) -> float:
    """The same measure taken row by row, max |got[r] - want[r]| / max |want[r]|, and the
    largest of them: a wrong row cannot hide behind a larger one elsewhere in the tensor.
    Rows of zeros must be zeros."""
    denom = np.abs(want).max(axis=1)
    err = np.abs(got - want).max(axis=1)
    zero = denom == 0.0
    if zero.any() and err[zero].max() > 0.0:
        return float("inf")
    return float((err[~zero] / denom[~zero]).max()) if (~zero).any() else 0.0


def tol_for(cfg) -> float:
    return 1e-5 if cfg.dtype == "f32" else 2e-2


def weights_of_factory(inp):
    """fp64 copies of one expert's weights at a time, taken from the very
    tensors the GPU path reads."""
    def weights_of(e):
        return to64(inp.w_gate[e]), to64(inp.w_up[e]), to64(inp.w_down[e])
    return weights_of


class GpuLayer:
    """Runs the forward hot path through the C ABI on tensors already on the GPU."""

    def __init__(self, cfg, inp, flags=fm.FLAG_LOCALITY):
        self.cfg, self.inp = cfg, inp
        self.shape = fm.shape_of(cfg, flags)
        dev = inp.x.device
        s = self.shape
        self.topk_idx = torch.empty(s.T, s.K, dtype=torch.int32, device=dev)
        self.topk_w = torch.empty(s.T, s.K, dtype=torch.float32, device=dev)
        self.sb = fm.SchedBuffers(s, dev)
        self.x_perm = torch.empty(s.P, s.d, dtype=s.torch_dtype, device=dev)
        self.y_perm = torch.empty(s.P, s.d, dtype=s.torch_dtype, device=dev)
        self.out = torch.empty(s.T, s.d, dtype=s.torch_dtype, device=dev)
        self.ws_ffn = fm.alloc_workspace(s, fm.WS_FFN, dev)
        self.ws_topk = fm.alloc_workspace(s, fm.WS_TOPK, dev)
        self.act_save = None

    def topk(self):
        i = self.inp
        fm.fine_topk(self.shape, i.x, i.w_router, i.bias, self.topk_idx, self.topk_w, self.ws_topk)

    def sched(self, place=None):
        self.sb.run(self.shape, self.topk_idx, place)

    def permute(self):
        fm.fine_permute(self.shape, self.inp.x, self.sb.pair_of_row, self.x_perm)

    def ffn(self, rank=-1):
        i = self.inp
        fm.fine_grouped_ffn(self.shape, rank, self.x_perm, i.w_gate, i.w_up, i.w_down, self.sb.seg_off, self.y_perm,
                            self.act_save, self.ws_ffn)

    def combine(self):
        fm.fine_combine(self.shape, self.y_perm, self.sb.row_of_pair, self.topk_w, self.out)

    def forward(self, place=None, per_rank=False):
        self.topk()
        self.sched(place)
        self.permute()
        if per_rank:
            for r in range(self.shape.G):
                self.ffn(r)
        else:
            self.ffn(-1)
        self.combine()
        torch.cuda.synchronize()


def check_schedule_against_oracle(sb, topk_idx_np, E, G, place=None, locality=True):
    """Bit-exact comparison of every scheduler output with the oracle run on
    the same topk_idx."""
    want = sched.schedule(topk_idx_np, E, G, place, locality)
    got = dict(load=sb.load, input=sb.input_eg, x=sb.x_eg, pair_dst=sb.pair_dst, row_of_pair=sb.row_of_pair,
               pair_of_row=sb.pair_of_row, seg_off=sb.seg_off, rank_off=sb.rank_off)
    for k, v in got.items():
        g = v.cpu().numpy().astype(np.int64)
        w = np.asarray(want[k]).astype(np.int64)
        assert g.shape == w.shape, (k, g.shape, w.shape)
        assert np.array_equal(g, w), "scheduler output %s differs from the oracle (first at %s)" % (
            k, np.argwhere(g != w)[:3].tolist())
    assert int(sb.max_load.cpu()[0]) == int(want["max_load"])
    return want


def check_router(cfg, inp, topk_idx, topk_w):
    """Routing parity: identical index lists for every token whose K-th /
    (K+1)-th fp64 logit gap is clear of the accumulation error; softmax weights
    within tolerance on those tokens; for the others the index sets must still be
    valid top-K sets up to that error."""
    logits = router.router_logits(to64(inp.x), to64(inp.w_router), to64(inp.bias))
    want_idx, want_w = router.topk_from_logits_fast(logits, cfg.K)
    gap_tol = 1e-5 if cfg.dtype == "f32" else 1e-3
    srt = -np.sort(-logits, axis=1)
    # a token is "clear" when all consecutive gaps among its top K+1 logits exceed gap_tol
    kk = min(cfg.K + 1, cfg.E)
    clear = (srt[:, :kk - 1] - srt[:, 1:kk] > gap_tol).all(axis=1) if kk > 1 else np.ones(cfg.T, bool)
    got_idx = topk_idx.cpu().numpy()
    got_w = to64(topk_w)
    assert clear.mean() > 0.5
    assert np.array_equal(got_idx[clear], want_idx[clear])
    assert np.abs(got_w[clear] - want_w[clear]).max() < (1e-5 if cfg.dtype == "f32" else 2e-3)
    # unclear tokens: every chosen logit within gap_tol of the true K-th largest, no repeats
    for t in np.nonzero(~clear)[0]:
        chosen = got_idx[t]
        assert len(set(chosen.tolist())) == cfg.K
        assert (logits[t, chosen] >= srt[t, cfg.K - 1] - 10 * gap_tol).all()
    return logits
