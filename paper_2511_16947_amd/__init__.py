"""Python binding of libfinemoe (ctypes): argument marshalling only.

Every step of the MoE-layer hot path (gate top-K, token scheduling, permute,
grouped SwiGLU expert FFN, combine, backward) runs in the HIP kernels behind the
C ABI declared in include/finemoe.h.  PyTorch is used for device memory and the
current stream, nothing else.  There is no CPU fallback: if the library has not
been built (python -m paper_2511_16947_amd.build) importing a function and
calling it raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfinemoe.so")

FINE_OK = 0
FINE_INVALID_ARG = -1
FINE_UNSUPPORTED = -2
FINE_WORKSPACE_TOO_SMALL = -3
FINE_INFEASIBLE = -4
FINE_HIP_ERROR = -5
FINE_F32, FINE_BF16 = 0, 1
FLAG_LOCALITY = 1
FLAG_ACT_SAVE_H = 16
# measurement and test switches (include/finemoe_measure.h; not part of the contract)
FLAG_SIMPLE_FFN, FLAG_ONLY_GEMM1, FLAG_ONLY_GEMM2 = 2, 4, 8
FLAG_TILE_SHIFT, FLAG_BWD_STAGE_SHIFT = 8, 12
WS_TOPK, WS_SCHED, WS_FFN, WS_BACKWARD = 0, 1, 2, 3

EXPORTS = ["fine_version", "fine_last_hip_error", "fine_workspace_bytes", "fine_topk", "fine_sched",
           "fine_sched_warm", "fine_sched_static", "fine_sched_comm", "fine_comm_replica_loads_host",
           "fine_permute", "fine_grouped_ffn", "fine_combine", "fine_backward", "fine_cayley_placement", "fine_replica_counts",
           "fine_eval_placements", "fine_place_search"]


class FineError(RuntimeError):
    def __init__(self, fn: str, code: int, hip: int = 0):
        names = {-1: "INVALID_ARG", -2: "UNSUPPORTED", -3: "WORKSPACE_TOO_SMALL", -4: "INFEASIBLE", -5: "HIP_ERROR"}
        super().__init__("%s failed: %s (%d)%s" % (fn, names.get(code, "?"), code,
                                                   ", hipError %d" % hip if code == FINE_HIP_ERROR else ""))
        self.code = code


class _Shape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("T", "d", "f", "E", "K", "G", "dtype", "flags")]


_lib = None


def load_library() -> ctypes.CDLL:
    """Loads libfinemoe.so from the package directory; raises if it is not built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            "%s is missing: build it with `python -m paper_2511_16947_amd.build` (there is no fallback path)" % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    vp, sz, i32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int32
    sp = ctypes.POINTER(_Shape)
    lib.fine_version.restype = ctypes.c_int
    lib.fine_version.argtypes = []
    lib.fine_last_hip_error.restype = ctypes.c_int
    lib.fine_last_hip_error.argtypes = []
    lib.fine_workspace_bytes.restype = sz
    lib.fine_workspace_bytes.argtypes = [sp, ctypes.c_int]
    lib.fine_topk.restype = ctypes.c_int
    lib.fine_topk.argtypes = [sp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.fine_sched.restype = ctypes.c_int
    lib.fine_sched.argtypes = [sp] + [vp] * 11 + [vp, sz, vp]
    lib.fine_sched_warm.restype = ctypes.c_int
    lib.fine_sched_warm.argtypes = [sp] + [vp] * 12 + [vp, sz, vp]
    lib.fine_sched_static.restype = ctypes.c_int
    lib.fine_sched_static.argtypes = [sp] + [vp] * 11 + [vp]
    lib.fine_sched_comm.restype = ctypes.c_int
    lib.fine_sched_comm.argtypes = [sp, vp, vp, i32, i32, i32] + [vp] * 9 + [vp, sz, vp]
    lib.fine_comm_replica_loads_host.restype = ctypes.c_int
    lib.fine_comm_replica_loads_host.argtypes = [i32, i32, vp, vp, vp, i32, i32, vp, vp]
    lib.fine_permute.restype = ctypes.c_int
    lib.fine_permute.argtypes = [sp, vp, vp, vp, vp]
    lib.fine_grouped_ffn.restype = ctypes.c_int
    lib.fine_grouped_ffn.argtypes = [sp, i32, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.fine_combine.restype = ctypes.c_int
    lib.fine_combine.argtypes = [sp, vp, vp, vp, vp, vp]
    lib.fine_backward.restype = ctypes.c_int
    lib.fine_backward.argtypes = [sp, i32] + [vp] * 16 + [ctypes.c_int, vp, sz, vp]
    lib.fine_cayley_placement.restype = ctypes.c_int
    lib.fine_cayley_placement.argtypes = [sp, i32, vp, i32, vp, i32, vp, vp]
    lib.fine_replica_counts.restype = ctypes.c_int
    lib.fine_replica_counts.argtypes = [sp, vp, i32, vp, vp]
    lib.fine_eval_placements.restype = ctypes.c_int
    lib.fine_eval_placements.argtypes = [sp, i32, vp, vp, vp, vp, vp]
    lib.fine_place_search.restype = ctypes.c_int
    lib.fine_place_search.argtypes = [sp, vp, vp, i32, i32, ctypes.c_uint32, vp, vp, vp, vp, vp]
    _lib = lib
    return lib


@dataclass(frozen=True)
class Shape:
    T: int
    d: int
    f: int
    E: int
    K: int
    G: int
    dtype: int = FINE_BF16
    flags: int = FLAG_LOCALITY

    @property
    def P(self) -> int:
        return self.T * self.K

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float32 if self.dtype == FINE_F32 else torch.bfloat16

    def c(self) -> _Shape:
        return _Shape(self.T, self.d, self.f, self.E, self.K, self.G, self.dtype, self.flags)


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device-resident contiguous tensors only"
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(fn: str, rc: int):
    if rc != FINE_OK:
        raise FineError(fn, rc, load_library().fine_last_hip_error())


def fine_version() -> int:
    return load_library().fine_version()


def fine_workspace_bytes(shape: Shape, which: int) -> int:
    cs = shape.c()
    return int(load_library().fine_workspace_bytes(ctypes.byref(cs), which))


def alloc_workspace(shape: Shape, which: int, device="cuda") -> torch.Tensor:
    n = fine_workspace_bytes(shape, which)
    if n == 0:
        raise FineError("fine_workspace_bytes", FINE_INVALID_ARG)
    return torch.empty(n, dtype=torch.uint8, device=device)


def fine_topk(shape: Shape, x, w_router, bias, topk_idx, topk_w, ws=None):
    cs = shape.c()
    rc = load_library().fine_topk(ctypes.byref(cs), _ptr(x), _ptr(w_router), _ptr(bias), _ptr(topk_idx), _ptr(topk_w),
                                  _ptr(ws), 0 if ws is None else ws.numel(), _stream())
    _check("fine_topk", rc)


def fine_sched(shape: Shape, topk_idx, place, load, input_eg, x_eg, max_load, pair_dst, row_of_pair, pair_of_row,
               seg_off, rank_off, ws):
    cs = shape.c()
    rc = load_library().fine_sched(ctypes.byref(cs), _ptr(topk_idx), _ptr(place), _ptr(load), _ptr(input_eg), _ptr(x_eg),
                                   _ptr(max_load), _ptr(pair_dst), _ptr(row_of_pair), _ptr(pair_of_row), _ptr(seg_off),
                                   _ptr(rank_off), _ptr(ws), ws.numel(), _stream())
    _check("fine_sched", rc)


def fine_sched_warm(shape: Shape, topk_idx, place, x_prev, load, input_eg, x_eg, max_load, pair_dst, row_of_pair,
                    pair_of_row, seg_off, rank_off, ws):
    cs = shape.c()
    rc = load_library().fine_sched_warm(ctypes.byref(cs), _ptr(topk_idx), _ptr(place), _ptr(x_prev), _ptr(load),
                                        _ptr(input_eg), _ptr(x_eg), _ptr(max_load), _ptr(pair_dst), _ptr(row_of_pair),
                                        _ptr(pair_of_row), _ptr(seg_off), _ptr(rank_off), _ptr(ws), ws.numel(), _stream())
    _check("fine_sched_warm", rc)


def fine_sched_static(shape: Shape, topk_idx, place, load, input_eg, x_eg, max_load, pair_dst, row_of_pair, pair_of_row,
                      seg_off, rank_off):
    cs = shape.c()
    rc = load_library().fine_sched_static(ctypes.byref(cs), _ptr(topk_idx), _ptr(place), _ptr(load), _ptr(input_eg),
                                          _ptr(x_eg), _ptr(max_load), _ptr(pair_dst), _ptr(row_of_pair),
                                          _ptr(pair_of_row), _ptr(seg_off), _ptr(rank_off), _stream())
    _check("fine_sched_static", rc)


def fine_sched_comm(shape: Shape, topk_idx, place, alpha_num: int, alpha_den: int, ranks_per_node: int, load, input_eg,
                    x_eg, comp_comm, pair_dst, row_of_pair, pair_of_row, seg_off, rank_off, ws):
    cs = shape.c()
    rc = load_library().fine_sched_comm(ctypes.byref(cs), _ptr(topk_idx), _ptr(place), alpha_num, alpha_den,
                                        ranks_per_node, _ptr(load), _ptr(input_eg), _ptr(x_eg), _ptr(comp_comm),
                                        _ptr(pair_dst), _ptr(row_of_pair), _ptr(pair_of_row), _ptr(seg_off),
                                        _ptr(rank_off), _ptr(ws), ws.numel(), _stream())
    _check("fine_sched_comm", rc)


def fine_comm_replica_loads_host(load, input_eg, place, alpha_num: int, alpha_den: int):
    """Host arrays in (anything numpy converts), (x_eg[E,G] int32, (C*, M*)) out; marshalling only."""
    import numpy as np
    load = np.ascontiguousarray(load, dtype=np.int32)
    input_eg = np.ascontiguousarray(input_eg, dtype=np.int32)
    place = np.ascontiguousarray(place, dtype=np.uint8)
    E, G = place.shape
    x = np.zeros((E, G), dtype=np.int32)
    cc = np.zeros(2, dtype=np.int32)
    rc = load_library().fine_comm_replica_loads_host(E, G, load.ctypes.data, input_eg.ctypes.data, place.ctypes.data,
                                                     alpha_num, alpha_den, x.ctypes.data, cc.ctypes.data)
    _check("fine_comm_replica_loads_host", rc)
    return x, (int(cc[0]), int(cc[1]))


def fine_permute(shape: Shape, x, pair_of_row, x_perm):
    cs = shape.c()
    _check("fine_permute", load_library().fine_permute(ctypes.byref(cs), _ptr(x), _ptr(pair_of_row), _ptr(x_perm), _stream()))


def fine_grouped_ffn(shape: Shape, rank: int, x_perm, w_gate, w_up, w_down, seg_off, y_perm, act_save, ws):
    cs = shape.c()
    rc = load_library().fine_grouped_ffn(ctypes.byref(cs), rank, _ptr(x_perm), _ptr(w_gate), _ptr(w_up), _ptr(w_down),
                                         _ptr(seg_off), _ptr(y_perm), _ptr(act_save), _ptr(ws), ws.numel(), _stream())
    _check("fine_grouped_ffn", rc)


def fine_combine(shape: Shape, y_perm, row_of_pair, topk_w, out):
    cs = shape.c()
    _check("fine_combine", load_library().fine_combine(ctypes.byref(cs), _ptr(y_perm), _ptr(row_of_pair), _ptr(topk_w),
                                                       _ptr(out), _stream()))


def fine_backward(shape: Shape, rank: int, d_out, x_perm, y_perm, act_save, w_gate, w_up, w_down, row_of_pair,
                  pair_of_row, seg_off, topk_w, d_x, d_topk_w, d_w_gate, d_w_up, d_w_down, accumulate: bool, ws):
    cs = shape.c()
    rc = load_library().fine_backward(ctypes.byref(cs), rank, _ptr(d_out), _ptr(x_perm), _ptr(y_perm), _ptr(act_save),
                                      _ptr(w_gate), _ptr(w_up), _ptr(w_down), _ptr(row_of_pair), _ptr(pair_of_row),
                                      _ptr(seg_off), _ptr(topk_w), _ptr(d_x), _ptr(d_topk_w), _ptr(d_w_gate),
                                      _ptr(d_w_up), _ptr(d_w_down), 1 if accumulate else 0, _ptr(ws), ws.numel(), _stream())
    _check("fine_backward", rc)


def fine_cayley_placement(shape: Shape, orders, gens, complete: int, place):
    """orders: sequence of ints; gens: sequence of tuples of len(orders) ints (host data); place: device tensor."""
    k = len(orders)
    o = (ctypes.c_int32 * k)(*[int(v) for v in orders])
    flat = [int(v) for s in gens for v in s]
    assert len(flat) == k * len(gens)
    g = (ctypes.c_int32 * max(1, len(flat)))(*flat)
    cs = shape.c()
    rc = load_library().fine_cayley_placement(ctypes.byref(cs), k, ctypes.cast(o, ctypes.c_void_p), len(gens),
                                              ctypes.cast(g, ctypes.c_void_p), complete, _ptr(place), _stream())
    _check("fine_cayley_placement", rc)


def fine_replica_counts(shape: Shape, load, slots: int, counts):
    cs = shape.c()
    _check("fine_replica_counts", load_library().fine_replica_counts(ctypes.byref(cs), _ptr(load), slots, _ptr(counts),
                                                                     _stream()))


def fine_eval_placements(shape: Shape, n: int, place, load, m_num, m_den):
    cs = shape.c()
    _check("fine_eval_placements", load_library().fine_eval_placements(ctypes.byref(cs), n, _ptr(place), _ptr(load),
                                                                       _ptr(m_num), _ptr(m_den), _stream()))


def fine_place_search(shape: Shape, load, counts, slots: int, n: int, seed: int, m_num, m_den, best, place):
    cs = shape.c()
    rc = load_library().fine_place_search(ctypes.byref(cs), _ptr(load), _ptr(counts), slots, n, seed & 0xFFFFFFFF,
                                          _ptr(m_num), _ptr(m_den), _ptr(best), _ptr(place), _stream())
    _check("fine_place_search", rc)


# ---------------------------------------------------------------------------
# Buffer bundles (allocation only; no arithmetic)
# ---------------------------------------------------------------------------

class SchedBuffers:
    """Device tensors for the outputs of fine_sched plus its workspace."""

    def __init__(self, shape: Shape, device="cuda"):
        i32 = dict(dtype=torch.int32, device=device)
        E, G, P = shape.E, shape.G, shape.P
        self.load = torch.empty(E, **i32)
        self.input_eg = torch.empty(E, G, **i32)
        self.x_eg = torch.empty(E, G, **i32)
        self.max_load = torch.empty(1, **i32)
        self.pair_dst = torch.empty(P, **i32)
        self.row_of_pair = torch.empty(P, **i32)
        self.pair_of_row = torch.empty(P, **i32)
        self.seg_off = torch.empty(G, E + 1, **i32)
        self.rank_off = torch.empty(G + 1, **i32)
        self.ws = alloc_workspace(shape, WS_SCHED, device)

    def run(self, shape: Shape, topk_idx, place=None, warm: bool = False):
        """warm: start from the replica loads this object holds from its last run."""
        fine_sched_warm(shape, topk_idx, place, self.x_eg if warm else None, self.load, self.input_eg, self.x_eg, self.max_load, self.pair_dst,
                   self.row_of_pair, self.pair_of_row, self.seg_off, self.rank_off, self.ws)


def shape_of(cfg, flags: int = FLAG_LOCALITY) -> Shape:
    """Shape from a workload LayerConfig (duck typed: T, d, f, E, K, G, dtype)."""
    return Shape(cfg.T, cfg.d, cfg.f, cfg.E, cfg.K, cfg.G, FINE_F32 if cfg.dtype == "f32" else FINE_BF16, flags)
