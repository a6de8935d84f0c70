"""Seeded synthetic inputs for one MoE layer under token scheduling.

This module only draws random tensors and builds expert-placement masks.  It
holds none of the method's arithmetic (no routing, no scheduling, no FFN): the
CPU oracle and the HIP library both consume exactly the tensors produced here,
so neither depends on the other.

The five layer shapes are the synthetic skewed-routing workloads the build is
measured on.  They stand in for the routers of the GPT / Mixtral models the
paper trains on Wikipedia (Section 6.1, Table 2 of the appendix): shapes come
from Table 2 (hidden 4096 / FFN 14336 / 8 experts / top-2 is its Mixtral 8x7B
row), skew from a per-expert router bias, because the paper observes that
expert loads are highly skewed and fluctuate (Section 2.3).

Draw recipe (all N(0, sigma) with sigma the standard deviation):
  generator stream "small"  (seed = 1000*seed + 1):  x[T,d] ~ N(0,1),
      W_r[d,E] ~ N(0,0.02), z[E] ~ N(0,1), d_out[T,d] ~ N(0,1) (in this order)
  generator stream per expert e (seed = 1000*seed + 100 + e):
      W_gate[d,f], W_up[d,f], W_down[f,d] ~ N(0,0.02) (in this order)
Every tensor is drawn in fp32 on the requested device with torch's Philox /
mt19937 generator for that device, then rounded once to the layer dtype.  A CPU
draw and a GPU draw of the same seed differ in value (different generators);
within one test or bench run both sides read the same tensors.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Optional

import numpy as np
import torch


@dataclass(frozen=True)
class LayerConfig:
    name: str
    T: int          # tokens
    d: int          # hidden size
    f: int          # expert FFN width
    E: int          # experts
    K: int          # top-K
    G: int          # logical EP ranks
    dtype: str      # "f32" or "bf16"
    seed: int
    bias_kind: str  # "scaled_z" (b = bias_scale * z) or "one_hot" (b[0] = bias_scale)
    bias_scale: float
    backward: bool = False

    @property
    def P(self) -> int:
        return self.T * self.K

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float32 if self.dtype == "f32" else torch.bfloat16


# The five workloads.  cfg4's bias scale 1.0 was chosen offline so that the
# hottest tenth of the experts receives about 40 % of the pairs; cfg5's b_0=+4
# is the binding parameter (the share it produces is reported, not tuned).
CONFIGS: Dict[str, LayerConfig] = {
    "cfg1_tiny_f32": LayerConfig("cfg1_tiny_f32", 256, 128, 256, 8, 2, 4, "f32", 0, "scaled_z", 1.5),
    "cfg2_mixtral": LayerConfig("cfg2_mixtral", 8192, 4096, 14336, 8, 2, 8, "bf16", 1, "scaled_z", 1.0),
    "cfg3_finegrained": LayerConfig("cfg3_finegrained", 4096, 2048, 768, 128, 8, 8, "bf16", 2, "scaled_z", 2.0),
    "cfg4_dsv3": LayerConfig("cfg4_dsv3", 4096, 7168, 2048, 256, 8, 32, "bf16", 3, "scaled_z", 1.0),
    "cfg5_train": LayerConfig("cfg5_train", 32768, 2048, 8192, 64, 2, 16, "bf16", 4, "one_hot", 4.0, True),
}


def scaled(cfg: LayerConfig, **kw) -> LayerConfig:
    """A copy of `cfg` with some fields replaced (used for reduced-size tests)."""
    d = dict(cfg.__dict__)
    d.update(kw)
    return LayerConfig(**d)


@dataclass
class LayerInputs:
    cfg: LayerConfig
    x: torch.Tensor            # [T,d] layer dtype
    w_router: torch.Tensor     # [d,E] layer dtype
    bias: torch.Tensor         # [E] fp32
    d_out: Optional[torch.Tensor]  # [T,d] layer dtype (backward only)
    w_gate: Optional[torch.Tensor] = None   # [E,d,f]
    w_up: Optional[torch.Tensor] = None     # [E,d,f]
    w_down: Optional[torch.Tensor] = None   # [E,f,d]
    extra: dict = field(default_factory=dict)


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _normal(shape, std: float, gen: torch.Generator, device, dtype: torch.dtype) -> torch.Tensor:
    t = torch.randn(shape, generator=gen, device=device, dtype=torch.float32)
    if std != 1.0:
        t.mul_(std)
    return t.to(dtype)


def expert_weights(cfg: LayerConfig, e: int, device="cpu"):
    """(W_gate[d,f], W_up[d,f], W_down[f,d]) of expert e, independent stream per expert."""
    gen = _gen(device, 1000 * cfg.seed + 100 + e)
    dt = cfg.torch_dtype
    wg = _normal((cfg.d, cfg.f), 0.02, gen, device, dt)
    wu = _normal((cfg.d, cfg.f), 0.02, gen, device, dt)
    wd = _normal((cfg.f, cfg.d), 0.02, gen, device, dt)
    return wg, wu, wd


def make_inputs(cfg: LayerConfig, device="cpu", with_weights: bool = True) -> LayerInputs:
    gen = _gen(device, 1000 * cfg.seed + 1)
    dt = cfg.torch_dtype
    x = _normal((cfg.T, cfg.d), 1.0, gen, device, dt)
    w_router = _normal((cfg.d, cfg.E), 0.02, gen, device, dt)
    z = torch.randn((cfg.E,), generator=gen, device=device, dtype=torch.float32)
    if cfg.bias_kind == "scaled_z":
        bias = (cfg.bias_scale * z).contiguous()
    elif cfg.bias_kind == "one_hot":
        bias = torch.zeros_like(z)
        bias[0] = cfg.bias_scale
    else:
        raise ValueError(cfg.bias_kind)
    d_out = _normal((cfg.T, cfg.d), 1.0, gen, device, dt) if cfg.backward else None
    inp = LayerInputs(cfg, x, w_router, bias, d_out)
    if with_weights:
        wg = torch.empty((cfg.E, cfg.d, cfg.f), device=device, dtype=dt)
        wu = torch.empty((cfg.E, cfg.d, cfg.f), device=device, dtype=dt)
        wd = torch.empty((cfg.E, cfg.f, cfg.d), device=device, dtype=dt)
        for e in range(cfg.E):
            a, b, c = expert_weights(cfg, e, device)
            wg[e].copy_(a)
            wu[e].copy_(b)
            wd[e].copy_(c)
            del a, b, c
        inp.w_gate, inp.w_up, inp.w_down = wg, wu, wd
    return inp


# ----------------------------------------------------------------------------
# Routing tables drawn directly (for scheduler-only tests: no router involved)
# ----------------------------------------------------------------------------

def random_topk(T: int, E: int, K: int, seed: int, skew: float = 0.0) -> np.ndarray:
    """topk_idx[T,K] int32: K distinct experts per token, expert popularity
    proportional to (rank+1)^(-skew) (Zipf-like, Section 6.3 uses such loads)."""
    rng = np.random.default_rng(seed)
    p = (np.arange(1, E + 1, dtype=np.float64)) ** (-skew)
    p = p[rng.permutation(E)]
    p /= p.sum()
    out = np.empty((T, K), dtype=np.int32)
    for t in range(T):
        out[t] = rng.choice(E, size=K, replace=False, p=p)
    return out


def drifting_topk_stream(T: int, E: int, K: int, n: int, seed: int, skew: float = 1.0, drift: float = 0.05):
    """Routing tables of n consecutive micro-batches (Section 4.1: the placement
    stays, the loads move a little from one micro-batch to the next).  Token t of
    micro-batch i picks the K largest of bias_i[e] + Gumbel noise; bias_0 is
    skew * log of a seeded Zipf(1) profile and bias_{i+1} = bias_i + drift * N(0,1).
    Yields int32 arrays [T,K] with distinct experts per token."""
    rng = np.random.default_rng(seed)
    bias = -skew * np.log(rng.permutation(E) + 1.0)
    for _ in range(n):
        scores = bias[None, :] + rng.gumbel(size=(T, E))
        yield np.argsort(-scores, axis=1, kind="stable")[:, :K].astype(np.int32)
        bias = bias + drift * rng.standard_normal(E)


def zipf_loads(E: int, total: int, s: float, seed: int) -> np.ndarray:
    """Integer expert loads summing to `total`, the i-th most loaded expert
    proportional to i^(-s); which expert is the i-th is a seeded permutation."""
    rng = np.random.default_rng(seed)
    w = np.arange(1, E + 1, dtype=np.float64) ** (-s)
    w /= w.sum()
    load = np.floor(w * total).astype(np.int64)
    rem = total - int(load.sum())
    load[:rem] += 1
    return load[rng.permutation(E)]


# ----------------------------------------------------------------------------
# Expert placements (masks place[E,G] in {0,1}); inputs of the scheduler
# ----------------------------------------------------------------------------

def placement_full(E: int, G: int) -> np.ndarray:
    return np.ones((E, G), dtype=np.uint8)


def placement_home(E: int, G: int) -> np.ndarray:
    """Vanilla EP: one replica per expert, expert e on rank floor(e*G/E)."""
    m = np.zeros((E, G), dtype=np.uint8)
    for e in range(E):
        m[e, (e * G) // E] = 1
    return m


def placement_from_edges(edges, G: int) -> np.ndarray:
    m = np.zeros((len(edges), G), dtype=np.uint8)
    for e, ranks in enumerate(edges):
        for g in ranks:
            m[e, g] = 1
    return m


def placement_cycle(G: int) -> np.ndarray:
    """Appendix B Example 1: Cayley graph of (Z_G,+) with generators +-1, a
    cycle; expert e joins ranks e and e+1 (mod G).  E = G."""
    return placement_from_edges([(e, (e + 1) % G) for e in range(G)], G)


def placement_complete_plus_matching(G: int) -> np.ndarray:
    """Appendix B Example 4 recipe: all G(G-1)/2 rank pairs, then one extra
    edge for each pair (0,1), (2,3), ...  For G=8 this gives 28+4=32 experts."""
    edges = [(a, b) for a in range(G) for b in range(a + 1, G)]
    edges += [(a, a + 1) for a in range(0, G, 2)]
    return placement_from_edges(edges, G)


def placement_torus4x4() -> np.ndarray:
    """Appendix B Example 2: Z_4 x Z_4 with generators (0,+-1), (+-1,0): the
    4x4 toroidal grid, 16 ranks, 32 experts."""
    edges = []
    for a in range(4):
        for b in range(4):
            v = 4 * a + b
            edges.append((v, 4 * a + (b + 1) % 4))
            edges.append((v, 4 * ((a + 1) % 4) + b))
    return placement_from_edges(edges, 16)


def placement_z2xz4() -> np.ndarray:
    """Appendix B Example 3: Z_2 x Z_4 with generators (0,+-1), (1,+-1); 8
    ranks, 16 experts; isomorphic to K_{4,4}."""
    edges = set()
    for a in range(2):
        for b in range(4):
            v = 4 * a + b
            for (da, db) in ((0, 1), (0, -1), (1, 1), (1, -1)):
                w = 4 * ((a + da) % 2) + (b + db) % 4
                edges.add((min(v, w), max(v, w)))
    return placement_from_edges(sorted(edges), 8)


def placement_circulant(E: int, G: int) -> np.ndarray:
    """Two replicas per expert on a circulant graph (ours, not the paper's):
    expert e joins rank a = e mod G and rank (a + 1 + (floor(e/G) mod (G-1))) mod G."""
    edges = []
    for e in range(E):
        a = e % G
        b = (a + 1 + ((e // G) % (G - 1))) % G
        edges.append((a, b))
    return placement_from_edges(edges, G)
