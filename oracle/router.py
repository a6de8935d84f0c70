"""Oracle: top-K gate (Section 2.1: the gate assigns each token to its top-K experts).

Test infrastructure only; see oracle/__init__.py.

The paper does not print the gate formula.  Reading used here: logits =
x . W_r + b in fp64; the K experts with the largest logits are listed in
descending logit order (equal logits: lower expert index first); the combine
weights are the softmax over those K logits.
"""
import numpy as np


def router_logits(x: np.ndarray, w_router: np.ndarray, bias) -> np.ndarray:
    """logits[T,E] in fp64 from (already dtype-rounded) inputs."""
    x = np.asarray(x, dtype=np.float64)
    w = np.asarray(w_router, dtype=np.float64)
    logits = x @ w
    if bias is not None:
        logits = logits + np.asarray(bias, dtype=np.float64)[None, :]
    return logits


def topk_from_logits(logits: np.ndarray, K: int):
    """(topk_idx[T,K] int32, topk_w[T,K] fp64): one token at a time."""
    T, E = logits.shape
    assert 1 <= K <= E
    idx = np.empty((T, K), dtype=np.int32)
    w = np.empty((T, K), dtype=np.float64)
    for t in range(T):
        row = logits[t]
        chosen = []
        taken = np.zeros(E, dtype=bool)
        for _ in range(K):
            best = -1
            for e in range(E):
                if taken[e]:
                    continue
                if best < 0 or row[e] > row[best]:   # strict: ties keep the lower index
                    best = e
            taken[best] = True
            chosen.append(best)
        sel = row[chosen]
        ex = np.exp(sel - sel.max())
        idx[t] = chosen
        w[t] = ex / ex.sum()
    return idx, w


def topk_from_logits_fast(logits: np.ndarray, K: int):
    """Same result as topk_from_logits through a stable library sort (for
    large T; tests check the two agree)."""
    order = np.argsort(-logits, axis=1, kind="stable")[:, :K]
    sel = np.take_along_axis(logits, order, axis=1)
    ex = np.exp(sel - sel.max(axis=1, keepdims=True))
    return order.astype(np.int32), ex / ex.sum(axis=1, keepdims=True)


def kth_gap(logits: np.ndarray, K: int) -> np.ndarray:
    """Gap between the K-th and (K+1)-th largest logit of each token (inf when
    K == E).  Tokens with a tiny gap may legitimately route differently in a
    lower-precision router."""
    T, E = logits.shape
    if K >= E:
        return np.full(T, np.inf)
    s = -np.sort(-logits, axis=1)
    return s[:, K - 1] - s[:, K]
