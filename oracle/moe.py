"""Oracle: expert computation, combine and their gradients.

Test infrastructure only; see oracle/__init__.py.

Section 2.1: the selected experts process a token and their results are
aggregated; Section 3: any replica of an expert computes a token
equivalently, so scheduling must not change the layer's output.  The FFN is a
SwiGLU MLP without biases (the paper only says "FFN"):
    FFN_e(v) = (silu(v Wg_e) * (v Wu_e)) Wd_e,   silu(a) = a / (1 + exp(-a)).
Everything is fp64; inputs arrive already rounded to the layer dtype.
"""
import numpy as np


def _sigmoid(a):
    return 1.0 / (1.0 + np.exp(-a))


def ffn_rows(X, Wg, Wu, Wd):
    """FFN of one expert on rows X[n,d] (three library matmuls)."""
    a = X @ Wg
    b = X @ Wu
    h = a * _sigmoid(a) * b
    return h @ Wd


def dense_reference(x, topk_idx, topk_w, weights_of):
    """out_ref[t] = sum_k topk_w[t,k] * FFN_{topk_idx[t,k]}(x[t]), token by
    token from the definition; never looks at a schedule.

    weights_of(e) -> (Wg[d,f], Wu[d,f], Wd[f,d]) as fp64 arrays."""
    x = np.asarray(x, dtype=np.float64)
    T, d = x.shape
    K = topk_idx.shape[1]
    out = np.zeros((T, d), dtype=np.float64)
    for t in range(T):
        acc = np.zeros(d, dtype=np.float64)
        for k in range(K):
            Wg, Wu, Wd = weights_of(int(topk_idx[t, k]))
            acc = acc + topk_w[t, k] * ffn_rows(x[t:t + 1], Wg, Wu, Wd)[0]
        out[t] = acc
    return out


def dense_reference_by_expert(x, topk_idx, topk_w, weights_of, tokens=None):
    """Same sums as dense_reference, visiting one expert at a time so that
    each expert's fp64 weights are materialised once.  `tokens` restricts the
    result to a subset of token indices (rows of the result follow `tokens`)."""
    x = np.asarray(x, dtype=np.float64)
    T, d = x.shape
    K = topk_idx.shape[1]
    tokens = np.arange(T) if tokens is None else np.asarray(tokens)
    contrib = np.zeros((tokens.shape[0], K, d), dtype=np.float64)
    sub_idx = topk_idx[tokens]
    for e in np.unique(sub_idx):
        ii, kk = np.nonzero(sub_idx == e)
        Wg, Wu, Wd = weights_of(int(e))
        contrib[ii, kk] = ffn_rows(x[tokens[ii]], Wg, Wu, Wd)
    out = np.zeros((tokens.shape[0], d), dtype=np.float64)
    for k in range(K):                      # k ascending, as in the definition
        out = out + topk_w[tokens, k][:, None] * contrib[:, k]
    return out


def permute(x, pair_of_row, K):
    """x_perm[row] = x[token of pair_of_row[row]] (replicate by top-K, sorted
    order; Section 4.4)."""
    return np.asarray(x)[np.asarray(pair_of_row) // K]


def grouped_ffn(x_perm, seg_off, weights_of):
    """Each rank runs its local replicas on its received rows, one (rank,
    expert) segment at a time (Section 3, Runtime)."""
    x_perm = np.asarray(x_perm, dtype=np.float64)
    G, E1 = seg_off.shape
    y = np.zeros_like(x_perm)
    for e in range(E1 - 1):
        W = None
        for g in range(G):
            lo, hi = int(seg_off[g, e]), int(seg_off[g, e + 1])
            if hi > lo:
                if W is None:
                    W = weights_of(e)
                y[lo:hi] = ffn_rows(x_perm[lo:hi], *W)
    return y


def combine(y_perm, row_of_pair, topk_w):
    """out[t] = sum_k topk_w[t,k] * y_perm[row_of_pair[t*K+k]], k ascending."""
    T, K = topk_w.shape
    rows = np.asarray(row_of_pair).reshape(T, K)
    out = np.zeros((T, y_perm.shape[1]), dtype=np.float64)
    for k in range(K):
        out = out + np.asarray(topk_w, dtype=np.float64)[:, k][:, None] * y_perm[rows[:, k]]
    return out


# --------------------------------------------------------------------------
# gradients of the dense definition (the router is not differentiated)
# --------------------------------------------------------------------------

def backward_dense(x, topk_idx, topk_w, weights_of, d_out, want_weight_grads=True, weight_grad_experts=None):
    """Closed-form gradients of L = sum(out * d_out) for the dense definition.

    With a = v Wg, b = v Wu, s = sigmoid(a), h = a s b, y = h Wd:
      dh = dy Wd^T;  da = dh * b * s * (1 + a (1 - s));  db = dh * a * s;
      dv = da Wg^T + db Wu^T;  dWg = v^T da;  dWu = v^T db;  dWd = h^T dy,
    where dy = topk_w[t,k] * d_out[t] for the pair (t,k), and
      d topk_w[t,k] = <d_out[t], FFN_e(x[t])>.
    Returns dict(d_x, d_topk_w, d_w_gate{e}, d_w_up{e}, d_w_down{e}); weight_grad_experts
    (a collection of expert indices) limits which experts' weight gradients are kept."""
    x = np.asarray(x, dtype=np.float64)
    d_out = np.asarray(d_out, dtype=np.float64)
    topk_w = np.asarray(topk_w, dtype=np.float64)
    T, d = x.shape
    K = topk_idx.shape[1]
    d_x = np.zeros((T, d), dtype=np.float64)
    d_w = np.zeros((T, K), dtype=np.float64)
    gWg, gWu, gWd = {}, {}, {}
    for e in np.unique(topk_idx):
        tt, kk = np.nonzero(topk_idx == e)
        Wg, Wu, Wd = weights_of(int(e))
        v = x[tt]
        a = v @ Wg
        b = v @ Wu
        s = _sigmoid(a)
        h = a * s * b
        y = h @ Wd
        d_w[tt, kk] = np.sum(d_out[tt] * y, axis=1)
        dy = topk_w[tt, kk][:, None] * d_out[tt]
        dh = dy @ Wd.T
        da = dh * b * s * (1.0 + a * (1.0 - s))
        db = dh * a * s
        np.add.at(d_x, tt, da @ Wg.T + db @ Wu.T)
        if want_weight_grads and (weight_grad_experts is None or int(e) in weight_grad_experts):
            gWg[int(e)] = v.T @ da
            gWu[int(e)] = v.T @ db
            gWd[int(e)] = h.T @ dy
    return dict(d_x=d_x, d_topk_w=d_w, d_w_gate=gWg, d_w_up=gWu, d_w_down=gWd)


def layer_loss(x, topk_idx, topk_w, weights_of, d_out):
    """L = sum(out * d_out) of the dense definition (for finite differences)."""
    out = dense_reference_by_expert(x, topk_idx, topk_w, weights_of)
    return float(np.sum(out * np.asarray(d_out, dtype=np.float64)))


def weight_grad_columns(x_rows, dy_rows, Wg, Wu, Wd, cols):
    """Selected columns of one expert's weight gradients without forming whole
    [n,f] matrices: for every j in cols returns
        d_w_gate[:, j], d_w_up[:, j]  (length d)   and   d_w_down[j, :]  (length d),
    from the same formulas as backward_dense, restricted to column j of
    a, b, h and dh.  x_rows[n,d] are the expert's input rows, dy_rows[n,d] the
    gradients of its outputs (already scaled by the combine weights)."""
    x_rows = np.asarray(x_rows, dtype=np.float64)
    dy_rows = np.asarray(dy_rows, dtype=np.float64)
    out = {}
    for j in cols:
        a = x_rows @ Wg[:, j]
        b = x_rows @ Wu[:, j]
        s = _sigmoid(a)
        h = a * s * b
        dh = dy_rows @ Wd[j, :]
        da = dh * b * s * (1.0 + a * (1.0 - s))
        db = dh * a * s
        out[int(j)] = (x_rows.T @ da, x_rows.T @ db, h @ dy_rows)
    return out
