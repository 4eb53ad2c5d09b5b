"""CPU fp64 oracle for one GPU's MoE expert layer, forward and backward.  TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's cpu_baseline leg may import this file.  It shares no code
with the HIP path and never calls it.  Everything is NumPy float64; `@` (matmul), `argsort(kind="stable")`
and `bincount` are the only library primitives used as steps.

What it computes is the plain definition of the layer the paper names (Section II-A: top-k gated expert FFNs;
notation table in Section III-A: E routed
experts, E_s shared always-active experts, top-k routing, n_mat = 3 SwiGLU matrices; Section III-A memory
model: W_up, W_gate in R^{d x f}, W_down in R^{f x d}, per-expert token sets s_e; Section III-B: dispatch
moves b*s*k rows of d_model values, combine is the reverse).  The paper gives no formula beyond that, so the
following readings are fixed here:

  * gate: softmax over all E logits, the k largest LOGITS are selected (descending, ties -> lower id),
    weight = that probability, divided by the sum over the selected ones when `renorm`;
  * shared experts are extra ids E..E+E_s-1 taken by every token with weight 1, outside the softmax;
  * FFN_e(v) = ( silu(v W_gate[e]) * (v W_up[e]) ) W_down[e],  silu(z) = z / (1 + exp(-z)), no biases;
  * dropless: every slot is processed, no capacity, no padding;
  * the gate weight multiplies the expert output at combine;
  * permutation = stable counting sort of slot ids s = t*K' + j by expert id.

Backward is the exact derivative of L = sum(out * dout) with respect to x (expert path only), the three
weight tensors, the gate weights and the logits.

Pins (tests/test_oracle_*.py): pure-Python brute force of every definition on tiny inputs, central finite
differences of every gradient, torch-CPU float64 autograd on a dense one-hot formulation of the same layer,
closed forms (renorm sums to 1, equal logits, E=1/k=1 reduces to a dense SwiGLU FFN), bijection / stability
invariants of the permutation.  The paper prints no worked numbers for this path, so no pin comes from it.
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


# --------------------------------------------------------------------------------------------------------------
# the learned gating function's linear map (Section II-A): logits = x W_r^T with one weight row per routed expert
# --------------------------------------------------------------------------------------------------------------
def router_logits(x, w_router):
    """logits[t,e] = <x[t], w_router[e]> for x [T,d], w_router [E,d].  The paper only says the gating function is
    learned; a bias-free linear map on the token is the reading fixed here (the usual MoE router)."""
    return np.asarray(x, dtype=F64) @ np.asarray(w_router, dtype=F64).T


def router_logits_bwd(x, w_router, dlogits):
    """Derivative of router_logits: (dx_router [T,d], dw_router [E,d]) for the upstream gradient dlogits [T,E]."""
    dl = np.asarray(dlogits, dtype=F64)
    return dl @ np.asarray(w_router, dtype=F64), dl.T @ np.asarray(x, dtype=F64)


def router_scales(x, w_router, dlogits):
    """Quadrature magnitudes of the terms of (logits, dx_router, dw_router), for the element-wise error bound."""
    x64, w64, dl = np.asarray(x, dtype=F64), np.asarray(w_router, dtype=F64), np.asarray(dlogits, dtype=F64)
    return (np.sqrt((x64 * x64) @ (w64 * w64).T), np.sqrt((dl * dl) @ (w64 * w64)), np.sqrt((dl * dl).T @ (x64 * x64)))


def closed_layer_forward(x, w_router, k, w_gate, w_up, w_down, E_shared=0, renorm=True, logits=None):
    """The layer closed from x: logits = x W_r^T -> top-k gate -> experts -> combine.  `logits`, when given, replaces
    the product (used to make the discrete top-k choice from a lower-precision copy of the logits while everything
    continuous stays in float64).  Returns (out, cache) with cache = (topk_idx, topk_w, probs)."""
    lg = router_logits(x, w_router) if logits is None else np.asarray(logits, dtype=F64)
    idx, w, probs = route_topk(lg, k, E_shared, renorm)
    out, _ = layer_forward(x, idx, w, w_gate, w_up, w_down)
    return out, (idx, w, probs)


def closed_layer_backward(x, w_router, k, w_gate, w_up, w_down, dout, cache, renorm=True):
    """Gradients of L = sum(out * dout) of closed_layer_forward with the top-k choice held fixed (it is piecewise
    constant): dx = expert-path term + router term, dw_router, and the three expert weight gradients."""
    idx, w, probs = cache
    g = layer_backward(x, idx, w, w_gate, w_up, w_down, dout)
    dlogits = route_topk_bwd(g["dtopk_w"], idx, w, probs, k, renorm)
    dx_router, dw_router = router_logits_bwd(x, w_router, dlogits)
    g = dict(g)
    g["dlogits"] = dlogits
    g["dx_router"] = dx_router
    g["dx_total"] = g["dx"] + dx_router
    g["dw_router"] = dw_router
    return g


# --------------------------------------------------------------------------------------------------------------
# routing (Section II-A gating; Section III-A symbols E, E_s, k)
# --------------------------------------------------------------------------------------------------------------


def softmax_rows(logits):
    """Row-wise softmax in float64 with max subtraction."""
    z = np.asarray(logits, dtype=F64)
    z = z - z.max(axis=1, keepdims=True)
    e = np.exp(z)
    return e / e.sum(axis=1, keepdims=True)


def route_topk(logits, k, E_shared=0, renorm=True):
    """Top-k softmax gating.

    logits [T,E] -> (topk_idx [T,K'] int32, topk_w [T,K'] float64, probs [T,E] float64), K' = k + E_shared.
    Selection compares logits (exactly), not probabilities: descending logit, equal logits -> lower expert id.
    """
    z = np.asarray(logits, dtype=F64)
    T, E = z.shape
    assert 1 <= k <= E
    # stable sort of -logit keeps the original (ascending id) order among equal logits
    order = np.argsort(-z, axis=1, kind="stable")
    return gate_of_selection(z, order[:, :k], E_shared, renorm)


def gate_of_selection(logits, sel, E_shared=0, renorm=True):
    """The continuous part of the gate for a GIVEN choice sel [T,k] of routed experts per token: probs = softmax over
    all E logits, weight of slot j = probs[sel_j], divided by the sum over the k chosen ones when `renorm`; shared
    slots appended with ids E.. and weight 1.  route_topk is this function applied to its own choice; a test may
    apply it to another valid choice (the choice is piecewise constant in the logits, so near a tie two choices
    are equally right and everything downstream is defined by the one taken).
    Returns (topk_idx [T,K'] int32, topk_w [T,K'] float64, probs [T,E] float64)."""
    z = np.asarray(logits, dtype=F64)
    T, E = z.shape
    sel = np.asarray(sel).astype(np.int64)
    k = sel.shape[1]
    probs = softmax_rows(z)
    w = np.take_along_axis(probs, sel, axis=1)
    if renorm:
        w = w / w.sum(axis=1, keepdims=True)
    idx = np.empty((T, k + E_shared), dtype=np.int32)
    wt = np.empty((T, k + E_shared), dtype=F64)
    idx[:, :k] = sel
    wt[:, :k] = w
    for j in range(E_shared):
        idx[:, k + j] = E + j
        wt[:, k + j] = 1.0
    return idx, wt, probs


def route_topk_bwd(dtopk_w, topk_idx, topk_w, probs, k, renorm=True):
    """Gradient of the gate weights with respect to the logits.

    renorm: the k weights are a softmax over the selected logits, so for selected j
            dlogit[sel_j] = w_j (dw_j - sum_i w_i dw_i) and 0 elsewhere.
    no renorm: w_j = p_{sel_j}, so dlogit[m] = p_m ( [m selected] dw_m - sum_j p_{sel_j} dw_j ) for every m.
    Shared slots (j >= k) carry constant weight 1 and contribute nothing.
    """
    dw = np.asarray(dtopk_w, dtype=F64)[:, :k]
    idx = np.asarray(topk_idx)[:, :k].astype(np.int64)
    w = np.asarray(topk_w, dtype=F64)[:, :k]
    p = np.asarray(probs, dtype=F64)
    T, E = p.shape
    dlogits = np.zeros((T, E), dtype=F64)
    rows = np.arange(T)[:, None]
    if renorm:
        inner = (w * dw).sum(axis=1, keepdims=True)
        dlogits[rows, idx] = w * (dw - inner)
    else:
        psel = p[rows, idx]
        inner = (psel * dw).sum(axis=1, keepdims=True)
        dlogits = -p * inner
        dlogits[rows, idx] += psel * dw
    return dlogits


# --------------------------------------------------------------------------------------------------------------
# permutation artefacts (local pack before the dispatch of Section III-B)
# --------------------------------------------------------------------------------------------------------------


def permute_maps(topk_idx, n_experts):
    """Stable counting sort of the slots s = t*K' + j by expert id.

    Returns counts [E'], offsets [E'+1] (exclusive prefix sum, offsets[E'] = N), row_of_slot [N],
    slot_of_row [N], all int32."""
    flat = np.asarray(topk_idx).reshape(-1).astype(np.int64)
    N = flat.size
    assert flat.size == 0 or (flat.min() >= 0 and flat.max() < n_experts)
    counts = np.bincount(flat, minlength=n_experts).astype(np.int32)
    offsets = np.zeros(n_experts + 1, dtype=np.int32)
    offsets[1:] = np.cumsum(counts)
    slot_of_row = np.argsort(flat, kind="stable").astype(np.int32)
    row_of_slot = np.empty(N, dtype=np.int32)
    row_of_slot[slot_of_row] = np.arange(N, dtype=np.int32)
    return counts, offsets, row_of_slot, slot_of_row


def permute_rows(x, slot_of_row, K_slots):
    """x_perm[r] = x[slot_of_row[r] // K'] (a copy of rows; works on any dtype, e.g. raw bf16 bit patterns)."""
    x = np.asarray(x)
    return x[np.asarray(slot_of_row, dtype=np.int64) // K_slots]


def permute_bwd(dx_perm, row_of_slot, K_slots):
    """dx[t] = sum_j dx_perm[row_of_slot[t*K'+j]] (the derivative of the row copy)."""
    g = np.asarray(dx_perm, dtype=F64)
    ros = np.asarray(row_of_slot, dtype=np.int64).reshape(-1, K_slots)
    return g[ros].sum(axis=1)


# --------------------------------------------------------------------------------------------------------------
# expert FFN (Section III-A: three matrices per expert, SwiGLU)
# --------------------------------------------------------------------------------------------------------------


def silu(z):
    return z / (1.0 + np.exp(-z))


def silu_grad(z):
    s = 1.0 / (1.0 + np.exp(-z))
    return s * (1.0 + z * (1.0 - s))


def expert_ffn(v, w_gate, w_up, w_down):
    """FFN(v) = (silu(v Wg) * (v Wu)) Wd for rows v [n,d]; Wg, Wu [d,f]; Wd [f,d].  Returns (Y, G, U, H)."""
    v = np.asarray(v, dtype=F64)
    Wg = np.asarray(w_gate, dtype=F64)
    Wu = np.asarray(w_up, dtype=F64)
    Wd = np.asarray(w_down, dtype=F64)
    G = v @ Wg
    U = v @ Wu
    H = silu(G) * U
    return H @ Wd, G, U, H


def expert_of_rows(offsets):
    """Expert id of every permuted row, from the offsets array."""
    offsets = np.asarray(offsets, dtype=np.int64)
    return np.repeat(np.arange(offsets.size - 1), np.diff(offsets))


def grouped_ffn_fwd(x_perm, offsets, w_gate, w_up, w_down, rows=None):
    """Y[r] = FFN_{e(r)}(x_perm[r]) where e(r) is the expert whose segment [offsets[e], offsets[e+1]) holds r.

    rows: optional sorted array of row ids to evaluate (slice mode); default all rows.
    Returns (Y, G, U) for the evaluated rows, in the order of `rows`."""
    xp = np.asarray(x_perm)
    offsets = np.asarray(offsets, dtype=np.int64)
    eor = expert_of_rows(offsets)
    rows = np.arange(xp.shape[0]) if rows is None else np.asarray(rows, dtype=np.int64)
    d = xp.shape[1]
    f = np.asarray(w_gate).shape[2]
    Y = np.zeros((rows.size, d), dtype=F64)
    G = np.zeros((rows.size, f), dtype=F64)
    U = np.zeros((rows.size, f), dtype=F64)
    for e in np.unique(eor[rows]):
        m = np.nonzero(eor[rows] == e)[0]
        y, g, u, _ = expert_ffn(xp[rows[m]], w_gate[e], w_up[e], w_down[e])
        Y[m], G[m], U[m] = y, g, u
    return Y, G, U


def grouped_ffn_bwd(dy_perm, x_perm, offsets, w_gate, w_up, w_down, rows=None, f_cols=None):
    """Backward of grouped_ffn_fwd for upstream gradient dy_perm [N,d].

    Per expert e over its rows: dH = dY Wd^T; dWd = H^T dY; dG = dH * U * silu'(G); dU = dH * silu(G);
    dWg = X^T dG; dWu = X^T dU; dX = dG Wg^T + dU Wu^T.  Experts without rows get dW = 0.

    Slice mode: `rows` restricts dX to those rows (needs the full f of those rows only); `f_cols` restricts the
    weight gradients to those f-indices: dWg[:, :, f_cols], dWu[:, :, f_cols], dWd[:, f_cols, :] (column j of
    dWg needs G, U, dH in column j only, over all rows of the expert).
    Returns (dX [len(rows), d] or None if rows is an empty list, dWg, dWu, dWd) -- the dW are None when
    f_cols is an empty list."""
    xp = np.asarray(x_perm)
    dyp = np.asarray(dy_perm)
    offsets = np.asarray(offsets, dtype=np.int64)
    Et = offsets.size - 1
    N, d = xp.shape
    f = np.asarray(w_gate).shape[2]
    eor = expert_of_rows(offsets)

    dX = None
    want_rows = np.arange(N) if rows is None else np.asarray(rows, dtype=np.int64)
    if want_rows.size:
        dX = np.zeros((want_rows.size, d), dtype=F64)
        for e in np.unique(eor[want_rows]):
            m = np.nonzero(eor[want_rows] == e)[0]
            Wg = np.asarray(w_gate[e], dtype=F64)
            Wu = np.asarray(w_up[e], dtype=F64)
            Wd = np.asarray(w_down[e], dtype=F64)
            X = np.asarray(xp[want_rows[m]], dtype=F64)
            dY = np.asarray(dyp[want_rows[m]], dtype=F64)
            G = X @ Wg
            U = X @ Wu
            dH = dY @ Wd.T
            dG = dH * U * silu_grad(G)
            dU = dH * silu(G)
            dX[m] = dG @ Wg.T + dU @ Wu.T

    dWg = dWu = dWd = None
    cols = np.arange(f) if f_cols is None else np.asarray(f_cols, dtype=np.int64)
    if cols.size:
        dWg = np.zeros((Et, d, cols.size), dtype=F64)
        dWu = np.zeros((Et, d, cols.size), dtype=F64)
        dWd = np.zeros((Et, cols.size, d), dtype=F64)
        for e in range(Et):
            lo, hi = offsets[e], offsets[e + 1]
            if hi == lo:
                continue
            X = np.asarray(xp[lo:hi], dtype=F64)
            dY = np.asarray(dyp[lo:hi], dtype=F64)
            Wg = np.asarray(np.asarray(w_gate[e])[:, cols], dtype=F64)
            Wu = np.asarray(np.asarray(w_up[e])[:, cols], dtype=F64)
            Wd = np.asarray(np.asarray(w_down[e])[cols, :], dtype=F64)
            G = X @ Wg
            U = X @ Wu
            H = silu(G) * U
            dH = dY @ Wd.T
            dG = dH * U * silu_grad(G)
            dU = dH * silu(G)
            dWg[e] = X.T @ dG
            dWu[e] = X.T @ dU
            dWd[e] = H.T @ dY
    return dX, dWg, dWu, dWd


# --------------------------------------------------------------------------------------------------------------
# combine (local unpack after the combine of Section III-B)
# --------------------------------------------------------------------------------------------------------------


def unpermute_combine(y_perm, row_of_slot, topk_w):
    """out[t] = sum_j w[t,j] * y_perm[row_of_slot[t*K'+j]]."""
    y = np.asarray(y_perm, dtype=F64)
    w = np.asarray(topk_w, dtype=F64)
    ros = np.asarray(row_of_slot, dtype=np.int64).reshape(w.shape)
    return (w[:, :, None] * y[ros]).sum(axis=1)


def unpermute_combine_bwd(dout, y_perm, row_of_slot, topk_w):
    """dy_perm[row_of_slot[s]] = w[s] * dout[t(s)];  dtopk_w[t,j] = <dout[t], y_perm[row_of_slot[t*K'+j]]>."""
    g = np.asarray(dout, dtype=F64)
    y = np.asarray(y_perm, dtype=F64)
    w = np.asarray(topk_w, dtype=F64)
    ros = np.asarray(row_of_slot, dtype=np.int64).reshape(w.shape)
    dy = np.zeros_like(y)
    dy[ros] = w[:, :, None] * g[:, None, :]
    dw = (g[:, None, :] * y[ros]).sum(axis=2)
    return dy, dw


# --------------------------------------------------------------------------------------------------------------
# the whole layer, by its per-token definition (no permutation anywhere)
# --------------------------------------------------------------------------------------------------------------


def layer_forward(x, topk_idx, topk_w, w_gate, w_up, w_down, tokens=None):
    """out[t] = sum_{j<K'} w[t,j] * FFN_{idx[t,j]}(x[t]), evaluated per token (grouped by expert only to batch
    the matmuls; no row is moved).  tokens: optional array of token ids (slice mode).
    Returns (out [len(tokens), d], ffn_out [len(tokens), K', d]) -- ffn_out[i,j] = FFN_{idx[t,j]}(x[t])."""
    x = np.asarray(x)
    idx = np.asarray(topk_idx).astype(np.int64)
    w = np.asarray(topk_w, dtype=F64)
    tokens = np.arange(x.shape[0]) if tokens is None else np.asarray(tokens, dtype=np.int64)
    Kp = idx.shape[1]
    d = x.shape[1]
    ffn_out = np.zeros((tokens.size, Kp, d), dtype=F64)
    sub_idx = idx[tokens]
    for e in np.unique(sub_idx):
        ti, ji = np.nonzero(sub_idx == e)
        y, _, _, _ = expert_ffn(x[tokens[ti]], w_gate[e], w_up[e], w_down[e])
        ffn_out[ti, ji] = y
    out = (w[tokens][:, :, None] * ffn_out).sum(axis=1)
    return out, ffn_out


def layer_backward(x, topk_idx, topk_w, w_gate, w_up, w_down, dout, tokens=None, f_cols=None):
    """Gradients of L = sum(out * dout) by the per-token definition.

    For slot (t,j) with expert e: y = FFN_e(x[t]); dtopk_w[t,j] = <dout[t], y>; the slot's upstream gradient is
    dy = w[t,j] dout[t]; dx[t] += dG Wg^T + dU Wu^T; dW*[e] += the slot's outer products.
    tokens restricts dx / dtopk_w to those tokens; f_cols restricts dWg/dWu to those columns and dWd to those
    rows (every token still contributes to the dW).  Pass an empty list to skip either part.
    Returns dict(dx, dtopk_w, dw_gate, dw_up, dw_down)."""
    x = np.asarray(x)
    idx = np.asarray(topk_idx).astype(np.int64)
    w = np.asarray(topk_w, dtype=F64)
    g = np.asarray(dout)
    T, d = x.shape
    Kp = idx.shape[1]
    Et = np.asarray(w_gate).shape[0]
    f = np.asarray(w_gate).shape[2]
    res = {"dx": None, "dtopk_w": None, "dw_gate": None, "dw_up": None, "dw_down": None}

    toks = np.arange(T) if tokens is None else np.asarray(tokens, dtype=np.int64)
    if toks.size:
        dx = np.zeros((toks.size, d), dtype=F64)
        dw = np.zeros((toks.size, Kp), dtype=F64)
        sub_idx = idx[toks]
        for e in np.unique(sub_idx):
            ti, ji = np.nonzero(sub_idx == e)
            Wg = np.asarray(w_gate[e], dtype=F64)
            Wu = np.asarray(w_up[e], dtype=F64)
            Wd = np.asarray(w_down[e], dtype=F64)
            X = np.asarray(x[toks[ti]], dtype=F64)
            D = np.asarray(g[toks[ti]], dtype=F64)
            G = X @ Wg
            U = X @ Wu
            H = silu(G) * U
            Y = H @ Wd
            dw[ti, ji] = (D * Y).sum(axis=1)
            dY = w[toks[ti], ji][:, None] * D
            dH = dY @ Wd.T
            dG = dH * U * silu_grad(G)
            dU = dH * silu(G)
            np.add.at(dx, ti, dG @ Wg.T + dU @ Wu.T)
        res["dx"], res["dtopk_w"] = dx, dw

    cols = np.arange(f) if f_cols is None else np.asarray(f_cols, dtype=np.int64)
    if cols.size:
        dWg = np.zeros((Et, d, cols.size), dtype=F64)
        dWu = np.zeros((Et, d, cols.size), dtype=F64)
        dWd = np.zeros((Et, cols.size, d), dtype=F64)
        for e in range(Et):
            ti, ji = np.nonzero(idx == e)
            if ti.size == 0:
                continue
            Wg = np.asarray(np.asarray(w_gate[e])[:, cols], dtype=F64)
            Wu = np.asarray(np.asarray(w_up[e])[:, cols], dtype=F64)
            Wd = np.asarray(np.asarray(w_down[e])[cols, :], dtype=F64)
            X = np.asarray(x[ti], dtype=F64)
            dY = w[ti, ji][:, None] * np.asarray(g[ti], dtype=F64)
            G = X @ Wg
            U = X @ Wu
            H = silu(G) * U
            dH = dY @ Wd.T
            dG = dH * U * silu_grad(G)
            dU = dH * silu(G)
            dWg[e] = X.T @ dG
            dWu[e] = X.T @ dU
            dWd[e] = H.T @ dY
        res["dw_gate"], res["dw_up"], res["dw_down"] = dWg, dWu, dWd
    return res


def layer_forward_staged(x, topk_idx, topk_w, w_gate, w_up, w_down, n_experts):
    """The same forward as layer_forward, but through the stages the C-ABI exposes (permute -> grouped FFN ->
    combine).  Used by the tests to pin the stage functions to the per-token definition."""
    Kp = np.asarray(topk_idx).shape[1]
    counts, offsets, ros, sor = permute_maps(topk_idx, n_experts)
    xp = permute_rows(np.asarray(x, dtype=F64), sor, Kp)
    Y, _, _ = grouped_ffn_fwd(xp, offsets, w_gate, w_up, w_down)
    return unpermute_combine(Y, ros, topk_w)


def layer_backward_staged(x, topk_idx, topk_w, w_gate, w_up, w_down, dout, n_experts):
    """Backward through the C-ABI's stages: combine_bwd -> grouped FFN bwd -> permute_bwd."""
    Kp = np.asarray(topk_idx).shape[1]
    counts, offsets, ros, sor = permute_maps(topk_idx, n_experts)
    xp = permute_rows(np.asarray(x, dtype=F64), sor, Kp)
    Y, _, _ = grouped_ffn_fwd(xp, offsets, w_gate, w_up, w_down)
    dY, dw = unpermute_combine_bwd(dout, Y, ros, topk_w)
    dXp, dWg, dWu, dWd = grouped_ffn_bwd(dY, xp, offsets, w_gate, w_up, w_down)
    dx = permute_bwd(dXp, ros, Kp)
    return {"dx": dx, "dtopk_w": dw, "dw_gate": dWg, "dw_up": dWu, "dw_down": dWd}


# --------------------------------------------------------------------------------------------------------------
# error measures and per-element magnitude scales used by the parity tests (thresholds live in the tests)
# --------------------------------------------------------------------------------------------------------------
#
# A contraction c_ij = sum_n a_in b_nj evaluated with rounded operands carries an error whose standard deviation
# is proportional to q_ij = sqrt(sum_n a_in^2 b_nj^2), the quadrature magnitude of its terms, and c_ij itself is
# of that magnitude unless its terms cancel.  The *_scales functions below return, for every output of a stage,
# such a magnitude: the same contraction applied to squared operand magnitudes, then a square root, where the
# magnitude of an intermediate is sqrt(value^2 + (its own quadrature)^2) pushed through the element-wise SwiGLU
# steps with first-order sensitivities.  A parity test bounds |got - ref| by rtol*(|ref| + q) element by
# element, so a cancelled (near-zero) element is held to the size of its own terms rather than to zero, and a
# heavy row or column is not hidden behind a global norm.


def quad(a, b):
    """sqrt( (a*a) @ (b*b) ): quadrature magnitude of the terms of a @ b."""
    a = np.asarray(a, dtype=F64)
    b = np.asarray(b, dtype=F64)
    return np.sqrt((a * a) @ (b * b))


def silu_grad2(z):
    """Second derivative of silu: s'(z) (2 + z (1 - 2 s(z))) with s the logistic function."""
    s = 1.0 / (1.0 + np.exp(-z))
    return s * (1.0 - s) * (2.0 + z * (1.0 - 2.0 * s))


def _expert_magnitudes(X, Wg, Wu, Wd):
    """(G, U, s_G, s_U, m_H) of one expert: values, quadrature scales of G and U, magnitude of H."""
    G = X @ Wg
    U = X @ Wu
    sG = quad(X, Wg)
    sU = quad(X, Wu)
    H = silu(G) * U
    mH = np.sqrt(H * H + (silu_grad(G) * U * sG) ** 2 + (silu(G) * sU) ** 2)
    return G, U, sG, sU, mH


def grouped_ffn_fwd_scales(x_perm, offsets, w_gate, w_up, w_down):
    """Scales of (Y, G, U) of grouped_ffn_fwd."""
    xp = np.asarray(x_perm, dtype=F64)
    offsets = np.asarray(offsets, dtype=np.int64)
    N, d = xp.shape
    f = np.asarray(w_gate).shape[2]
    qY, qG, qU = np.zeros((N, d)), np.zeros((N, f)), np.zeros((N, f))
    for e in range(offsets.size - 1):
        lo, hi = offsets[e], offsets[e + 1]
        if hi == lo:
            continue
        Wg = np.asarray(w_gate[e], dtype=F64)
        Wu = np.asarray(w_up[e], dtype=F64)
        Wd = np.asarray(w_down[e], dtype=F64)
        _, _, sG, sU, mH = _expert_magnitudes(xp[lo:hi], Wg, Wu, Wd)
        qG[lo:hi], qU[lo:hi] = sG, sU
        qY[lo:hi] = quad(mH, Wd)
    return qY, qG, qU


def grouped_ffn_bwd_scales(dy_perm, x_perm, offsets, w_gate, w_up, w_down):
    """Scales of (dX, dWg, dWu, dWd) of grouped_ffn_bwd."""
    xp = np.asarray(x_perm, dtype=F64)
    dyp = np.asarray(dy_perm, dtype=F64)
    offsets = np.asarray(offsets, dtype=np.int64)
    Et = offsets.size - 1
    N, d = xp.shape
    f = np.asarray(w_gate).shape[2]
    qX = np.zeros((N, d))
    qWg, qWu, qWd = np.zeros((Et, d, f)), np.zeros((Et, d, f)), np.zeros((Et, f, d))
    for e in range(Et):
        lo, hi = offsets[e], offsets[e + 1]
        if hi == lo:
            continue
        X, dY = xp[lo:hi], dyp[lo:hi]
        Wg = np.asarray(w_gate[e], dtype=F64)
        Wu = np.asarray(w_up[e], dtype=F64)
        Wd = np.asarray(w_down[e], dtype=F64)
        G, U, sG, sU, mH = _expert_magnitudes(X, Wg, Wu, Wd)
        dH = dY @ Wd.T
        mdH = np.sqrt(dH * dH + quad(dY, Wd.T) ** 2)
        mdG = np.sqrt((mdH * U * silu_grad(G)) ** 2 + (dH * silu_grad(G) * sU) ** 2 + (dH * U * silu_grad2(G) * sG) ** 2)
        mdU = np.sqrt((mdH * silu(G)) ** 2 + (dH * silu_grad(G) * sG) ** 2)
        qX[lo:hi] = np.sqrt(quad(mdG, Wg.T) ** 2 + quad(mdU, Wu.T) ** 2)
        qWg[e] = quad(X.T, mdG)
        qWu[e] = quad(X.T, mdU)
        qWd[e] = quad(mH.T, dY)
    return qX, qWg, qWu, qWd


def unpermute_combine_scale(y_scale, row_of_slot, topk_w):
    """Scale of out = sum_j w_j y_j given the magnitude of every y row: sqrt(sum_j w_j^2 m_j^2)."""
    q = np.asarray(y_scale, dtype=F64)
    w = np.asarray(topk_w, dtype=F64)
    ros = np.asarray(row_of_slot, dtype=np.int64).reshape(w.shape)
    return np.sqrt(((w[:, :, None] * q[ros]) ** 2).sum(axis=1))


def layer_scales_staged(x, topk_idx, topk_w, w_gate, w_up, w_down, dout, n_experts):
    """Scales of every output of one forward+backward of the layer (out, dx, dtopk_w, dw_gate, dw_up, dw_down),
    assembled from the stage scales along the staged evaluation."""
    Kp = np.asarray(topk_idx).shape[1]
    w = np.asarray(topk_w, dtype=F64)
    counts, offsets, ros, sor = permute_maps(topk_idx, n_experts)
    xp = permute_rows(np.asarray(x, dtype=F64), sor, Kp)
    Y, _, _ = grouped_ffn_fwd(xp, offsets, w_gate, w_up, w_down)
    qY, _, _ = grouped_ffn_fwd_scales(xp, offsets, w_gate, w_up, w_down)
    mY = np.sqrt(Y * Y + qY * qY)
    q_out = unpermute_combine_scale(mY, ros, w)
    dY, _ = unpermute_combine_bwd(dout, Y, ros, w)
    g = np.asarray(dout, dtype=F64)
    rr = ros.reshape(w.shape)
    q_dw = np.sqrt(((g[:, None, :] * mY[rr]) ** 2).sum(axis=2))
    dX, _, _, _ = grouped_ffn_bwd(dY, xp, offsets, w_gate, w_up, w_down, f_cols=[])
    qX, qWg, qWu, qWd = grouped_ffn_bwd_scales(dY, xp, offsets, w_gate, w_up, w_down)
    mX = np.sqrt(dX * dX + qX * qX)
    q_dx = np.sqrt((mX[rr] ** 2).sum(axis=1))
    return {"out": q_out, "dx": q_dx, "dtopk_w": q_dw, "dw_gate": qWg, "dw_up": qWu, "dw_down": qWd}


def layer_scales(x, topk_idx, topk_w, w_gate, w_up, w_down, dout, n_experts, tokens=None, f_cols=None):
    """The same scales by the per-token definition, with the slice mode of layer_backward: `tokens` restricts out,
    dx and dtopk_w to those tokens, `f_cols` restricts the weight-gradient scales to those f-indices.  Pass an
    empty list to skip either part."""
    x = np.asarray(x)
    idx = np.asarray(topk_idx).astype(np.int64)
    w = np.asarray(topk_w, dtype=F64)
    g = np.asarray(dout)
    T, d = x.shape
    Kp = idx.shape[1]
    f = np.asarray(w_gate).shape[2]
    res = {"out": None, "dx": None, "dtopk_w": None, "dw_gate": None, "dw_up": None, "dw_down": None}

    toks = np.arange(T) if tokens is None else np.asarray(tokens, dtype=np.int64)
    if toks.size:
        q_out2 = np.zeros((toks.size, d), dtype=F64)
        q_dx2 = np.zeros((toks.size, d), dtype=F64)
        q_dw = np.zeros((toks.size, Kp), dtype=F64)
        sub_idx = idx[toks]
        for e in np.unique(sub_idx):
            ti, ji = np.nonzero(sub_idx == e)
            Wg = np.asarray(w_gate[e], dtype=F64)
            Wu = np.asarray(w_up[e], dtype=F64)
            Wd = np.asarray(w_down[e], dtype=F64)
            X = np.asarray(x[toks[ti]], dtype=F64)
            D = np.asarray(g[toks[ti]], dtype=F64)
            wt = w[toks[ti], ji][:, None]
            G, U, sG, sU, mH = _expert_magnitudes(X, Wg, Wu, Wd)
            Y = (silu(G) * U) @ Wd
            mY = np.sqrt(Y * Y + quad(mH, Wd) ** 2)
            np.add.at(q_out2, ti, (wt * mY) ** 2)
            q_dw[ti, ji] = np.sqrt(((D * mY) ** 2).sum(axis=1))
            dY = wt * D
            dH = dY @ Wd.T
            mdH = np.sqrt(dH * dH + quad(dY, Wd.T) ** 2)
            mdG = np.sqrt((mdH * U * silu_grad(G)) ** 2 + (dH * silu_grad(G) * sU) ** 2 + (dH * U * silu_grad2(G) * sG) ** 2)
            mdU = np.sqrt((mdH * silu(G)) ** 2 + (dH * silu_grad(G) * sG) ** 2)
            dG = dH * U * silu_grad(G)
            dU = dH * silu(G)
            dX = dG @ Wg.T + dU @ Wu.T
            np.add.at(q_dx2, ti, dX * dX + quad(mdG, Wg.T) ** 2 + quad(mdU, Wu.T) ** 2)
        res["out"], res["dx"], res["dtopk_w"] = np.sqrt(q_out2), np.sqrt(q_dx2), q_dw

    cols = np.arange(f) if f_cols is None else np.asarray(f_cols, dtype=np.int64)
    if cols.size:
        qWg = np.zeros((n_experts, d, cols.size), dtype=F64)
        qWu = np.zeros((n_experts, d, cols.size), dtype=F64)
        qWd = np.zeros((n_experts, cols.size, d), dtype=F64)
        for e in range(n_experts):
            ti, ji = np.nonzero(idx == e)
            if ti.size == 0:
                continue
            Wg = np.asarray(np.asarray(w_gate[e])[:, cols], dtype=F64)
            Wu = np.asarray(np.asarray(w_up[e])[:, cols], dtype=F64)
            Wd = np.asarray(np.asarray(w_down[e])[cols, :], dtype=F64)
            X = np.asarray(x[ti], dtype=F64)
            dY = w[ti, ji][:, None] * np.asarray(g[ti], dtype=F64)
            G, U, sG, sU, mH = _expert_magnitudes(X, Wg, Wu, Wd)
            dH = dY @ Wd.T
            mdH = np.sqrt(dH * dH + quad(dY, Wd.T) ** 2)
            mdG = np.sqrt((mdH * U * silu_grad(G)) ** 2 + (dH * silu_grad(G) * sU) ** 2 + (dH * U * silu_grad2(G) * sG) ** 2)
            mdU = np.sqrt((mdH * silu(G)) ** 2 + (dH * silu_grad(G) * sG) ** 2)
            qWg[e] = quad(X.T, mdG)
            qWu[e] = quad(X.T, mdU)
            qWd[e] = quad(mH.T, dY)
        res["dw_gate"], res["dw_up"], res["dw_down"] = qWg, qWu, qWd
    return res


def rel_to_max_error(got, ref):
    """max_i |got_i - ref_i| / max_i |ref_i|  (0 when both are all-zero)."""
    got = np.asarray(got, dtype=F64)
    ref = np.asarray(ref, dtype=F64)
    den = np.abs(ref).max() if ref.size else 0.0
    num = np.abs(got - ref).max() if ref.size else 0.0
    if den == 0.0:
        return 0.0 if num == 0.0 else np.inf
    return num / den


def elementwise_excess(got, ref, scale, rtol):
    """max_i ( |got_i - ref_i| - rtol*(|ref_i| + scale_i) ); <= 0 means every element is within bound."""
    got = np.asarray(got, dtype=F64)
    ref = np.asarray(ref, dtype=F64)
    if ref.size == 0:
        return 0.0
    return float((np.abs(got - ref) - rtol * (np.abs(ref) + np.asarray(scale, dtype=F64))).max())


# --------------------------------------------------------------------------------------------------------------
# load balancing through expert migration (Section VI): load statistics and the hill-climbing swap rebalancer
# --------------------------------------------------------------------------------------------------------------
def group_loads(load, groups):
    """s_k = sum of the loads of the experts in group k; `groups` is a list of lists of expert ids."""
    return [int(sum(int(load[e]) for e in g)) for g in groups]


def load_imbalance(load, groups):
    """max_k s_k / mean_k s_k (1.0 = perfectly balanced; 1.0 as well when nothing was routed at all)."""
    s = group_loads(load, groups)
    tot = sum(s)
    return 1.0 if tot == 0 else max(s) * len(s) / tot


def rebalance_hill_climbing(load, groups, max_iters=100):
    """The swap rebalancer of Section VI, Algorithm 2, by brute force from what a step means.

    A step looks at the group with the largest summed load and the one with the smallest.  Every exchange of one
    expert of the former with one of the latter is actually carried out on a copy of the placement, the two sums are
    recomputed from scratch, and the exchange that leaves the smallest difference between them wins, provided that
    difference is smaller than before; if none is, the search ends.  Readings where the paper is silent: the largest /
    smallest group and the winning exchange are the first ones in stored order among equals (groups, then members of
    the heavy group, then members of the light group), and an exchange puts each expert in the other's position.
    Returns (groups, swaps) with swaps = [(expert that left the heavy group, expert that left the light group), ...]
    in the order performed; the input is not modified."""
    placement = [list(g) for g in groups]
    swaps = []
    for _ in range(max_iters):
        sums = group_loads(load, placement)
        heavy = sums.index(max(sums))
        light = sums.index(min(sums))
        before = sums[heavy] - sums[light]
        candidates = []
        for i in range(len(placement[heavy])):
            for j in range(len(placement[light])):
                trial = [list(g) for g in placement]
                trial[heavy][i], trial[light][j] = trial[light][j], trial[heavy][i]
                after = group_loads(load, trial)
                candidates.append((abs(after[heavy] - after[light]), i, j))
        if not candidates:
            break
        after, i, j = min(candidates)          # smallest remaining difference; first (i, j) among equals
        if after >= before:
            break
        swaps.append((placement[heavy][i], placement[light][j]))
        placement[heavy][i], placement[light][j] = placement[light][j], placement[heavy][i]
    return placement, swaps


# --------------------------------------------------------------------------------------------------------------
# the local (single-GPU) steps of the hierarchical all-to-all (Section V, Algorithm 1)
#
# One rank holds a send buffer S [N, D] with N = num_nodes * R rows (R = ranks per node): row n*R + l goes to local
# rank l of node n.  The algorithm's own steps that touch only this rank's memory are written out below in its
# notation as the row maps they define; the exchanges between ranks are not part of this library (halo_all_to_all_reference simulates them
# on the host only to pin the local steps against the definition of an all-to-all).
# --------------------------------------------------------------------------------------------------------------
def halo_remote_nodes(num_nodes, node_id):
    """N_- : the other nodes, in increasing order."""
    return [n for n in range(num_nodes) if n != node_id]


def halo_pack_remote(S, num_nodes, R, node_id):
    """Phase 2 pack, as the row map it defines: row i R + r of the packed buffer is the row of S addressed to local
    rank r of the i-th remote node.  Shape [M R, D]."""
    S = np.asarray(S)
    rem = halo_remote_nodes(num_nodes, node_id)
    out = np.empty((len(rem) * R,) + S.shape[1:], dtype=S.dtype)
    for i, n in enumerate(rem):
        for r in range(R):
            out[i * R + r] = S[n * R + r]
    return out


def halo_repack_phase3(F2r, M, R):
    """Phase 3 repack, as the map it defines: the received buffer holds, for the i-th remote node, one row per local
    rank r (row i R + r); output row r is the concatenation over i of those rows, i.e. everything the remote nodes
    sent for local rank r.  Shape [R, M D]."""
    F2r = np.asarray(F2r)
    D = F2r.shape[1]
    out = np.empty((R, M * D), dtype=F2r.dtype)
    for r in range(R):
        for i in range(M):
            out[r, i * D:(i + 1) * D] = F2r[i * R + r]
    return out


def halo_unpack_output(P1, F3r, num_nodes, R, node_id):
    """Final placement, as the map it defines: output row n R + p is what rank p of node n sent to this rank.  The own
    node's R rows are the phase-1 result; the i-th remote node's row p is the i-th D-wide piece of row p of the
    phase-3 result."""
    P1, F3r = np.asarray(P1), np.asarray(F3r)
    D = P1.shape[1]
    out = np.empty((num_nodes * R, D), dtype=P1.dtype)
    for p in range(R):
        out[node_id * R + p] = P1[p]
        for i, n in enumerate(halo_remote_nodes(num_nodes, node_id)):
            out[n * R + p] = F3r[p, i * D:(i + 1) * D]
    return out


def halo_all_to_all_reference(send, num_nodes, R):
    """The whole three-phase algorithm over all num_nodes*R ranks with the exchanges done by plain host indexing:
    `send[g]` is rank g's S [N, D].  Returns the list of every rank's output O.  (Used only by the pins: the result
    must be the all-to-all, O_g[j] = S_j[g].)"""
    W = num_nodes * R
    rank = lambda n, l: n * R + l  # noqa: E731
    out = []
    P1 = [None] * W
    F2s = [None] * W
    for g in range(W):
        n, l = divmod(g, R)
        F2s[g] = halo_pack_remote(send[g], num_nodes, R, n)
    for g in range(W):
        n, l = divmod(g, R)
        # phase 1: intra-node all-to-all of the node's own R rows: rank l receives row l of every local peer's block
        P1[g] = np.stack([np.asarray(send[rank(n, p)])[n * R + l] for p in range(R)])
    F3r = [None] * W
    F3s = [None] * W
    for g in range(W):
        n, l = divmod(g, R)
        rem = halo_remote_nodes(num_nodes, n)
        # phase 2: slice i of the receive buffer comes from the same local rank of the i-th remote node, which sends
        # the slice it packed for this node
        parts = []
        for src_node in rem:
            peer = rank(src_node, l)
            i_at_peer = halo_remote_nodes(num_nodes, src_node).index(n)
            parts.append(F2s[peer][i_at_peer * R:(i_at_peer + 1) * R])
        F3s[g] = halo_repack_phase3(np.concatenate(parts), len(rem), R) if rem else None
    for g in range(W):
        n, l = divmod(g, R)
        M = num_nodes - 1
        if M:
            D = np.asarray(send[g]).shape[1]
            # phase 3: intra-node all-to-all of the [R, M D] buffers: rank l receives row l of every local peer
            F3r[g] = np.stack([F3s[rank(n, p)][l] for p in range(R)])
        else:
            F3r[g] = np.empty((R, 0), dtype=np.asarray(send[g]).dtype)
        out.append(halo_unpack_output(P1[g], F3r[g], num_nodes, R, n))
    return out
