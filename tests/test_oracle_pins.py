"""Pins for the CPU oracle: everything here runs without a GPU and compares the oracle with something other
than itself -- pure-Python brute force of each definition, closed forms, central finite differences, and
torch-CPU float64 autograd on a dense one-hot formulation of the layer.

The paper (Sections II-A, III-A, III-B) prints no worked numbers for this path, so no pin comes from it; the
hand-computed fixture under tests/golden/ is derived from the definitions, as its header says.
"""
import math
import os

import numpy as np
import pytest
import torch

from oracle import moe_oracle as O
import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------------------------------------------------
# helpers: pure-Python definitions (loops only, no NumPy arithmetic)
# ---------------------------------------------------------------------------------------------------------


def py_softmax(row):
    m = max(row)
    e = [math.exp(v - m) for v in row]
    s = sum(e)
    return [v / s for v in e]


def py_route(logits, k, E_shared, renorm):
    T, E = len(logits), len(logits[0])
    idx, wts = [], []
    for t in range(T):
        p = py_softmax(logits[t])
        taken = []
        for _ in range(k):
            best = None
            for e in range(E):
                if e in taken:
                    continue
                if best is None or logits[t][e] > logits[t][best]:   # strict > keeps the lower id on ties
                    best = e
            taken.append(best)
        w = [p[e] for e in taken]
        if renorm:
            s = sum(w)
            w = [v / s for v in w]
        idx.append(taken + [E + j for j in range(E_shared)])
        wts.append(w + [1.0] * E_shared)
    return idx, wts


def py_ffn(v, Wg, Wu, Wd):
    d, f = len(Wg), len(Wg[0])
    h = []
    for c in range(f):
        g = sum(v[i] * Wg[i][c] for i in range(d))
        u = sum(v[i] * Wu[i][c] for i in range(d))
        h.append(g / (1.0 + math.exp(-g)) * u)
    return [sum(h[c] * Wd[c][i] for c in range(f)) for i in range(d)]


def small_case(T=7, d=5, f=6, E=4, k=2, E_shared=0, seed=0, ties=False):
    rng = np.random.default_rng(seed)
    Et = E + E_shared
    x = rng.standard_normal((T, d))
    Wg = rng.standard_normal((Et, d, f)) * 0.5
    Wu = rng.standard_normal((Et, d, f)) * 0.5
    Wd = rng.standard_normal((Et, f, d)) * 0.5
    logits = rng.standard_normal((T, E))
    if ties:
        logits = np.round(logits * 2) / 2      # many exact ties
    dout = rng.standard_normal((T, d))
    return x, Wg, Wu, Wd, logits, dout


# ---------------------------------------------------------------------------------------------------------
# routing
# ---------------------------------------------------------------------------------------------------------


@pytest.mark.parametrize("renorm", [True, False])
@pytest.mark.parametrize("E_shared", [0, 2])
@pytest.mark.parametrize("ties", [False, True])
def test_route_matches_brute_force(renorm, E_shared, ties):
    for seed in range(4):
        _, _, _, _, logits, _ = small_case(T=9, E=6, k=3, seed=seed, ties=ties)
        idx, w, probs = O.route_topk(logits, 3, E_shared, renorm)
        pidx, pw = py_route(logits.tolist(), 3, E_shared, renorm)
        assert idx.tolist() == pidx
        np.testing.assert_allclose(w, np.array(pw), rtol=1e-13, atol=0)
        for t in range(logits.shape[0]):
            np.testing.assert_allclose(probs[t], py_softmax(logits[t].tolist()), rtol=1e-13)


def test_route_properties_and_closed_forms():
    rng = np.random.default_rng(1)
    logits = rng.standard_normal((50, 16)).astype(np.float32)
    idx, w, p = O.route_topk(logits, 4, 0, True)
    # selected logits dominate unselected ones, indices distinct, descending order
    for t in range(50):
        sel = idx[t]
        assert len(set(sel.tolist())) == 4
        rest = np.setdiff1d(np.arange(16), sel)
        assert logits[t, sel].min() >= logits[t, rest].max()
        assert np.all(np.diff(logits[t, sel]) <= 0)
    np.testing.assert_allclose(w.sum(axis=1), 1.0, rtol=1e-14)
    # k = E without renorm: the weights are the whole softmax, so they sum to 1 and idx is a permutation
    idx, w, p = O.route_topk(logits, 16, 0, False)
    np.testing.assert_allclose(w.sum(axis=1), 1.0, rtol=1e-14)
    assert np.all(np.sort(idx, axis=1) == np.arange(16))
    # E = 1: weight 1 either way
    one = rng.standard_normal((5, 1))
    for rn in (True, False):
        idx, w, _ = O.route_topk(one, 1, 0, rn)
        assert np.all(idx == 0) and np.all(w == 1.0)
    # equal logits: ids 0..k-1 in order, weight 1/k (renorm) or 1/E (no renorm)
    eq = np.full((3, 8), 0.7)
    idx, w, _ = O.route_topk(eq, 3, 0, True)
    assert idx.tolist() == [[0, 1, 2]] * 3
    np.testing.assert_allclose(w, 1.0 / 3, rtol=1e-15)
    idx, w, _ = O.route_topk(eq, 3, 0, False)
    np.testing.assert_allclose(w, 1.0 / 8, rtol=1e-15)
    # shift invariance
    idx0, w0, _ = O.route_topk(logits.astype(np.float64), 4, 0, False)
    idx1, w1, _ = O.route_topk(logits.astype(np.float64) + 3.25, 4, 0, False)
    assert np.array_equal(idx0, idx1)
    np.testing.assert_allclose(w0, w1, rtol=1e-12)
    # experts at -1e30 / -inf are never chosen while k finite logits exist
    lg = logits.copy()
    lg[:, 5] = -1e30
    lg[:, 9] = -np.inf
    idx, w, _ = O.route_topk(lg, 4, 0, True)
    assert not np.any((idx == 5) | (idx == 9))
    assert np.all(np.isfinite(w))
    # shared experts: appended ids, weight 1
    idx, w, _ = O.route_topk(logits, 2, 3, True)
    assert idx[:, 2:].tolist() == [[16, 17, 18]] * 50 and np.all(w[:, 2:] == 1.0)


def test_route_golden_hand_computed():
    """tests/golden/route_small.txt: a 2-token example worked by hand from the definition (ln-valued logits make
    the softmax rational)."""
    rows = [l.split() for l in open(os.path.join(GOLDEN, "route_small.txt")) if l.strip() and l[0] != "#"]
    logits = np.array([[math.log(float(v)) for v in r[1:5]] for r in rows if r[0] == "expw"])
    want_idx = [[int(v) for v in r[1:]] for r in rows if r[0] == "idx"]
    want_w_rn = [[float(eval(v)) for v in r[1:]] for r in rows if r[0] == "w_renorm"]
    want_w = [[float(eval(v)) for v in r[1:]] for r in rows if r[0] == "w_plain"]
    idx, w, _ = O.route_topk(logits, 2, 0, True)
    assert idx.tolist() == want_idx
    np.testing.assert_allclose(w, want_w_rn, rtol=1e-14)
    idx, w, _ = O.route_topk(logits, 2, 0, False)
    np.testing.assert_allclose(w, want_w, rtol=1e-14)


# ---------------------------------------------------------------------------------------------------------
# permutation artefacts
# ---------------------------------------------------------------------------------------------------------


@pytest.mark.parametrize("seed", range(5))
def test_permute_maps_brute_force_and_invariants(seed):
    rng = np.random.default_rng(seed)
    T, Kp, Et = 23, 3, 7
    idx = rng.integers(0, Et - 1, size=(T, Kp))        # expert Et-1 stays empty
    counts, offsets, ros, sor = O.permute_maps(idx, Et)
    flat = idx.reshape(-1).tolist()
    N = T * Kp
    # definition, in loops
    c = [0] * Et
    for e in flat:
        c[e] += 1
    off = [0]
    for e in range(Et):
        off.append(off[-1] + c[e])
    want_ros = []
    for s in range(N):
        want_ros.append(off[flat[s]] + sum(1 for s2 in range(s) if flat[s2] == flat[s]))
    assert counts.tolist() == c and offsets.tolist() == off and ros.tolist() == want_ros
    assert counts[Et - 1] == 0
    # invariants
    assert counts.sum() == N and offsets[-1] == N and np.all(np.diff(offsets) >= 0)
    assert sorted(ros.tolist()) == list(range(N))
    assert np.array_equal(sor[ros], np.arange(N))
    e_of_row = np.array(flat)[sor]
    assert np.all(np.diff(e_of_row) >= 0)
    for e in range(Et):
        seg = sor[offsets[e]:offsets[e + 1]]
        assert np.all(np.diff(seg) > 0)          # stability: slot ids increase inside an expert
    # a library stable sort gives the same order
    assert sor.tolist() == sorted(range(N), key=lambda s: flat[s])
    # row copy
    x = rng.integers(0, 65535, size=(T, 4)).astype(np.uint16)
    xp = O.permute_rows(x, sor, Kp)
    for r in range(N):
        assert np.array_equal(xp[r], x[sor[r] // Kp])


def test_shared_expert_segment_is_identity():
    logits = np.random.default_rng(0).standard_normal((11, 5))
    idx, w, _ = O.route_topk(logits, 2, 2, True)
    counts, offsets, ros, sor = O.permute_maps(idx, 7)
    assert counts[5] == 11 and counts[6] == 11
    for j, e in enumerate((5, 6)):
        seg = sor[offsets[e]:offsets[e + 1]]
        assert np.array_equal(seg // 4, np.arange(11))       # token order
        assert np.all(seg % 4 == 2 + j)


# ---------------------------------------------------------------------------------------------------------
# FFN, combine, whole layer
# ---------------------------------------------------------------------------------------------------------


def test_silu_closed_forms():
    assert O.silu(np.array(0.0)) == 0.0
    np.testing.assert_allclose(O.silu(np.array(math.log(3.0))), math.log(3.0) * 0.75, rtol=1e-15)
    np.testing.assert_allclose(O.silu_grad(np.array(0.0)), 0.5, rtol=1e-15)
    z = np.linspace(-6, 6, 25)
    h = 1e-6
    np.testing.assert_allclose(O.silu_grad(z), (O.silu(z + h) - O.silu(z - h)) / (2 * h), rtol=1e-8, atol=1e-9)
    np.testing.assert_allclose(O.silu_grad2(z), (O.silu_grad(z + h) - O.silu_grad(z - h)) / (2 * h), rtol=1e-7, atol=1e-9)


@pytest.mark.parametrize("E_shared", [0, 1])
def test_layer_forward_matches_per_token_loops(E_shared):
    x, Wg, Wu, Wd, logits, _ = small_case(T=6, d=4, f=5, E=3, k=2, E_shared=E_shared, seed=3)
    idx, w, _ = O.route_topk(logits, 2, E_shared, True)
    out, ffn_out = O.layer_forward(x, idx, w, Wg, Wu, Wd)
    for t in range(6):
        acc = [0.0] * 4
        for j in range(idx.shape[1]):
            e = int(idx[t, j])
            y = py_ffn(x[t].tolist(), Wg[e].tolist(), Wu[e].tolist(), Wd[e].tolist())
            np.testing.assert_allclose(ffn_out[t, j], y, rtol=1e-12, atol=1e-14)
            acc = [a + w[t, j] * v for a, v in zip(acc, y)]
        np.testing.assert_allclose(out[t], acc, rtol=1e-12, atol=1e-14)
    # the staged evaluation (permute -> grouped FFN -> combine) is the same function
    out2 = O.layer_forward_staged(x, idx, w, Wg, Wu, Wd, 3 + E_shared)
    np.testing.assert_allclose(out2, out, rtol=1e-12, atol=1e-14)
    # slice mode returns the same rows
    sub, _ = O.layer_forward(x, idx, w, Wg, Wu, Wd, tokens=[4, 1])
    np.testing.assert_allclose(sub, out[[4, 1]], rtol=1e-14)


def test_dense_reduction_E1_k1_against_torch():
    """E = 1, k = 1: the layer is a plain dense SwiGLU FFN; torch's own silu and matmul define it."""
    x, Wg, Wu, Wd, _, dout = small_case(T=8, d=6, f=9, E=1, k=1, seed=5)
    for rn in (True, False):
        idx, w, _ = O.route_topk(np.zeros((8, 1)), 1, 0, rn)
        out, _ = O.layer_forward(x, idx, w, Wg, Wu, Wd)
        tx, tg, tu, td = (torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (x, Wg[0], Wu[0], Wd[0]))
        ref = (torch.nn.functional.silu(tx @ tg) * (tx @ tu)) @ td
        np.testing.assert_allclose(out, ref.detach().numpy(), rtol=1e-12, atol=1e-14)
        (ref * torch.tensor(dout)).sum().backward()
        g = O.layer_backward(x, idx, w, Wg, Wu, Wd, dout)
        np.testing.assert_allclose(g["dx"], tx.grad.numpy(), rtol=1e-11, atol=1e-13)
        np.testing.assert_allclose(g["dw_gate"][0], tg.grad.numpy(), rtol=1e-11, atol=1e-13)
        np.testing.assert_allclose(g["dw_up"][0], tu.grad.numpy(), rtol=1e-11, atol=1e-13)
        np.testing.assert_allclose(g["dw_down"][0], td.grad.numpy(), rtol=1e-11, atol=1e-13)


def torch_dense_layer(x, Wg, Wu, Wd, logits, k, E_shared, renorm):
    """Independent formulation: every expert runs on every token, a dense [T,E'] gate matrix (zeros for
    unselected experts) combines them.  torch.topk + autograd, float64."""
    E = logits.shape[1]
    p = torch.softmax(logits, dim=1)
    top = torch.topk(logits, k, dim=1)
    sel_p = torch.gather(p, 1, top.indices)
    if renorm:
        sel_p = sel_p / sel_p.sum(dim=1, keepdim=True)
    gate = torch.zeros(x.shape[0], E + E_shared, dtype=torch.float64)
    gate = gate.scatter(1, top.indices, sel_p)
    if E_shared:
        gate = torch.cat([gate[:, :E], torch.ones(x.shape[0], E_shared, dtype=torch.float64)], dim=1)
    out = torch.zeros_like(x)
    for e in range(E + E_shared):
        y = (torch.nn.functional.silu(x @ Wg[e]) * (x @ Wu[e])) @ Wd[e]
        out = out + gate[:, e:e + 1] * y
    return out, top.indices


@pytest.mark.parametrize("renorm", [True, False])
@pytest.mark.parametrize("E_shared", [0, 2])
def test_all_gradients_against_torch_autograd(renorm, E_shared):
    x, Wg, Wu, Wd, logits, dout = small_case(T=10, d=6, f=7, E=5, k=2, E_shared=E_shared, seed=11)
    k = 2
    idx, w, probs = O.route_topk(logits, k, E_shared, renorm)
    tx, tg, tu, td, tl = (torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (x, Wg, Wu, Wd, logits))
    out_t, top_idx = torch_dense_layer(tx, tg, tu, td, tl, k, E_shared, renorm)
    assert np.array_equal(top_idx.numpy(), idx[:, :k])
    out, _ = O.layer_forward(x, idx, w, Wg, Wu, Wd)
    np.testing.assert_allclose(out, out_t.detach().numpy(), rtol=1e-12, atol=1e-14)
    (out_t * torch.tensor(dout)).sum().backward()

    g = O.layer_backward(x, idx, w, Wg, Wu, Wd, dout)
    # torch's dx also holds nothing from the router here because logits is an independent leaf
    np.testing.assert_allclose(g["dx"], tx.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(g["dw_gate"], tg.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(g["dw_up"], tu.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(g["dw_down"], td.grad.numpy(), rtol=1e-10, atol=1e-12)
    dlogits = O.route_topk_bwd(g["dtopk_w"], idx, w, probs, k, renorm)
    np.testing.assert_allclose(dlogits, tl.grad.numpy(), rtol=1e-10, atol=1e-12)

    # the staged backward (combine_bwd -> grouped bwd -> permute_bwd) is the same function
    gs = O.layer_backward_staged(x, idx, w, Wg, Wu, Wd, dout, 5 + E_shared)
    for key in g:
        np.testing.assert_allclose(gs[key], g[key], rtol=1e-11, atol=1e-13)

    # slice mode agrees with the full result
    sl = O.layer_backward(x, idx, w, Wg, Wu, Wd, dout, tokens=[7, 2, 3], f_cols=[5, 0])
    np.testing.assert_allclose(sl["dx"], g["dx"][[7, 2, 3]], rtol=1e-13)
    np.testing.assert_allclose(sl["dtopk_w"], g["dtopk_w"][[7, 2, 3]], rtol=1e-13)
    np.testing.assert_allclose(sl["dw_gate"], g["dw_gate"][:, :, [5, 0]], rtol=1e-13)
    np.testing.assert_allclose(sl["dw_up"], g["dw_up"][:, :, [5, 0]], rtol=1e-13)
    np.testing.assert_allclose(sl["dw_down"], g["dw_down"][:, [5, 0], :], rtol=1e-13)


def test_gradients_by_central_finite_differences():
    x, Wg, Wu, Wd, logits, dout = small_case(T=5, d=4, f=5, E=4, k=2, E_shared=1, seed=21)
    k, Es = 2, 1
    for renorm in (True, False):
        idx, w, probs = O.route_topk(logits, k, Es, renorm)

        def loss(x_=x, Wg_=Wg, Wu_=Wu, Wd_=Wd, lg_=logits):
            i2, w2, _ = O.route_topk(lg_, k, Es, renorm)
            assert np.array_equal(i2, idx)           # perturbations must not change the selection
            o, _ = O.layer_forward(x_, i2, w2, Wg_, Wu_, Wd_)
            return float((o * dout).sum())

        g = O.layer_backward(x, idx, w, Wg, Wu, Wd, dout)
        dlogits = O.route_topk_bwd(g["dtopk_w"], idx, w, probs, k, renorm)
        h = 1e-6
        rng = np.random.default_rng(0)
        for name, arr, grad in (("x_", x, g["dx"]), ("Wg_", Wg, g["dw_gate"]), ("Wu_", Wu, g["dw_up"]),
                                ("Wd_", Wd, g["dw_down"]), ("lg_", logits, dlogits)):
            flat_ids = rng.choice(arr.size, size=min(arr.size, 25), replace=False)
            for fi in flat_ids:
                pos = np.unravel_index(fi, arr.shape)
                ap, am = arr.copy(), arr.copy()
                ap[pos] += h
                am[pos] -= h
                fd = (loss(**{name: ap}) - loss(**{name: am})) / (2 * h)
                assert abs(fd - grad[pos]) <= 1e-6 * max(1.0, abs(grad[pos])), (name, pos, fd, grad[pos])


# ---------------------------------------------------------------------------------------------------------
# the router's linear map and the layer closed from x
# ---------------------------------------------------------------------------------------------------------


def test_router_logits_and_backward_match_loops():
    rng = np.random.default_rng(5)
    T, d, E = 4, 5, 3
    x, wr, dl = rng.standard_normal((T, d)), rng.standard_normal((E, d)), rng.standard_normal((T, E))
    lg = O.router_logits(x, wr)
    dxr, dwr = O.router_logits_bwd(x, wr, dl)
    sl, sx, sw = O.router_scales(x, wr, dl)
    for t in range(T):
        for e in range(E):
            assert abs(lg[t, e] - sum(x[t, i] * wr[e, i] for i in range(d))) < 1e-13
            assert abs(sl[t, e] - math.sqrt(sum((x[t, i] * wr[e, i]) ** 2 for i in range(d)))) < 1e-13
    for t in range(T):
        for i in range(d):
            assert abs(dxr[t, i] - sum(dl[t, e] * wr[e, i] for e in range(E))) < 1e-13
            assert abs(sx[t, i] - math.sqrt(sum((dl[t, e] * wr[e, i]) ** 2 for e in range(E)))) < 1e-13
    for e in range(E):
        for i in range(d):
            assert abs(dwr[e, i] - sum(dl[t, e] * x[t, i] for t in range(T))) < 1e-13
            assert abs(sw[e, i] - math.sqrt(sum((dl[t, e] * x[t, i]) ** 2 for t in range(T)))) < 1e-13
    # a one-hot token reads out a column of the weight; a one-hot upstream gradient reads out a weight row / a token
    assert np.array_equal(O.router_logits(np.eye(d)[2:3], wr)[0], wr[:, 2])
    hot = np.zeros((T, E)); hot[1, 2] = 1.0
    dxh, dwh = O.router_logits_bwd(x, wr, hot)
    assert np.array_equal(dxh[1], wr[2]) and not dxh[[0, 2, 3]].any()
    assert np.array_equal(dwh[2], x[1]) and not dwh[[0, 1]].any()


@pytest.mark.parametrize("renorm", [True, False])
@pytest.mark.parametrize("E_shared", [0, 1])
def test_closed_layer_against_torch_autograd(renorm, E_shared):
    """x is the only leaf on the token side: torch's x.grad then holds the expert-path term plus the router term."""
    x, Wg, Wu, Wd, _, dout = small_case(T=9, d=6, f=5, E=4, k=2, E_shared=E_shared, seed=31)
    wr = np.random.default_rng(32).standard_normal((4, 6))
    k = 2
    out, cache = O.closed_layer_forward(x, wr, k, Wg, Wu, Wd, E_shared, renorm)
    tx, tg, tu, td, tw = (torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (x, Wg, Wu, Wd, wr))
    out_t, top_idx = torch_dense_layer(tx, tg, tu, td, tx @ tw.T, k, E_shared, renorm)
    assert np.array_equal(top_idx.numpy(), cache[0][:, :k])
    np.testing.assert_allclose(out, out_t.detach().numpy(), rtol=1e-12, atol=1e-14)
    (out_t * torch.tensor(dout)).sum().backward()
    g = O.closed_layer_backward(x, wr, k, Wg, Wu, Wd, dout, cache, renorm)
    np.testing.assert_allclose(g["dx_total"], tx.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(g["dw_router"], tw.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(g["dw_gate"], tg.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(g["dw_down"], td.grad.numpy(), rtol=1e-10, atol=1e-12)
    assert np.abs(g["dx_router"]).max() > 1e-3 * np.abs(g["dx"]).max()   # the router term is not negligible here
    # logits given from outside (e.g. a float32 copy) decide the selection; the continuous part is unchanged
    out2, cache2 = O.closed_layer_forward(x, wr, k, Wg, Wu, Wd, E_shared, renorm, logits=O.router_logits(x, wr).astype(np.float32))
    assert np.array_equal(cache2[0], cache[0])
    np.testing.assert_allclose(out2, out, rtol=1e-6)


def test_closed_layer_router_gradients_by_finite_differences():
    x, Wg, Wu, Wd, _, dout = small_case(T=5, d=4, f=5, E=4, k=2, E_shared=0, seed=41)
    wr = np.random.default_rng(42).standard_normal((4, 4))
    out, cache = O.closed_layer_forward(x, wr, 2, Wg, Wu, Wd)
    g = O.closed_layer_backward(x, wr, 2, Wg, Wu, Wd, dout, cache)

    def loss(x_=x, wr_=wr):
        o, c = O.closed_layer_forward(x_, wr_, 2, Wg, Wu, Wd)
        assert np.array_equal(c[0], cache[0])
        return float((o * dout).sum())

    h = 1e-6
    for name, arr, grad in (("x_", x, g["dx_total"]), ("wr_", wr, g["dw_router"])):
        for pos in np.ndindex(arr.shape):
            ap, am = arr.copy(), arr.copy()
            ap[pos] += h
            am[pos] -= h
            fd = (loss(**{name: ap}) - loss(**{name: am})) / (2 * h)
            assert abs(fd - grad[pos]) <= 1e-6 * max(1.0, abs(grad[pos])), (name, pos, fd, grad[pos])


def test_router_weight_generator_matches_the_logit_recipe():
    sh = W.MoEShape(T=64, d_model=128, d_ffn=64, E=8, k=2)
    xb = W.make_tokens(sh, 3)
    wr = W.bf16_bits_to_f32(W.make_router_weight(sh, 3))
    assert wr.shape == (8, 128)
    np.testing.assert_array_equal(O.router_logits(W.bf16_bits_to_f32(xb), wr).astype(np.float32), W.make_router_logits(sh, xb, 3))


def test_empty_expert_gets_zero_dw_and_stage_oracles():
    x, Wg, Wu, Wd, logits, dout = small_case(T=9, d=4, f=6, E=5, k=2, seed=4)
    logits[:, 3] = -1e30
    idx, w, _ = O.route_topk(logits, 2, 0, True)
    g = O.layer_backward(x, idx, w, Wg, Wu, Wd, dout)
    assert not np.any(g["dw_gate"][3]) and not np.any(g["dw_up"][3]) and not np.any(g["dw_down"][3])
    counts, offsets, ros, sor = O.permute_maps(idx, 5)
    assert counts[3] == 0
    # combine / combine_bwd / permute_bwd by loops
    rng = np.random.default_rng(2)
    y = rng.standard_normal((18, 4))
    out = O.unpermute_combine(y, ros, w)
    dy, dw = O.unpermute_combine_bwd(dout, y, ros, w)
    dxp = rng.standard_normal((18, 4))
    dx = O.permute_bwd(dxp, ros, 2)
    for t in range(9):
        acc = np.zeros(4)
        accx = np.zeros(4)
        for j in range(2):
            r = ros[t * 2 + j]
            acc += w[t, j] * y[r]
            accx += dxp[r]
            np.testing.assert_allclose(dy[r], w[t, j] * dout[t], rtol=1e-15)
            np.testing.assert_allclose(dw[t, j], float(np.dot(dout[t], y[r])), rtol=1e-13)
        np.testing.assert_allclose(out[t], acc, rtol=1e-14)
        np.testing.assert_allclose(dx[t], accx, rtol=1e-14)
    # linearity of the layer in W_down and in the gate weights
    o1, _ = O.layer_forward(x, idx, w, Wg, Wu, Wd)
    o2, _ = O.layer_forward(x, idx, 3.0 * w, Wg, Wu, 0.5 * Wd)
    np.testing.assert_allclose(o2, 1.5 * o1, rtol=1e-13)


def test_grouped_ffn_slices():
    x, Wg, Wu, Wd, logits, dout = small_case(T=12, d=4, f=6, E=4, k=2, seed=8)
    idx, w, _ = O.route_topk(logits, 2, 0, True)
    counts, offsets, ros, sor = O.permute_maps(idx, 4)
    xp = O.permute_rows(x, sor, 2)
    dyp = np.random.default_rng(3).standard_normal(xp.shape)
    Y, G, U = O.grouped_ffn_fwd(xp, offsets, Wg, Wu, Wd)
    Ys, Gs, Us = O.grouped_ffn_fwd(xp, offsets, Wg, Wu, Wd, rows=[0, 5, 23])
    np.testing.assert_allclose(Ys, Y[[0, 5, 23]], rtol=1e-14)
    np.testing.assert_allclose(Gs, G[[0, 5, 23]], rtol=1e-14)
    dX, dWg, dWu, dWd = O.grouped_ffn_bwd(dyp, xp, offsets, Wg, Wu, Wd)
    dXs, dWgs, dWus, dWds = O.grouped_ffn_bwd(dyp, xp, offsets, Wg, Wu, Wd, rows=[3, 17], f_cols=[4, 1])
    np.testing.assert_allclose(dXs, dX[[3, 17]], rtol=1e-13)
    np.testing.assert_allclose(dWgs, dWg[:, :, [4, 1]], rtol=1e-13)
    np.testing.assert_allclose(dWus, dWu[:, :, [4, 1]], rtol=1e-13)
    np.testing.assert_allclose(dWds, dWd[:, [4, 1], :], rtol=1e-13)


def test_error_measures_and_scales():
    ref = np.array([[1.0, -2.0], [0.0, 4.0]])
    got = ref + np.array([[0.0, 0.04], [0.0, -0.02]])
    assert abs(O.rel_to_max_error(got, ref) - 0.01) < 1e-15
    assert O.rel_to_max_error(np.zeros(3), np.zeros(3)) == 0.0
    scale = np.array([[0.5, 1.0], [2.0, 0.0]])
    exc = max(0.04 - 0.01 * (2.0 + 1.0), 0.02 - 0.01 * 4.0, -0.01 * 1.5, -0.01 * 2.0)
    assert abs(O.elementwise_excess(got, ref, scale, 0.01) - exc) < 1e-15
    # quadrature magnitude by loops; a one-term contraction has scale |value|
    rng = np.random.default_rng(0)
    a, b = rng.standard_normal((3, 5)), rng.standard_normal((5, 4))
    q = O.quad(a, b)
    for i in range(3):
        for j in range(4):
            assert abs(q[i, j] - math.sqrt(sum((a[i, n] * b[n, j]) ** 2 for n in range(5)))) < 1e-14
    np.testing.assert_allclose(O.quad(a[:, :1], b[:1]), np.abs(a[:, :1] @ b[:1]), rtol=1e-14)
    # stage scales: shapes follow the outputs, empty experts have scale 0, and scale >= |value| / sqrt(terms)
    x, Wg, Wu, Wd, logits, dout = small_case(T=9, d=4, f=6, E=5, k=2, seed=4)
    logits[:, 3] = -1e30
    idx, w, _ = O.route_topk(logits, 2, 0, True)
    sc = O.layer_scales(x, idx, w, Wg, Wu, Wd, dout, 5)
    # per-token evaluation == staged evaluation; slices == full[slice]
    st = O.layer_scales_staged(x, idx, w, Wg, Wu, Wd, dout, 5)
    for key in sc:
        np.testing.assert_allclose(sc[key], st[key], rtol=1e-11, atol=1e-14)
    sl = O.layer_scales(x, idx, w, Wg, Wu, Wd, dout, 5, tokens=[6, 0], f_cols=[3, 1])
    np.testing.assert_allclose(sl["out"], sc["out"][[6, 0]], rtol=1e-13)
    np.testing.assert_allclose(sl["dx"], sc["dx"][[6, 0]], rtol=1e-13)
    np.testing.assert_allclose(sl["dtopk_w"], sc["dtopk_w"][[6, 0]], rtol=1e-13)
    np.testing.assert_allclose(sl["dw_gate"], sc["dw_gate"][:, :, [3, 1]], rtol=1e-13)
    np.testing.assert_allclose(sl["dw_down"], sc["dw_down"][:, [3, 1], :], rtol=1e-13)
    g = O.layer_backward(x, idx, w, Wg, Wu, Wd, dout)
    out, _ = O.layer_forward(x, idx, w, Wg, Wu, Wd)
    assert sc["out"].shape == out.shape and sc["dx"].shape == g["dx"].shape
    assert sc["dtopk_w"].shape == g["dtopk_w"].shape
    for key in ("dw_gate", "dw_up", "dw_down"):
        assert sc[key].shape == g[key].shape and not np.any(sc[key][3]) and np.all(sc[key] >= 0)
        n_terms = 18
        assert np.all(sc[key] * math.sqrt(n_terms) >= np.abs(g[key]) - 1e-12)     # Cauchy-Schwarz


@pytest.mark.parametrize("renorm", [True, False])
def test_gate_of_a_given_selection_matches_loops(renorm):
    """gate_of_selection on a choice that is NOT the top-k (any distinct experts, any order): the weights are the
    softmax probabilities of the chosen experts (over their sum when renormalised), by pure-Python loops."""
    rng = np.random.default_rng(8)
    T, E, k, Es = 9, 6, 3, 2
    logits = rng.standard_normal((T, E)) * 2
    sel = np.stack([rng.permutation(E)[:k] for _ in range(T)])
    idx, w, probs = O.gate_of_selection(logits, sel, Es, renorm)
    for t in range(T):
        p = py_softmax(list(logits[t]))
        ws = [p[e] for e in sel[t]]
        if renorm:
            tot = sum(ws)
            ws = [v / tot for v in ws]
        assert list(idx[t]) == list(sel[t]) + [E, E + 1]
        assert all(abs(w[t, j] - ws[j]) < 1e-15 for j in range(k)) and list(w[t, k:]) == [1.0, 1.0]
        assert all(abs(probs[t, e] - p[e]) < 1e-15 for e in range(E))


def test_scales_are_the_size_of_the_error_of_perturbed_operands():
    """Pins every *_scales function from BOTH sides.  Each float operand of a stage is multiplied by (1 + s*n) with
    n ~ N(0,1) and s = 2^-9 (half a bf16 ulp, the rounding a reduced-precision evaluation applies), the stage is
    re-evaluated in float64, and over many draws the rms error of every single output element must lie within
    [0.3, 3] x s x (its scale).  A scale that is several times too large (which would loosen every element-wise
    parity bound) or too small fails; so does one whose propagation through the SwiGLU chain drops a term."""
    sig, draws = 2.0 ** -9, 200
    rng = np.random.default_rng(5)

    def noisy(a):
        return a * (1.0 + sig * rng.standard_normal(a.shape))

    def check(name, ref, scale, samples):
        err = np.sqrt(np.mean([(s - ref) ** 2 for s in samples], axis=0))
        m = scale > 0
        assert np.all(err[~m] == 0.0), name                      # scale 0 only where nothing can move
        ratio = err[m] / (sig * scale[m])
        assert 0.3 <= ratio.min() and ratio.max() <= 3.0, (name, ratio.min(), ratio.max())

    x, Wg, Wu, Wd, logits, dout = small_case(T=24, d=12, f=10, E=4, k=2, E_shared=1, seed=11)
    logits[:, 3] = -1e30                                          # one empty expert
    Et, Kp = 5, 3
    idx, w, _ = O.route_topk(logits, 2, 1, True)
    counts, offsets, ros, sor = O.permute_maps(idx, Et)
    assert counts[3] == 0
    xp = O.permute_rows(x, sor, Kp)
    dyp = rng.standard_normal(xp.shape) * rng.random((xp.shape[0], 1))

    ref = O.grouped_ffn_fwd(xp, offsets, Wg, Wu, Wd)
    sc = O.grouped_ffn_fwd_scales(xp, offsets, Wg, Wu, Wd)
    smp = [O.grouped_ffn_fwd(noisy(xp), offsets, noisy(Wg), noisy(Wu), noisy(Wd)) for _ in range(draws)]
    for i, name in enumerate(("Y", "G", "U")):
        check("fwd " + name, ref[i], sc[i], [s[i] for s in smp])

    ref = O.grouped_ffn_bwd(dyp, xp, offsets, Wg, Wu, Wd)
    sc = O.grouped_ffn_bwd_scales(dyp, xp, offsets, Wg, Wu, Wd)
    smp = [O.grouped_ffn_bwd(noisy(dyp), noisy(xp), offsets, noisy(Wg), noisy(Wu), noisy(Wd)) for _ in range(draws)]
    for i, name in enumerate(("dX", "dWg", "dWu", "dWd")):
        check("bwd " + name, ref[i], sc[i], [s[i] for s in smp])

    out, _ = O.layer_forward(x, idx, w, Wg, Wu, Wd)
    g = O.layer_backward(x, idx, w, Wg, Wu, Wd, dout)
    outs, gs = [], []
    for _ in range(draws):
        a = (noisy(x), idx, noisy(w), noisy(Wg), noisy(Wu), noisy(Wd))
        outs.append(O.layer_forward(*a)[0])
        gs.append(O.layer_backward(*a, noisy(dout)))
    for fn in (O.layer_scales, O.layer_scales_staged):
        sc = fn(x, idx, w, Wg, Wu, Wd, dout, Et)
        check(fn.__name__ + " out", out, sc["out"], outs)
        for key in ("dx", "dtopk_w", "dw_gate", "dw_up", "dw_down"):
            check(fn.__name__ + " " + key, g[key], sc[key], [s[key] for s in gs])

    ym, wt = rng.standard_normal((ros.size, 7)), rng.random(w.shape)
    check("combine", O.unpermute_combine(ym, ros, wt), O.unpermute_combine_scale(np.abs(ym), ros, wt),
          [O.unpermute_combine(noisy(ym), ros, noisy(wt)) for _ in range(draws)])

    wr, dl = rng.standard_normal((4, 12)) * 0.3, rng.standard_normal((24, 4))
    ql, qx, qw = O.router_scales(x, wr, dl)
    check("logits", O.router_logits(x, wr), ql, [O.router_logits(noisy(x), noisy(wr)) for _ in range(draws)])
    ref = O.router_logits_bwd(x, wr, dl)
    smp = [O.router_logits_bwd(noisy(x), noisy(wr), noisy(dl)) for _ in range(draws)]
    check("dx_router", ref[0], qx, [s[0] for s in smp])
    check("dw_router", ref[1], qw, [s[1] for s in smp])


# ---------------------------------------------------------------------------------------------------------
# workloads (input recipes) -- structure checks that use the oracle's routing
# ---------------------------------------------------------------------------------------------------------


def test_bf16_round_to_nearest_even():
    # 1 + 2^-8 is exactly halfway between bf16 neighbours 1.0 (even) and 1 + 2^-7 (odd) -> rounds to 1.0
    a = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 2.0 ** -7 + 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, -3.1415926],
                 dtype=np.float32)
    b = W.bf16_bits_to_f32(W.f32_to_bf16_bits(a))
    assert b[0] == 1.0 and b[1] == 1.0 and b[2] == np.float32(1.0 + 2.0 ** -6) and b[3] == np.float32(1.0 + 2.0 ** -7)
    assert abs(b[4] + 3.1415926) < 2.0 ** -7 * 2
    t = torch.tensor(a).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(b, t)
    r = np.random.default_rng(0).standard_normal(10000).astype(np.float32)
    assert np.array_equal(W.bf16_bits_to_f32(W.f32_to_bf16_bits(r)),
                          torch.tensor(r).to(torch.bfloat16).to(torch.float32).numpy())


def test_workload_shapes_and_counts():
    s = W.WORKLOADS
    assert s["mixtral"].shape.flops_fwd_bwd() == pytest.approx(8.659e12, rel=1e-3)
    assert s["finegrained"].shape.N == 65536 and s["finegrained"].shape.E_total == 66
    assert s["imbalance"].shape.flops_fwd_bwd() == pytest.approx(4.948e12, rel=1e-3)
    inp = W.make_layer_inputs(s["tiny"], seed=0)
    sh = inp["shape"]
    idx, w, _ = O.route_topk(inp["logits"], sh.k, sh.E_shared, True)
    counts, *_ = O.permute_maps(idx, sh.E_total)
    assert counts.sum() == sh.T * sh.k                 # E[s_e] = T k / E exactly in the mean (Section III-A)
    assert counts.min() > 0


def test_forced_imbalance_recipe_hits_its_target():
    w = W.WORKLOADS["imbalance"]
    s = w.shape
    logits, roles = W.make_forced_imbalance_logits(s, seed=0)
    assert (roles == 2).sum() == 13 and (roles == 0).sum() == 26
    idx, _, _ = O.route_topk(logits, s.k, 0, True)
    counts, *_ = O.permute_maps(idx, s.E)
    assert counts[roles == 0].sum() == 0
    share = counts[roles == 2].sum() / counts.sum()
    assert 0.58 <= share <= 0.62, share


def test_zipf_shard_recipe():
    w = W.WORKLOADS["shard"]
    idx, gw = W.make_zipf_shard_routing(w.shape, seed=0)
    counts, *_ = O.permute_maps(idx, w.shape.E)
    assert counts.sum() == 4096 and counts.max() > 900 and counts.min() < 40
    assert gw.dtype == np.float32 and gw.min() >= 0 and gw.max() < 1
