"""Parity of the HIP path against the CPU fp64 oracle, element by element, through the C ABI.

Bar: routing indices, counts, offsets, both maps and the permuted rows are bit-exact.  Floating-point outputs
and gradients stay within max relative error 2e-2 (bf16 operands, fp32 accumulation, against fp64), read as
BOTH  max|got-ref| / max|ref| <= 2e-2  per tensor and, for every element,  |got-ref| <= 2e-2*(|ref| + q)  where
q is the quadrature magnitude of the terms of the contraction that forms the element (so an element whose
terms cancel is held to the size of its terms, and a dropped tile, row or k-tail cannot hide behind a norm).
The fp32 gate paths (topk_w, probs, dlogits) are held to 1e-5.
"""
import warnings

import numpy as np
import pytest
import torch

import workloads as W
from oracle import moe_oracle as O

pytestmark = pytest.mark.gpu

TOL = 2e-2
TOL_GATE = 1e-5


# ---------------------------------------------------------------------------------------------------------
# helpers
# ---------------------------------------------------------------------------------------------------------

def dev_bf16(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def host_bits(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def host_f32(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        return W.bf16_bits_to_f32(host_bits(t))
    return t.cpu().numpy()


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def assert_close(got, ref, scale, tol=TOL, what=""):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.all(np.isfinite(got)), what
    r = O.rel_to_max_error(got, ref)
    x = O.elementwise_excess(got, ref, scale, tol)
    # the other element-wise reading of the bound, |got-ref| <= tol*|ref| + tol*rms(ref): reported, not enforced (an
    # element of a heavy-tailed tensor whose terms are much larger than the tensor's rms may exceed it legitimately)
    if ref.size:
        rms = float(np.sqrt(np.mean(ref * ref)))
        x_rms = float((np.abs(got - ref) - tol * np.abs(ref) - tol * rms).max())
        if x_rms > 0.0:
            warnings.warn(f"{what}: rms-form element-wise bound exceeded by {x_rms:.3e} (rms(ref) = {rms:.3e})")
    assert r <= tol, f"{what}: max-relative error {r:.3e} > {tol}"
    assert x <= 0.0, f"{what}: element-wise bound exceeded by {x:.3e}"


def f32w(inp, key):
    return W.bf16_bits_to_f32(inp[key])


def ws_for(moe, shape):
    return torch.empty(max(moe.workspace_bytes(shape), 256), dtype=torch.uint8, device="cuda")


# ---------------------------------------------------------------------------------------------------------
# routing
# ---------------------------------------------------------------------------------------------------------

ROUTE_CASES = [
    # T, E, k, E_shared, renorm, kind
    (256, 8, 2, 0, 1, "normal"),
    (100, 8, 8, 0, 0, "normal"),
    (333, 16, 1, 0, 1, "ties"),
    (257, 32, 4, 1, 1, "normal"),
    (1000, 64, 6, 2, 1, "normal"),
    (1000, 64, 6, 2, 0, "ties"),
    (513, 128, 4, 0, 1, "dead"),
    (77, 160, 8, 0, 1, "normal"),
    (50, 384, 16, 3, 0, "ties"),
    (40, 1000, 70, 0, 1, "normal"),
    (1, 8, 2, 0, 1, "normal"),
]


def make_logits(T, E, kind, seed):
    rng = np.random.default_rng(seed)
    lg = rng.standard_normal((T, E)).astype(np.float32) * 2
    if kind == "ties":
        lg = np.round(lg * 2) / 2
    if kind == "dead":
        lg[:, rng.choice(E, E // 5, replace=False)] = -1e30
        lg[:, 3] = -np.inf
    return lg.astype(np.float32)


@pytest.mark.parametrize("T,E,k,Es,renorm,kind", ROUTE_CASES)
def test_route_topk_and_bwd(moe, T, E, k, Es, renorm, kind):
    s = moe.Shape(T, 64, 64, E, k, Es, renorm)
    lg = make_logits(T, E, kind, seed=T + E)
    idx_ref, w_ref, p_ref = O.route_topk(lg, k, Es, bool(renorm))
    d_lg = dev(lg)
    idx = torch.full((T, k + Es), -7, dtype=torch.int32, device="cuda")
    w = torch.zeros((T, k + Es), dtype=torch.float32, device="cuda")
    probs = torch.zeros((T, E), dtype=torch.float32, device="cuda")
    moe.moe_route_topk(s, d_lg, idx, w, probs)
    torch.cuda.synchronize()
    assert np.array_equal(idx.cpu().numpy(), idx_ref)                      # bit-exact indices
    np.testing.assert_allclose(w.cpu().numpy(), w_ref, rtol=TOL_GATE, atol=1e-30)
    np.testing.assert_allclose(probs.cpu().numpy(), p_ref, rtol=TOL_GATE, atol=1e-30)
    # probs_save may be omitted
    idx2 = torch.zeros_like(idx)
    w2 = torch.zeros_like(w)
    moe.moe_route_topk(s, d_lg, idx2, w2, None)
    assert torch.equal(idx2, idx) and torch.equal(w2, w)
    # backward
    rng = np.random.default_rng(5)
    dw = rng.standard_normal((T, k + Es)).astype(np.float32)
    dl_ref = O.route_topk_bwd(dw, idx_ref, w.cpu().numpy(), probs.cpu().numpy(), k, bool(renorm))
    dl = torch.full((T, E), 99.0, dtype=torch.float32, device="cuda")
    moe.moe_route_topk_bwd(s, dev(dw), idx, w, probs, dl)
    torch.cuda.synchronize()
    # dlogits is a difference of products of w (<= 1) and dw, so fp32 rounding scales with max|dw| (k = 1 with
    # renorm has the exact result 0)
    scale = np.abs(dw).max()
    assert np.abs(dl.cpu().numpy() - dl_ref).max() <= TOL_GATE * scale


# ---------------------------------------------------------------------------------------------------------
# permutation and the streaming kernels
# ---------------------------------------------------------------------------------------------------------

PERM_CASES = [
    # T, d, E, k, E_shared, kind
    (256, 512, 8, 2, 0, "uniform"),
    (1500, 128, 5, 3, 0, "skewed"),          # N = 4500: several 1024-slot blocks and a ragged tail
    (1111, 192, 64, 6, 2, "uniform"),
    (4096, 64, 32, 1, 0, "skewed"),          # k = 1: an expert-parallel shard
    (3000, 64, 128, 4, 0, "dead"),
    (700, 64, 1000, 5, 24, "uniform"),       # E' = 1024, the ABI limit
    (1, 64, 8, 2, 0, "uniform"),
    (600, 64, 4, 4, 0, "uniform"),           # k = E
]


def make_topk_idx(T, E, k, Es, kind, seed):
    rng = np.random.default_rng(seed)
    if kind == "uniform":
        p = np.ones(E)
    elif kind == "skewed":
        p = 1.0 / np.arange(1, E + 1) ** 1.2
    else:
        p = np.ones(E)
        p[rng.choice(E, E // 5, replace=False)] = 0.0
        p[: max(E // 10, 1)] *= 30
    p = p / p.sum()
    idx = np.empty((T, k + Es), dtype=np.int32)
    for t in range(T):
        idx[t, :k] = rng.choice(E, size=k, replace=False, p=p)
    for j in range(Es):
        idx[:, k + j] = E + j
    return idx


@pytest.mark.parametrize("T,d,E,k,Es,kind", PERM_CASES)
def test_permute_maps_rows_and_streams(moe, T, d, E, k, Es, kind):
    s = moe.Shape(T, d, 64, E, k, Es, 1)
    Et, Kp, N = E + Es, k + Es, T * (k + Es)
    idx = make_topk_idx(T, E, k, Es, kind, seed=T)
    xb = W.make_tokens(W.MoEShape(T, d, 64, E, k, Es), seed=T)
    counts_ref, offsets_ref, ros_ref, sor_ref = O.permute_maps(idx, Et)
    ws = ws_for(moe, s)
    d_idx, d_x = dev(idx), dev_bf16(xb)
    outs = []
    for rep in range(2):            # twice: the result must not depend on scheduling
        counts = torch.full((Et,), -1, dtype=torch.int32, device="cuda")
        offsets = torch.full((Et + 1,), -1, dtype=torch.int32, device="cuda")
        ros = torch.full((N,), -1, dtype=torch.int32, device="cuda")
        sor = torch.full((N,), -1, dtype=torch.int32, device="cuda")
        xp = torch.zeros((N, d), dtype=torch.bfloat16, device="cuda")
        moe.moe_permute(s, d_x, d_idx, xp, counts, offsets, ros, sor, ws)
        torch.cuda.synchronize()
        outs.append((counts, offsets, ros, sor, xp))
    counts, offsets, ros, sor, xp = outs[0]
    assert np.array_equal(counts.cpu().numpy(), counts_ref)
    assert np.array_equal(offsets.cpu().numpy(), offsets_ref)
    assert np.array_equal(ros.cpu().numpy(), ros_ref)
    assert np.array_equal(sor.cpu().numpy(), sor_ref)
    assert np.array_equal(host_bits(xp), O.permute_rows(xb, sor_ref, Kp))
    for a, b in zip(outs[0], outs[1]):
        assert torch.equal(a, b)
    # maps only (x, x_perm both NULL)
    ros2 = torch.zeros_like(ros)
    sor2 = torch.zeros_like(sor)
    moe.moe_permute(s, None, d_idx, None, counts, offsets, ros2, sor2, ws)
    assert torch.equal(ros2, ros) and torch.equal(sor2, sor)

    # combine, combine_bwd, permute_bwd on random bf16 rows
    rng = np.random.default_rng(T + 1)
    yb = W.f32_to_bf16_bits(rng.standard_normal((N, d)).astype(np.float32))
    gb = W.f32_to_bf16_bits(rng.standard_normal((T, d)).astype(np.float32))
    wt = rng.random((T, Kp)).astype(np.float32)
    y64, g64 = W.bf16_bits_to_f32(yb), W.bf16_bits_to_f32(gb)
    d_y, d_g, d_w = dev_bf16(yb), dev_bf16(gb), dev(wt)
    out = torch.zeros((T, d), dtype=torch.bfloat16, device="cuda")
    moe.moe_unpermute_combine(s, d_y, ros, d_w, out)
    assert_close(host_f32(out), O.unpermute_combine(y64, ros_ref, wt),
                 O.unpermute_combine_scale(np.abs(y64), ros_ref, wt), what="combine")
    dy = torch.zeros((N, d), dtype=torch.bfloat16, device="cuda")
    dtw = torch.zeros((T, Kp), dtype=torch.float32, device="cuda")
    moe.moe_unpermute_combine_bwd(s, d_g, d_y, ros, d_w, dy, dtw)
    dy_ref, dtw_ref = O.unpermute_combine_bwd(g64, y64, ros_ref, wt)
    assert_close(host_f32(dy), dy_ref, 0.0, what="combine_bwd dy")
    q_dtw = np.sqrt(((g64.astype(np.float64)[:, None, :] * y64[ros_ref.reshape(T, Kp)]) ** 2).sum(axis=2))
    assert_close(dtw.cpu().numpy(), dtw_ref, q_dtw, tol=1e-4, what="combine_bwd dtopk_w")
    dx = torch.zeros((T, d), dtype=torch.bfloat16, device="cuda")
    moe.moe_permute_bwd(s, d_y, ros, dx)
    assert_close(host_f32(dx), O.permute_bwd(y64, ros_ref, Kp),
                 O.unpermute_combine_scale(np.abs(y64), ros_ref, np.ones((T, Kp))), what="permute_bwd")


def test_permute_is_deterministic_over_100_runs(moe):
    """The order of equal keys never depends on scheduling: 100 runs of one larger shape (64 rank blocks, 128
    experts of which a fifth are empty and a tenth are hot), every output bit for bit the first run's and the oracle's."""
    T, d, E, k = 16384, 256, 128, 4
    s = moe.Shape(T, d, 64, E, k, 0, 1)
    N = T * k
    rng = np.random.default_rng(77)
    p = np.ones(E)
    p[rng.choice(E, E // 5, replace=False)] = 0.0
    p[: E // 10] *= 30
    # top-k without replacement by the Gumbel trick (input recipe only)
    keys = np.log(np.maximum(p, 1e-300))[None, :] + rng.gumbel(size=(T, E))
    idx = np.argsort(-keys, axis=1)[:, :k].astype(np.int32)
    xb = W.make_tokens(W.MoEShape(T, d, 64, E, k, 0), seed=3)
    counts_ref, offsets_ref, ros_ref, sor_ref = O.permute_maps(idx, E)
    ws = ws_for(moe, s)
    d_idx, d_x = dev(idx), dev_bf16(xb)
    first = None
    for rep in range(100):
        counts = torch.full((E,), -1, dtype=torch.int32, device="cuda")
        offsets = torch.full((E + 1,), -1, dtype=torch.int32, device="cuda")
        ros = torch.full((N,), -1, dtype=torch.int32, device="cuda")
        sor = torch.full((N,), -1, dtype=torch.int32, device="cuda")
        xp = torch.zeros((N, d), dtype=torch.bfloat16, device="cuda")
        moe.moe_permute(s, d_x, d_idx, xp, counts, offsets, ros, sor, ws)
        cur = (counts, offsets, ros, sor, xp)
        if first is None:
            first = cur
            assert np.array_equal(counts.cpu().numpy(), counts_ref) and np.array_equal(offsets.cpu().numpy(), offsets_ref)
            assert np.array_equal(ros.cpu().numpy(), ros_ref) and np.array_equal(sor.cpu().numpy(), sor_ref)
            assert np.array_equal(host_bits(xp), O.permute_rows(xb, sor_ref, k))
        else:
            for a, b in zip(first, cur):
                assert torch.equal(a, b), rep


def test_permute_empty_batch(moe):
    s = moe.Shape(0, 64, 64, 8, 2, 0, 1)
    ws = ws_for(moe, s)
    counts = torch.full((8,), -1, dtype=torch.int32, device="cuda")
    offsets = torch.full((9,), -1, dtype=torch.int32, device="cuda")
    e_i = torch.zeros((16,), dtype=torch.int32, device="cuda")
    e_b = torch.zeros((16,), dtype=torch.bfloat16, device="cuda")
    moe.moe_permute(s, e_b, e_i, e_b, counts, offsets, e_i, e_i, ws)
    torch.cuda.synchronize()
    assert counts.cpu().tolist() == [0] * 8 and offsets.cpu().tolist() == [0] * 9


# ---------------------------------------------------------------------------------------------------------
# grouped FFN, stage by stage
# ---------------------------------------------------------------------------------------------------------

FFN_CASES = [
    # T, d, f, E, k, E_shared, dead experts
    (300, 192, 320, 5, 2, 0, 1),       # d, f multiples of 64 but not of 128: column masks; one empty expert
    (256, 512, 1024, 8, 2, 0, 0),      # the tiny workload's shape
    (700, 128, 256, 3, 1, 1, 0),       # ~230 rows per expert + a 700-row shared expert: several row tiles, ragged
    (90, 256, 128, 16, 2, 0, 5),       # experts with a handful of rows
    (600, 256, 2048, 2, 1, 0, 0),      # few tiles and a long K in Y = H W_down and dX: the last-round tiles are split along K
    (513, 64, 64, 1, 1, 0, 0),         # one expert, the smallest legal widths, a one-row third tile
    (40, 128, 192, 24, 1, 0, 20),      # most experts empty: zero-filled weight gradients, experts ordered by row count
]


def staged_inputs(T, d, f, E, k, Es, dead, seed=0):
    shape = W.MoEShape(T, d, f, E, k, Es)
    inp = W.random_layer_inputs(shape, seed=seed, dead_experts=dead)
    idx, w, probs = O.route_topk(inp["logits"], k, Es, True)
    counts, offsets, ros, sor = O.permute_maps(idx, E + Es)
    xp_bits = O.permute_rows(inp["x"], sor, k + Es)
    return shape, inp, idx, w, counts, offsets, ros, sor, xp_bits


@pytest.mark.parametrize("T,d,f,E,k,Es,dead", FFN_CASES)
def test_grouped_ffn_fwd_bwd(moe, T, d, f, E, k, Es, dead):
    shape, inp, idx, w, counts, offsets, ros, sor, xp_bits = staged_inputs(T, d, f, E, k, Es, dead)
    if dead:
        assert counts.min() == 0
    s = moe.Shape.of(shape)
    N, Et = s.N, s.E_total
    ws = ws_for(moe, s)
    d_xp, d_off = dev_bf16(xp_bits), dev(offsets)
    d_wg, d_wu, d_wd = dev_bf16(inp["w_gate"]), dev_bf16(inp["w_up"]), dev_bf16(inp["w_down"])
    y = torch.zeros((N, d), dtype=torch.bfloat16, device="cuda")
    sg = torch.zeros((N, f), dtype=torch.bfloat16, device="cuda")
    su = torch.zeros((N, f), dtype=torch.bfloat16, device="cuda")
    moe.moe_grouped_ffn_fwd(s, d_xp, d_off, d_wg, d_wu, d_wd, y, sg, su, ws)
    torch.cuda.synchronize()
    wg, wu, wd = f32w(inp, "w_gate"), f32w(inp, "w_up"), f32w(inp, "w_down")
    xp = W.bf16_bits_to_f32(xp_bits)
    Y, G, U = O.grouped_ffn_fwd(xp, offsets, wg, wu, wd)
    qY, qG, qU = O.grouped_ffn_fwd_scales(xp, offsets, wg, wu, wd)
    assert_close(host_f32(sg), G, qG, what="save_g")
    assert_close(host_f32(su), U, qU, what="save_u")
    assert_close(host_f32(y), Y, qY, what="y_perm")

    # backward with an upstream gradient of the combine's scale
    rng = np.random.default_rng(9)
    dy_bits = W.f32_to_bf16_bits((rng.standard_normal((N, d)) * rng.random((N, 1))).astype(np.float32))
    dyp = W.bf16_bits_to_f32(dy_bits)
    dX, dWg, dWu, dWd = O.grouped_ffn_bwd(dyp, xp, offsets, wg, wu, wd)
    dxp = torch.zeros((N, d), dtype=torch.bfloat16, device="cuda")
    gwg = torch.full((Et, d, f), 7.0, dtype=torch.float32, device="cuda")
    gwu = torch.full((Et, d, f), 7.0, dtype=torch.float32, device="cuda")
    gwd = torch.full((Et, f, d), 7.0, dtype=torch.float32, device="cuda")
    moe.moe_grouped_ffn_bwd(s, dev_bf16(dy_bits), d_xp, d_off, d_wg, d_wu, d_wd, sg, su, dxp, gwg, gwu, gwd, 0, ws)
    torch.cuda.synchronize()
    qX, qWg, qWu, qWd = O.grouped_ffn_bwd_scales(dyp, xp, offsets, wg, wu, wd)
    assert_close(host_f32(dxp), dX, qX, what="dx_perm")
    assert_close(gwg.cpu().numpy(), dWg, qWg, what="dw_gate")
    assert_close(gwu.cpu().numpy(), dWu, qWu, what="dw_up")
    assert_close(gwd.cpu().numpy(), dWd, qWd, what="dw_down")
    for e in np.nonzero(counts == 0)[0]:      # empty experts: exact zeros when overwriting
        assert not gwg[e].any() and not gwu[e].any() and not gwd[e].any()
    # accumulate = 1 adds to what is there (and leaves empty experts untouched)
    base = 0.25
    gwg.fill_(base); gwu.fill_(base); gwd.fill_(base)
    moe.moe_grouped_ffn_bwd(s, dev_bf16(dy_bits), d_xp, d_off, d_wg, d_wu, d_wd, sg, su, dxp, gwg, gwu, gwd, 1, ws)
    torch.cuda.synchronize()
    assert_close(gwg.cpu().numpy() - base, dWg, qWg + 1e-5, what="dw_gate accumulate")
    assert_close(gwd.cpu().numpy() - base, dWd, qWd + 1e-5, what="dw_down accumulate")
    for e in np.nonzero(counts == 0)[0]:
        assert torch.all(gwu[e] == base)


HEIGHT_COUNTS = [1, 31, 33, 64, 65, 128, 129, 256, 257, 300, 320, 321, 0, 577, 512 + 65]
FEW_COUNTS = [33, 300, 65, 0, 130]
MANY_TILE_COUNTS = [1300, 70, 0, 1400, 1024 + 30]   # 5 row tiles with a tall last one, 6 with a short last one, 4 with a tall one


@pytest.mark.parametrize("d,f,counts", [(128, 256, HEIGHT_COUNTS), (256, 1088, HEIGHT_COUNTS), (3072, 256, HEIGHT_COUNTS),
                                        (128, 3136, HEIGHT_COUNTS), (3072, 1536, FEW_COUNTS),
                                        (256, 2304, MANY_TILE_COUNTS)])
def test_grouped_ffn_every_tile_height(moe, d, f, counts):
    """Experts whose row counts hit every height class of a row tile and both sides of every class boundary: 1..64 rows
    (one 32-row block per wavefront), 65..128, 129..256, 257..320 (a full tile that carries up to 64 more rows), 321
    (a full tile plus a short one), an empty expert, and a multi-tile expert whose remainder rides on its last tile.
    (f = 1088 = 4 * 256 + 64 also puts a 64-wide last column tile on every class.  The last two shapes make few tiles
    with a contraction of 48 k-steps or more, which the kernels then cut along K: d = 3072 in dH, whose arriving part
    applies the d(SwiGLU) epilogue to the summed parts, and f = 3136 = 49 * 64 in the down projection and in dX; the
    fifth case, on a few experts, has both dH and dX cut their tiles in one backward call, one after the other on the
    same arrival counters.  The last case has experts of more than four row tiles, which the kernels walk column tile by
    column tile with a tall tile first, next to one of four row tiles, walked in bands of 8 column tiles: f = 2304 is 9
    column tiles, i.e. a full band and a band of one.)"""
    counts = np.array(counts, dtype=np.int64)
    E, N = counts.size, int(counts.sum())
    offsets = np.zeros(E + 1, dtype=np.int32)
    offsets[1:] = np.cumsum(counts)
    shape = W.MoEShape(N, d, f, E, 1)        # (T = N rows with one slot each: only the sizes matter here)
    s = moe.Shape.of(shape)
    rng = np.random.default_rng(d + f)
    xp_bits = W.f32_to_bf16_bits(rng.standard_normal((N, d)).astype(np.float32))
    dy_bits = W.f32_to_bf16_bits((rng.standard_normal((N, d)) * rng.random((N, 1))).astype(np.float32))
    wgb, wub, wdb = W.make_expert_weights(shape, seed=1, std=0.05)
    ws = ws_for(moe, s)
    d_xp, d_off = dev_bf16(xp_bits), dev(offsets)
    d_wg, d_wu, d_wd = dev_bf16(wgb), dev_bf16(wub), dev_bf16(wdb)
    y = torch.full((N, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    sg = torch.full((N, f), float("nan"), dtype=torch.bfloat16, device="cuda")
    su = torch.full((N, f), float("nan"), dtype=torch.bfloat16, device="cuda")
    moe.moe_grouped_ffn_fwd(s, d_xp, d_off, d_wg, d_wu, d_wd, y, sg, su, ws)
    xp, dyp = W.bf16_bits_to_f32(xp_bits), W.bf16_bits_to_f32(dy_bits)
    wg, wu, wd = W.bf16_bits_to_f32(wgb), W.bf16_bits_to_f32(wub), W.bf16_bits_to_f32(wdb)
    Y, G, U = O.grouped_ffn_fwd(xp, offsets, wg, wu, wd)
    qY, qG, qU = O.grouped_ffn_fwd_scales(xp, offsets, wg, wu, wd)
    assert_close(host_f32(sg), G, qG, what="save_g")
    assert_close(host_f32(su), U, qU, what="save_u")
    assert_close(host_f32(y), Y, qY, what="y_perm")
    dxp = torch.full((N, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    gwg = torch.full((E, d, f), 7.0, dtype=torch.float32, device="cuda")
    gwu = torch.full((E, d, f), 7.0, dtype=torch.float32, device="cuda")
    gwd = torch.full((E, f, d), 7.0, dtype=torch.float32, device="cuda")
    moe.moe_grouped_ffn_bwd(s, dev_bf16(dy_bits), d_xp, d_off, d_wg, d_wu, d_wd, sg, su, dxp, gwg, gwu, gwd, 0, ws)
    dX, dWg, dWu, dWd = O.grouped_ffn_bwd(dyp, xp, offsets, wg, wu, wd)
    qX, qWg, qWu, qWd = O.grouped_ffn_bwd_scales(dyp, xp, offsets, wg, wu, wd)
    assert_close(host_f32(dxp), dX, qX, what="dx_perm")
    assert_close(gwg.cpu().numpy(), dWg, qWg, what="dw_gate")
    assert_close(gwu.cpu().numpy(), dWu, qWu, what="dw_up")
    assert_close(gwd.cpu().numpy(), dWd, qWd, what="dw_down")
    empty = int(np.nonzero(counts == 0)[0][0])
    assert not gwg[empty].any() and not gwd[empty].any()    # the empty expert


# ---------------------------------------------------------------------------------------------------------
# the whole layer, forward + backward, against the per-token definition
# ---------------------------------------------------------------------------------------------------------

def run_layer(moe, inp, renorm=1):
    sh = inp["shape"]
    s = moe.Shape(sh.T, sh.d_model, sh.d_ffn, sh.E, sh.k, sh.E_shared, renorm)
    buf = moe.MoeLayerBuffers(s)
    x, dout = dev_bf16(inp["x"]), dev_bf16(inp["dout"])
    wg, wu, wd = dev_bf16(inp["w_gate"]), dev_bf16(inp["w_up"]), dev_bf16(inp["w_down"])
    if "logits" in inp:
        logits = dev(inp["logits"])
    else:
        logits = None
        buf.topk_idx.copy_(dev(inp["topk_idx"]))
        buf.topk_w.copy_(dev(inp["topk_w"]))
    moe.layer_forward(buf, x, wg, wu, wd, logits)
    moe.layer_backward(buf, dout, wg, wu, wd, accumulate=False, with_router=logits is not None)
    torch.cuda.synchronize()
    return s, buf


def check_layer_against_definition(moe, inp, renorm=1):
    sh = inp["shape"]
    s, buf = run_layer(moe, inp, renorm)
    if "logits" in inp:
        idx, w, probs = O.route_topk(inp["logits"], sh.k, sh.E_shared, bool(renorm))
        assert np.array_equal(buf.topk_idx.cpu().numpy(), idx)
        np.testing.assert_allclose(buf.topk_w.cpu().numpy(), w, rtol=TOL_GATE)
    else:
        idx, w, probs = inp["topk_idx"], inp["topk_w"].astype(np.float64), None
    counts, offsets, ros, sor = O.permute_maps(idx, sh.E_total)
    assert np.array_equal(buf.counts.cpu().numpy(), counts)
    assert np.array_equal(buf.offsets.cpu().numpy(), offsets)
    assert np.array_equal(buf.row_of_slot.cpu().numpy(), ros)
    assert np.array_equal(buf.slot_of_row.cpu().numpy(), sor)
    assert np.array_equal(host_bits(buf.x_perm), O.permute_rows(inp["x"], sor, sh.K_slots))
    x, dout = f32w(inp, "x"), f32w(inp, "dout")
    wg, wu, wd = f32w(inp, "w_gate"), f32w(inp, "w_up"), f32w(inp, "w_down")
    out, _ = O.layer_forward(x, idx, w, wg, wu, wd)
    q = O.layer_scales(x, idx, w, wg, wu, wd, dout, sh.E_total)
    assert_close(host_f32(buf.out), out, q["out"], what="out")
    g = O.layer_backward(x, idx, w, wg, wu, wd, dout)
    assert_close(host_f32(buf.dx), g["dx"], q["dx"], what="dx")
    assert_close(buf.dtopk_w.cpu().numpy(), g["dtopk_w"], q["dtopk_w"], what="dtopk_w")
    assert_close(buf.dw_gate.cpu().numpy(), g["dw_gate"], q["dw_gate"], what="dw_gate")
    assert_close(buf.dw_up.cpu().numpy(), g["dw_up"], q["dw_up"], what="dw_up")
    assert_close(buf.dw_down.cpu().numpy(), g["dw_down"], q["dw_down"], what="dw_down")
    if probs is not None:
        dl = O.route_topk_bwd(g["dtopk_w"], idx, w, probs, sh.k, bool(renorm))
        # dlogits is linear in dtopk_w with coefficients <= 1: held to the largest dtopk_w scale of its token
        q_dl = np.broadcast_to(q["dtopk_w"].max(axis=1, keepdims=True), dl.shape)
        assert_close(buf.dlogits.cpu().numpy(), dl, q_dl, what="dlogits")
    return counts


@pytest.mark.parametrize("renorm", [1, 0])
def test_layer_tiny_workload(moe, renorm):
    inp = W.make_layer_inputs(W.WORKLOADS["tiny"], seed=0)
    check_layer_against_definition(moe, inp, renorm)


@pytest.mark.parametrize("name", ["mixtral", "finegrained", "shard", "imbalance"])
def test_layer_scaled_down_workloads(moe, name):
    """Same E, k, shared experts and routing recipe as the full workload; d, f / 8 and T / 4 so that the full
    fp64 oracle finishes in seconds."""
    w = W.scaled_down(W.WORKLOADS[name])
    inp = W.make_layer_inputs(w, seed=0)
    counts = check_layer_against_definition(moe, inp)
    if name == "imbalance":
        assert (counts == 0).sum() >= 20 and counts.max() > 4 * counts[counts > 0].mean()
    if name == "shard":
        assert counts.min() < 16


def test_dense_reduction_on_gpu(moe):
    """E = 1, k = 1: the layer is a dense SwiGLU FFN with gate weight 1."""
    sh = W.MoEShape(200, 128, 192, 1, 1)
    inp = W.random_layer_inputs(sh, seed=3)
    check_layer_against_definition(moe, inp)


def test_recomputing_backward_is_bit_identical(moe):
    """Checkpointed forward (G, U not kept) + recomputing backward: bit for bit the saving pair's outputs (same
    kernels on the same inputs), and within the bound of the oracle's grouped FFN like the saving pair."""
    wl = W.scaled_down(W.WORKLOADS["finegrained"])
    sh = wl.shape
    inp = W.make_layer_inputs(wl, seed=5)
    s = moe.Shape.of(sh)
    idx, w, _ = O.route_topk(inp["logits"], sh.k, sh.E_shared, True)
    counts, offsets, ros, sor = O.permute_maps(idx, sh.E_total)
    x_perm = dev_bf16(O.permute_rows(inp["x"], sor, sh.K_slots))
    dy = dev_bf16(W.f32_to_bf16_bits(np.random.default_rng(9).standard_normal((sh.N, sh.d_model)).astype(np.float32)))
    wg, wu, wd = dev_bf16(inp["w_gate"]), dev_bf16(inp["w_up"]), dev_bf16(inp["w_down"])
    off = dev(offsets.astype(np.int32))
    ws = ws_for(moe, s)
    e = lambda *sz, dtype=torch.bfloat16: torch.empty(*sz, dtype=dtype, device="cuda")  # noqa: E731
    y1, y2, sg, su = e(sh.N, sh.d_model), e(sh.N, sh.d_model), e(sh.N, sh.d_ffn), e(sh.N, sh.d_ffn)
    moe.moe_grouped_ffn_fwd(s, x_perm, off, wg, wu, wd, y1, sg, su, ws)
    moe.moe_grouped_ffn_fwd(s, x_perm, off, wg, wu, wd, y2, None, None, ws)
    assert torch.equal(y1.view(torch.int16), y2.view(torch.int16))
    outs = []
    for mode in ("saved", "recompute"):
        dx = e(sh.N, sh.d_model)
        dws = [e(sh.E_total, sh.d_model, sh.d_ffn, dtype=torch.float32), e(sh.E_total, sh.d_model, sh.d_ffn, dtype=torch.float32),
               e(sh.E_total, sh.d_ffn, sh.d_model, dtype=torch.float32)]
        if mode == "saved":
            moe.moe_grouped_ffn_bwd(s, dy, x_perm, off, wg, wu, wd, sg, su, dx, dws[0], dws[1], dws[2], 0, ws)
        else:
            moe.moe_grouped_ffn_bwd_recompute(s, dy, x_perm, off, wg, wu, wd, dx, dws[0], dws[1], dws[2], 0, ws)
        outs.append([dx.view(torch.int16)] + [t.view(torch.int32) for t in dws])
    for a, b in zip(*outs):
        assert torch.equal(a, b)
    # ... and the recomputing call is held to the oracle directly
    wgf, wuf, wdf = f32w(inp, "w_gate"), f32w(inp, "w_up"), f32w(inp, "w_down")
    xpf, dyf = host_f32(x_perm), host_f32(dy)
    dX, dWg, dWu, dWd = O.grouped_ffn_bwd(dyf, xpf, offsets, wgf, wuf, wdf)
    qX, qWg, qWu, qWd = O.grouped_ffn_bwd_scales(dyf, xpf, offsets, wgf, wuf, wdf)
    assert_close(host_f32(dx), dX, qX, what="recompute dx_perm")
    assert_close(dws[0].cpu().numpy(), dWg, qWg, what="recompute dw_gate")
    assert_close(dws[1].cpu().numpy(), dWu, qWu, what="recompute dw_up")
    assert_close(dws[2].cpu().numpy(), dWd, qWd, what="recompute dw_down")
    Y, _, _ = O.grouped_ffn_fwd(xpf, offsets, wgf, wuf, wdf)
    assert_close(host_f32(y2), Y, O.grouped_ffn_fwd_scales(xpf, offsets, wgf, wuf, wdf)[0], what="checkpointed forward y_perm")


def test_grouped_ffn_with_no_rows(moe):
    """T = 0: nothing to compute, but overwritten weight gradients must be exact zeros and accumulated ones untouched."""
    shape = W.MoEShape(0, 128, 64, 4, 2)
    s = moe.Shape.of(shape)
    ws = ws_for(moe, s)
    off = torch.zeros(5, dtype=torch.int32, device="cuda")
    z = torch.zeros((16,), dtype=torch.bfloat16, device="cuda")
    wts = [torch.randn(4, 128, 64, device="cuda").to(torch.bfloat16), torch.randn(4, 128, 64, device="cuda").to(torch.bfloat16),
           torch.randn(4, 64, 128, device="cuda").to(torch.bfloat16)]
    dws = [torch.full((4, 128, 64), 3.0, device="cuda"), torch.full((4, 128, 64), 3.0, device="cuda"), torch.full((4, 64, 128), 3.0, device="cuda")]
    moe.moe_grouped_ffn_fwd(s, z, off, wts[0], wts[1], wts[2], z, z, z, ws)
    moe.moe_grouped_ffn_bwd(s, z, z, off, wts[0], wts[1], wts[2], z, z, z, dws[0], dws[1], dws[2], 1, ws)
    assert all(bool((t == 3.0).all()) for t in dws)
    moe.moe_grouped_ffn_bwd(s, z, z, off, wts[0], wts[1], wts[2], z, z, z, dws[0], dws[1], dws[2], 0, ws)
    assert all(not bool(t.any()) for t in dws)
