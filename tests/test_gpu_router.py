"""Parity of the router's linear map (logits = x W_r^T), its backward, and the layer closed from x, against the CPU
fp64 oracle, through the C ABI.

Bar: the logits and both router gradients are bf16 x bf16 products accumulated in fp32 (the upstream dlogits enters
as a bf16 head plus a bf16 remainder), so they are held to 2e-3 in the two-part criterion of test_gpu_parity.py
(per tensor relative to the largest reference value, per element relative to |ref| + quadrature magnitude); the
bf16 output dx and everything downstream of the expert path keep the 2e-2 bar.  The top-k choice is discrete: the
closed-layer test checks that the GPU's choice is a valid top-k of the reference logits within the logits' own error
and identical to the oracle's wherever the choice is forced, then evaluates the oracle for that choice.
"""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import moe_oracle as O
from test_gpu_parity import TOL, TOL_GATE, assert_close, dev, dev_bf16, f32w, host_f32, ws_for

pytestmark = pytest.mark.gpu

TOL_ROUTER = 2e-3


def router_case(T, d, E, seed):
    sh = W.MoEShape(T=T, d_model=d, d_ffn=64, E=E, k=1)
    xb = W.make_tokens(sh, seed)
    wrb = W.make_router_weight(sh, seed, std=0.05)
    dl = (np.random.default_rng([seed, 21]).standard_normal((T, E)) * 0.3).astype(np.float32)
    return sh, xb, wrb, dl


ROUTER_SHAPES = [
    # T, d, E: one tile, ragged token tail, E not a multiple of 4 / of 8, E over 128 (dx on the grouped GEMM kernel), many tiles
    (256, 512, 8), (777, 256, 60), (300, 128, 7), (1000, 192, 300), (4096, 1024, 128), (64, 64, 1), (2500, 2048, 16),
    # every expert-group count of the skinny dx kernel (32, 64, 128 padded experts) with ragged E, more columns than one
    # block's 1024, fewer tokens than one stage of 64
    (500, 320, 96), (130, 1280, 33), (40, 2112, 32),
    # the forward kernel for many experts and many tokens (both operands through LDS): 64- and 128-expert tiles, ragged
    # E (also not a multiple of 4), a ragged token tail, two expert tiles
    (8192, 256, 60), (8200, 128, 99), (8192, 192, 160),
    # the router of the two workloads bench.py times it on, at full size
    (4096, 4096, 8), (16384, 4096, 128),
]


@pytest.mark.parametrize("T,d,E", ROUTER_SHAPES)
def test_router_forward_and_backward(moe, T, d, E):
    sh, xb, wrb, dl = router_case(T, d, E, seed=T + E)
    s = moe.Shape.of(sh)
    ws = ws_for(moe, s)
    x, wr = dev_bf16(xb), dev_bf16(wrb)
    logits = torch.full((T, E), float("nan"), dtype=torch.float32, device="cuda")
    moe.moe_router_fwd(s, x, wr, logits, ws)
    xf, wf = W.bf16_bits_to_f32(xb), W.bf16_bits_to_f32(wrb)
    ref = O.router_logits(xf, wf)
    q_l, q_x, q_w = O.router_scales(xf, wf, dl)
    assert_close(logits.cpu().numpy(), ref, q_l, tol=TOL_ROUTER, what="logits")

    dxr = torch.full((T, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    dwr = torch.full((E, d), float("nan"), dtype=torch.float32, device="cuda")
    moe.moe_router_bwd(s, x, wr, dev(dl), dxr, dwr, 0, ws)
    rdx, rdw = O.router_logits_bwd(xf, wf, dl)
    assert_close(host_f32(dxr), rdx, q_x, tol=TOL, what="dx_router")          # bf16 output
    assert_close(dwr.cpu().numpy(), rdw, q_w, tol=TOL_ROUTER, what="dw_router")
    # accumulate: a second call with half the upstream gradient adds half of the first result
    moe.moe_router_bwd(s, x, wr, dev(dl * np.float32(0.5)), dxr, dwr, 1, ws)
    assert_close(dwr.cpu().numpy(), 1.5 * rdw, 1.5 * q_w, tol=TOL_ROUTER, what="dw_router accumulated")
    assert_close(host_f32(dxr), 0.5 * rdx, 0.5 * q_x, tol=TOL, what="dx_router (never accumulated)")


def test_permute_bwd_add(moe):
    sh = W.MoEShape(T=300, d_model=256, d_ffn=64, E=8, k=3)
    inp = W.random_layer_inputs(sh, seed=3)
    s = moe.Shape.of(sh)
    idx, _, _ = O.route_topk(inp["logits"], sh.k, 0, True)
    _, _, ros, _ = O.permute_maps(idx, sh.E_total)
    rng = np.random.default_rng(8)
    dxp = W.f32_to_bf16_bits(rng.standard_normal((sh.N, sh.d_model)).astype(np.float32))
    add = W.f32_to_bf16_bits(rng.standard_normal((sh.T, sh.d_model)).astype(np.float32))
    dx = torch.empty(sh.T, sh.d_model, dtype=torch.bfloat16, device="cuda")
    moe.moe_permute_bwd_add(s, dev_bf16(dxp), dev(ros), dev_bf16(add), dx)
    ref = O.permute_bwd(W.bf16_bits_to_f32(dxp), ros, sh.K_slots) + W.bf16_bits_to_f32(add)
    # fp32 sum of K'+1 bf16 values, one bf16 rounding: half an ulp of the result plus the fp32 sum's own rounding
    assert np.all(np.abs(host_f32(dx) - ref) <= np.abs(ref) * 2.0 ** -8 + 1e-6)


@pytest.mark.parametrize("name", ["tiny", "finegrained", "imbalance"])
def test_closed_layer(moe, name):
    wl = W.WORKLOADS[name]
    wl = wl if name == "tiny" else W.scaled_down(wl)
    sh = wl.shape
    inp = W.make_layer_inputs(wl, seed=2)
    wrb = W.make_router_weight(sh, seed=2, std=0.05)
    s = moe.Shape.of(sh)
    buf = moe.MoeLayerBuffers(s)
    x, dout, wr = dev_bf16(inp["x"]), dev_bf16(inp["dout"]), dev_bf16(wrb)
    wg, wu, wd = dev_bf16(inp["w_gate"]), dev_bf16(inp["w_up"]), dev_bf16(inp["w_down"])
    moe.layer_forward(buf, x, wg, wu, wd, w_router=wr)
    moe.layer_backward(buf, dout, wg, wu, wd, x=x, w_router=wr)
    torch.cuda.synchronize()

    xf, wf, df = f32w(inp, "x"), W.bf16_bits_to_f32(wrb), f32w(inp, "dout")
    Wg, Wu, Wd = f32w(inp, "w_gate"), f32w(inp, "w_up"), f32w(inp, "w_down")
    lg64 = O.router_logits(xf, wf)
    q_l = O.router_scales(xf, wf, np.zeros_like(lg64))[0]
    assert_close(buf.logits.cpu().numpy(), lg64, q_l, tol=TOL_ROUTER, what="logits")
    # The top-k choice is piecewise constant in the logits, and the GPU takes it from its own fp32 logits.  Where
    # the k-th and (k+1)-th reference logits are closer than the logits' error, two choices are equally right; the
    # GPU's is checked to be a valid one (no unselected reference logit beats a selected one by more than the error
    # of the row's logits, listed by descending logit within that error), and everything continuous is then
    # evaluated by the oracle for THAT choice, for every token, with no condition on the checks that follow.
    got_lg = buf.logits.cpu().numpy().astype(np.float64)
    row_err = np.abs(got_lg - lg64).max(axis=1) + np.abs(lg64).max(axis=1) * 2.0 ** -23
    got_idx = buf.topk_idx.cpu().numpy()
    sel = got_idx[:, :sh.k].astype(np.int64)
    assert ((sel >= 0) & (sel < sh.E)).all()
    assert all(len(set(r)) == sh.k for r in sel.tolist())                      # distinct experts per token
    sel_lg = np.take_along_axis(lg64, sel, axis=1)
    unsel = lg64.copy()
    np.put_along_axis(unsel, sel, -np.inf, axis=1)
    assert (sel_lg.min(axis=1) >= unsel.max(axis=1) - 2 * row_err).all()       # a valid top-k of the reference logits
    assert (sel_lg[:, :-1] >= sel_lg[:, 1:] - 2 * row_err[:, None]).all()      # in descending order
    for j in range(sh.E_shared):
        assert (got_idx[:, sh.k + j] == sh.E + j).all()
    # most tokens are decided outright, and there the choice is the oracle's own
    ref_idx, _, _ = O.route_topk(lg64.astype(np.float32), sh.k, sh.E_shared, True)
    srt = np.sort(lg64, axis=1)[:, ::-1]
    margin = srt[:, sh.k - 1] - srt[:, sh.k] if sh.E > sh.k else np.full(sh.T, np.inf)
    decided = margin > 4 * row_err
    assert decided.mean() > 0.98
    assert all(set(got_idx[t, :sh.k]) == set(ref_idx[t, :sh.k]) for t in np.nonzero(decided)[0])
    cache = O.gate_of_selection(lg64, sel, sh.E_shared, True)
    assert np.array_equal(cache[0], got_idx)
    out_ref, _ = O.layer_forward(xf, cache[0], cache[1], Wg, Wu, Wd)

    g = O.closed_layer_backward(xf, wf, sh.k, Wg, Wu, Wd, df, cache, True)
    q = O.layer_scales_staged(xf, cache[0], cache[1], Wg, Wu, Wd, df, sh.E_total)
    _, q_xr, q_wr = O.router_scales(xf, wf, g["dlogits"])
    # a logit error e moves a gate weight by at most 2e of itself; the gate's own fp32 arithmetic adds 1e-5
    assert (np.abs(buf.topk_w.cpu().numpy() - cache[1]) <= (4 * row_err[:, None] + TOL_GATE) * cache[1]).all()
    assert_close(host_f32(buf.out), out_ref, q["out"], what="out")
    dl_scale = np.abs(g["dtopk_w"]).max()
    assert np.abs(buf.dlogits.cpu().numpy() - g["dlogits"]).max() <= TOL * dl_scale   # inherits dtopk_w's bf16 inputs
    assert_close(buf.dw_router.cpu().numpy(), g["dw_router"], q_wr + TOL * np.abs(g["dw_router"]).max(), tol=TOL, what="dw_router")
    assert_close(host_f32(buf.dx), g["dx_total"], np.sqrt(q["dx"] ** 2 + q_xr ** 2), what="dx (expert path + router)")
    assert_close(buf.dw_gate.cpu().numpy(), g["dw_gate"], q["dw_gate"], what="dw_gate")
    assert_close(buf.dw_up.cpu().numpy(), g["dw_up"], q["dw_up"], what="dw_up")
    assert_close(buf.dw_down.cpu().numpy(), g["dw_down"], q["dw_down"], what="dw_down")
