"""Parity at the full workload sizes, in the launch configuration bench.py times (MoeLayerBuffers + layer_forward /
layer_backward), against the fp64 oracle's slice mode:

  * every integer artefact in full (indices, counts, offsets, both maps) and the permuted rows, bit-exact;
  * out, dx, dtopk_w for 48 seeded-random tokens plus tokens of the smallest and the largest non-empty expert;
  * dW_gate, dW_up on 16 seeded f-columns and dW_down on the same 16 f-rows, for EVERY expert (empty ones included);
  * dlogits in full, from the GPU's own dtopk_w (the gate backward is a separate entry point).

Bar as in test_gpu_parity.py: per tensor max|got-ref|/max|ref| <= 2e-2 and per element |got-ref| <= 2e-2(|ref| + q).
"""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import moe_oracle as O
from test_gpu_parity import TOL, TOL_GATE, assert_close, dev, dev_bf16, f32w, host_bits, host_f32

pytestmark = pytest.mark.gpu


def pick_tokens(idx, counts, T, seed, n_random=48, n_per_extreme=8):
    rng = np.random.default_rng(seed)
    toks = set(rng.choice(T, size=min(n_random, T), replace=False).tolist())
    live = np.nonzero(counts > 0)[0]
    small, large = live[np.argmin(counts[live])], live[np.argmax(counts[live])]
    for e in (small, large):
        t_of_e = np.nonzero((idx == e).any(axis=1))[0]
        toks.update(t_of_e[:n_per_extreme].tolist())
    return np.array(sorted(toks), dtype=np.int64), int(small), int(large)


@pytest.mark.parametrize("name", ["mixtral", "finegrained", "shard", "imbalance"])
def test_full_size_workload(moe, name):
    wl = W.WORKLOADS[name]
    sh = wl.shape
    print(f"[fullsize] {name}: generating inputs", flush=True)
    inp = W.make_layer_inputs(wl, seed=0)
    s = moe.Shape.of(sh)
    buf = moe.MoeLayerBuffers(s)
    x, dout = dev_bf16(inp["x"]), dev_bf16(inp["dout"])
    wg, wu, wd = dev_bf16(inp["w_gate"]), dev_bf16(inp["w_up"]), dev_bf16(inp["w_down"])
    if "logits" in inp:
        logits = dev(inp["logits"])
    else:
        logits = None
        buf.topk_idx.copy_(dev(inp["topk_idx"]))
        buf.topk_w.copy_(dev(inp["topk_w"]))
    print(f"[fullsize] {name}: running fwd+bwd on the GPU", flush=True)
    moe.layer_forward(buf, x, wg, wu, wd, logits)
    moe.layer_backward(buf, dout, wg, wu, wd, accumulate=False, with_router=logits is not None)
    torch.cuda.synchronize()

    # ---- integer artefacts, in full
    if logits is not None:
        idx, w, probs = O.route_topk(inp["logits"], sh.k, sh.E_shared, True)
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
    assert counts.sum() == sh.N
    if name == "imbalance":
        assert (counts == 0).sum() == 26 and 0.58 <= counts[inp["roles"] == 2].sum() / sh.N <= 0.62
    if name == "shard":
        assert counts.min() < 40 and counts.max() > 900

    # ---- sampled tokens: out, dx, dtopk_w
    toks, e_small, e_large = pick_tokens(idx, counts, sh.T, seed=1)
    print(f"[fullsize] {name}: oracle on {toks.size} tokens (smallest expert {e_small}: {counts[e_small]} rows, "
          f"largest {e_large}: {counts[e_large]} rows)", flush=True)
    xf, df = f32w(inp, "x"), f32w(inp, "dout")
    Wg, Wu, Wd = inp["w_gate"], inp["w_up"], inp["w_down"]

    class LazyF32:           # widen one expert at a time: the oracle indexes [e] and converts to fp64 itself
        def __init__(self, bits):
            self.bits = bits
            self.shape = bits.shape

        def __getitem__(self, e):
            return W.bf16_bits_to_f32(self.bits[e])

        def __array__(self, dtype=None, copy=None):   # np.asarray(w).shape is all the oracle asks of the whole tensor
            return np.broadcast_to(np.float32(0), self.shape)

    lg, lu, ld = LazyF32(Wg), LazyF32(Wu), LazyF32(Wd)
    out_ref, _ = O.layer_forward(xf, idx, w, lg, lu, ld, tokens=toks)
    g = O.layer_backward(xf, idx, w, lg, lu, ld, df, tokens=toks, f_cols=[])
    q = O.layer_scales(xf, idx, w, lg, lu, ld, df, sh.E_total, tokens=toks, f_cols=[])
    tt = torch.from_numpy(toks).cuda()
    assert_close(host_f32(buf.out[tt]), out_ref, q["out"], what="out[sample]")
    assert_close(host_f32(buf.dx[tt]), g["dx"], q["dx"], what="dx[sample]")
    assert_close(buf.dtopk_w[tt].cpu().numpy(), g["dtopk_w"], q["dtopk_w"], what="dtopk_w[sample]")

    # ---- weight gradients on 16 f-columns / f-rows, every expert
    cols = np.sort(np.random.default_rng(2).choice(sh.d_ffn, size=16, replace=False))
    print(f"[fullsize] {name}: oracle weight gradients on f-indices {cols.tolist()}", flush=True)
    gw = O.layer_backward(xf, idx, w, lg, lu, ld, df, tokens=[], f_cols=cols)
    qw = O.layer_scales(xf, idx, w, lg, lu, ld, df, sh.E_total, tokens=[], f_cols=cols)
    ct = torch.from_numpy(cols).cuda()
    assert_close(buf.dw_gate[:, :, ct].cpu().numpy(), gw["dw_gate"], qw["dw_gate"], what="dw_gate[:, :, cols]")
    assert_close(buf.dw_up[:, :, ct].cpu().numpy(), gw["dw_up"], qw["dw_up"], what="dw_up[:, :, cols]")
    assert_close(buf.dw_down[:, ct, :].cpu().numpy(), gw["dw_down"], qw["dw_down"], what="dw_down[:, cols, :]")
    for e in np.nonzero(counts == 0)[0][:4]:          # empty experts: exact zeros over the whole slab
        assert not buf.dw_gate[int(e)].any() and not buf.dw_down[int(e)].any()

    # ---- gate backward, in full, from the GPU's own dtopk_w
    if probs is not None:
        dtw = buf.dtopk_w.cpu().numpy()
        dl = O.route_topk_bwd(dtw, idx, buf.topk_w.cpu().numpy(), buf.probs.cpu().numpy(), sh.k, True)
        scale = np.abs(dtw).max()
        assert np.abs(buf.dlogits.cpu().numpy() - dl).max() <= TOL_GATE * scale
    del buf, wg, wu, wd
    torch.cuda.empty_cache()
