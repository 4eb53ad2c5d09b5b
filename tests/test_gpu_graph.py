"""A whole layer step (forward + backward, ragged counts read on the device) captured into a HIP graph: every replay,
with new inputs written into the graph's static tensors and eager work and synchronisations in between, must give
bit for bit what the eager call order gives on the same inputs (same kernels, same launch shapes, fixed reduction
orders), and the eager result itself is held to the oracle by the parity tests."""
import numpy as np
import pytest
import torch

import workloads as W
from test_gpu_parity import dev, dev_bf16

pytestmark = pytest.mark.gpu

CASES = [
    ("tiny", W.WORKLOADS["tiny"]),
    ("imbalance_scaled", W.scaled_down(W.WORKLOADS["imbalance"])),      # empty experts, ragged tiles, split tails
    ("finegrained_scaled", W.scaled_down(W.WORKLOADS["finegrained"])),  # shared experts
]


def _tensors(buf, with_router):
    names = ["topk_idx", "topk_w", "counts", "offsets", "row_of_slot", "slot_of_row", "x_perm", "y_perm", "out",
             "dy_perm", "dtopk_w", "dx_perm", "dx", "dw_gate", "dw_up", "dw_down"]
    if with_router:
        names += ["probs", "dlogits"]
    return {n: getattr(buf, n) for n in names}


@pytest.mark.parametrize("name,wl", CASES, ids=[c[0] for c in CASES])
def test_graph_replays_match_eager(moe, name, wl):
    sh = wl.shape
    s = moe.Shape.of(sh)
    inp = W.make_layer_inputs(wl, seed=0)
    if "logits" not in inp:
        pytest.skip("workload without router logits")
    x, dout, logits = dev_bf16(inp["x"]), dev_bf16(inp["dout"]), dev(inp["logits"])
    wg, wu, wd = dev_bf16(inp["w_gate"]), dev_bf16(inp["w_up"]), dev_bf16(inp["w_down"])
    buf_graph, buf_eager = moe.MoeLayerBuffers(s), moe.MoeLayerBuffers(s)
    step = moe.CapturedLayerStep(buf_graph, x, dout, wg, wu, wd, logits=logits)
    for replay in range(3):
        print(f"[graph] {name}: replay {replay}", flush=True)
        other = W.make_layer_inputs(wl, seed=10 + replay)      # new inputs, and with them another routing
        x.copy_(dev_bf16(other["x"])); dout.copy_(dev_bf16(other["dout"])); logits.copy_(dev(other["logits"]))
        step.replay()
        torch.cuda.synchronize()
        moe.layer_forward(buf_eager, x, wg, wu, wd, logits)
        moe.layer_backward(buf_eager, dout, wg, wu, wd)
        torch.cuda.synchronize()
        got, ref = _tensors(buf_graph, True), _tensors(buf_eager, True)
        for n in got:
            a, b = got[n], ref[n]
            if a.dtype == torch.bfloat16:
                a, b = a.view(torch.int16), b.view(torch.int16)
            assert torch.equal(a, b), f"{name}: replay {replay}: {n} differs from the eager result"
        assert int(buf_graph.counts.sum()) == s.N
