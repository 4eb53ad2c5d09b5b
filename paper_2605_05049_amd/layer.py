"""Buffer set and call order of one MoE expert layer step.  Torch is used for device memory only: every
computation is one of the C-ABI entry points, called in the order of the per-layer flow (routing -> pack ->
experts -> unpack/combine, then the reverse for backward)."""
from __future__ import annotations

from . import binding as B


class MoeLayerBuffers:
    """All device buffers one forward+backward of a layer touches, allocated once."""

    def __init__(self, shape, device="cuda", with_backward=True, with_router=True):
        import torch
        s = B.Shape.of(shape)
        self.shape = s
        dev = torch.device(device)
        bf, i32, f32 = torch.bfloat16, torch.int32, torch.float32
        N, T, d, f, Et, Kp = s.N, s.T, s.d_model, s.d_ffn, s.E_total, s.K_slots
        e = lambda *sz, dtype: torch.empty(*sz, dtype=dtype, device=dev)  # noqa: E731
        self.topk_idx = e(T, Kp, dtype=i32)
        self.topk_w = e(T, Kp, dtype=f32)
        self.probs = e(T, s.E, dtype=f32) if with_router else None
        self.counts = e(Et, dtype=i32)
        self.offsets = e(Et + 1, dtype=i32)
        self.row_of_slot = e(N, dtype=i32)
        self.slot_of_row = e(N, dtype=i32)
        self.x_perm = e(N, d, dtype=bf)
        self.save_g = e(N, f, dtype=bf)
        self.save_u = e(N, f, dtype=bf)
        self.y_perm = e(N, d, dtype=bf)
        self.out = e(T, d, dtype=bf)
        self.ws = torch.empty(max(B.workspace_bytes(s), 256), dtype=torch.uint8, device=dev)
        if with_backward:
            self.dy_perm = e(N, d, dtype=bf)
            self.dtopk_w = e(T, Kp, dtype=f32)
            self.dx_perm = e(N, d, dtype=bf)
            self.dx = e(T, d, dtype=bf)
            self.dw_gate = e(Et, d, f, dtype=f32)
            self.dw_up = e(Et, d, f, dtype=f32)
            self.dw_down = e(Et, f, d, dtype=f32)
            self.dlogits = e(T, s.E, dtype=f32) if with_router else None
        # the layer closed from x (router weight given): logits, the router's term of dx, the router weight gradient
        self.logits = e(T, s.E, dtype=f32) if with_router else None
        if with_backward and with_router:
            self.dx_router = e(T, d, dtype=bf)
            self.dw_router = e(s.E, d, dtype=f32)


def layer_forward(buf: MoeLayerBuffers, x, w_gate, w_up, w_down, logits=None, w_router=None, stream=None):
    """routing (skipped when logits is None: buf.topk_idx / buf.topk_w were filled by the caller, as for an
    expert-parallel shard) -> permute -> grouped FFN -> combine.  With `w_router` the logits are computed first
    (buf.logits = x W_r^T).  Returns buf.out."""
    s = buf.shape
    if w_router is not None:
        B.moe_router_fwd(s, x, w_router, buf.logits, buf.ws, stream)
        logits = buf.logits
    if logits is not None:
        B.moe_route_topk(s, logits, buf.topk_idx, buf.topk_w, buf.probs, stream)
    B.moe_permute(s, x, buf.topk_idx, buf.x_perm, buf.counts, buf.offsets, buf.row_of_slot, buf.slot_of_row, buf.ws, stream)
    B.moe_grouped_ffn_fwd(s, buf.x_perm, buf.offsets, w_gate, w_up, w_down, buf.y_perm, buf.save_g, buf.save_u, buf.ws, stream)
    B.moe_unpermute_combine(s, buf.y_perm, buf.row_of_slot, buf.topk_w, buf.out, stream)
    return buf.out


def layer_backward(buf: MoeLayerBuffers, dout, w_gate, w_up, w_down, accumulate=False, with_router=True, x=None,
                   w_router=None, stream=None):
    """combine_bwd -> grouped FFN bwd -> permute_bwd -> route_bwd.  Results land in buf.dx, buf.dw_*, buf.dtopk_w,
    buf.dlogits.  With `x` and `w_router` the layer is closed from x: route_bwd -> router_bwd come before the
    un-permutation, buf.dx then holds the expert-path term plus the router's term, and buf.dw_router is filled."""
    s = buf.shape
    if w_router is not None:
        B.moe_unpermute_combine_bwd(s, dout, buf.y_perm, buf.row_of_slot, buf.topk_w, buf.dy_perm, buf.dtopk_w, stream)
        B.moe_grouped_ffn_bwd(s, buf.dy_perm, buf.x_perm, buf.offsets, w_gate, w_up, w_down, buf.save_g, buf.save_u,
                              buf.dx_perm, buf.dw_gate, buf.dw_up, buf.dw_down, accumulate, buf.ws, stream)
        B.moe_route_topk_bwd(s, buf.dtopk_w, buf.topk_idx, buf.topk_w, buf.probs, buf.dlogits, stream)
        B.moe_router_bwd(s, x, w_router, buf.dlogits, buf.dx_router, buf.dw_router, accumulate, buf.ws, stream)
        B.moe_permute_bwd_add(s, buf.dx_perm, buf.row_of_slot, buf.dx_router, buf.dx, stream)
        return
    B.moe_unpermute_combine_bwd(s, dout, buf.y_perm, buf.row_of_slot, buf.topk_w, buf.dy_perm, buf.dtopk_w, stream)
    B.moe_grouped_ffn_bwd(s, buf.dy_perm, buf.x_perm, buf.offsets, w_gate, w_up, w_down, buf.save_g, buf.save_u,
                          buf.dx_perm, buf.dw_gate, buf.dw_up, buf.dw_down, accumulate, buf.ws, stream)
    B.moe_permute_bwd(s, buf.dx_perm, buf.row_of_slot, buf.dx, stream)
    if with_router and buf.dlogits is not None:
        B.moe_route_topk_bwd(s, buf.dtopk_w, buf.topk_idx, buf.topk_w, buf.probs, buf.dlogits, stream)


class CapturedLayerStep:
    """One forward+backward of a layer recorded into a HIP graph and replayed with a single launch.

    Every node of the graph is one of the library's kernels: the entry points allocate nothing, never synchronise
    the host, take the ragged counts from device memory and clear their own counters with kernels (no memset
    nodes), so a whole step can be captured.  torch.cuda.CUDAGraph drives the capture.  The tensors passed in are the
    graph's static inputs: refill them in place (`x.copy_(...)`) and call `replay()`; results land in `buf` as
    after `layer_forward` + `layer_backward`."""

    def __init__(self, buf: MoeLayerBuffers, x, dout, w_gate, w_up, w_down, logits=None, w_router=None,
                 accumulate=False, with_router=True, warmup=2):
        import torch
        self.buf = buf
        self._args = (x, dout, w_gate, w_up, w_down, logits, w_router, accumulate, with_router)
        side = torch.cuda.Stream()  # default priority
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for _ in range(warmup):
                self._step()
        torch.cuda.current_stream().wait_stream(side)
        self.graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(self.graph):
            self._step()

    def _step(self):
        x, dout, w_gate, w_up, w_down, logits, w_router, accumulate, with_router = self._args
        layer_forward(self.buf, x, w_gate, w_up, w_down, logits=logits, w_router=w_router)
        layer_backward(self.buf, dout, w_gate, w_up, w_down, accumulate=accumulate, with_router=with_router,
                       x=x if w_router is not None else None, w_router=w_router)

    def replay(self):
        self.graph.replay()
