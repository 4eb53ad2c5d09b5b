"""ctypes binding of libmoe_gfx950.so.  Argument marshalling only; see include/moe.h for the semantics."""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, Structure, c_char_p, c_int, c_int32, c_size_t, c_void_p
from typing import Optional

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
_LIB_NAME = "libmoe_gfx950.so"
_lib = None

EXPORTED_SYMBOLS = (
    "moe_status_str", "moe_workspace_bytes", "moe_abi_version",
    "moe_profile_enable", "moe_profile_count", "moe_profile_get", "moe_profile_reset",
    "moe_route_topk", "moe_route_topk_bwd", "moe_permute", "moe_permute_noalloc", "moe_permute_bwd", "moe_permute_bwd_add",
    "moe_router_fwd", "moe_router_bwd", "moe_grouped_ffn_fwd", "moe_grouped_ffn_bwd", "moe_grouped_ffn_bwd_recompute",
    "moe_unpermute_combine", "moe_unpermute_combine_bwd",
    "moe_load_accumulate", "moe_load_imbalance", "moe_rebalance_experts",
    "moe_halo_pack_remote", "moe_halo_repack", "moe_halo_unpack",
)


class MoeError(RuntimeError):
    def __init__(self, fn: str, status: int):
        self.status = status
        super().__init__(f"{fn} failed: {status} ({status_str(status)})")


class _CShape(Structure):
    _fields_ = [("T", c_int32), ("d_model", c_int32), ("d_ffn", c_int32), ("E", c_int32), ("k", c_int32),
                ("E_shared", c_int32), ("renorm", c_int32)]


class Shape:
    """Problem statement of one layer: T tokens, d_model, d_ffn, E routed experts, top-k, E_shared, renorm."""

    def __init__(self, T, d_model, d_ffn, E, k, E_shared=0, renorm=1):
        self.T, self.d_model, self.d_ffn, self.E, self.k = int(T), int(d_model), int(d_ffn), int(E), int(k)
        self.E_shared, self.renorm = int(E_shared), int(renorm)
        self._c = _CShape(self.T, self.d_model, self.d_ffn, self.E, self.k, self.E_shared, self.renorm)

    @classmethod
    def of(cls, s) -> "Shape":
        """From any object with the same attribute names (e.g. a workloads.MoEShape)."""
        return s if isinstance(s, Shape) else cls(s.T, s.d_model, s.d_ffn, s.E, s.k, s.E_shared, s.renorm)

    E_total = property(lambda self: self.E + self.E_shared)
    K_slots = property(lambda self: self.k + self.E_shared)
    N = property(lambda self: self.T * (self.k + self.E_shared))


def library_path() -> str:
    """The in-tree library; MOE_LIBRARY_PATH overrides it (e.g. to try another build of the same ABI)."""
    return os.environ.get("MOE_LIBRARY_PATH") or os.path.join(PKG_DIR, _LIB_NAME)


def load_library():
    """Loads the shared library (once).  Raises if it has not been built: there is no fallback path."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                           "(or python paper_2605_05049_amd/build.py) first; there is no CPU fallback")
    lib = ctypes.CDLL(path)
    sp = POINTER(_CShape)
    lib.moe_status_str.restype = c_char_p
    lib.moe_status_str.argtypes = [c_int]
    lib.moe_workspace_bytes.restype = c_size_t
    lib.moe_workspace_bytes.argtypes = [sp]
    lib.moe_abi_version.restype = c_int
    lib.moe_abi_version.argtypes = []
    lib.moe_profile_enable.restype = c_int
    lib.moe_profile_enable.argtypes = [c_int]
    lib.moe_profile_count.restype = c_int
    lib.moe_profile_count.argtypes = []
    lib.moe_profile_get.restype = c_int
    lib.moe_profile_get.argtypes = [c_int, POINTER(c_char_p), POINTER(ctypes.c_float)]
    lib.moe_profile_reset.restype = c_int
    lib.moe_profile_reset.argtypes = []
    V = c_void_p
    sigs = {
        "moe_route_topk": [sp, V, V, V, V, V],
        "moe_route_topk_bwd": [sp, V, V, V, V, V, V],
        "moe_permute": [sp, V, V, V, V, V, V, V, V, c_size_t, V],
        "moe_permute_noalloc": [sp, V, V, V, V, V, V, V, V],
        "moe_permute_bwd": [sp, V, V, V, V],
        "moe_permute_bwd_add": [sp, V, V, V, V, V],
        "moe_router_fwd": [sp, V, V, V, V, c_size_t, V],
        "moe_router_bwd": [sp, V, V, V, V, V, c_int, V, c_size_t, V],
        "moe_grouped_ffn_fwd": [sp, V, V, V, V, V, V, V, V, V, c_size_t, V],
        "moe_grouped_ffn_bwd": [sp, V, V, V, V, V, V, V, V, V, V, V, V, c_int, V, c_size_t, V],
        "moe_grouped_ffn_bwd_recompute": [sp, V, V, V, V, V, V, V, V, V, V, c_int, V, c_size_t, V],
        "moe_unpermute_combine": [sp, V, V, V, V, V],
        "moe_unpermute_combine_bwd": [sp, V, V, V, V, V, V, V],
    }
    sigs["moe_halo_pack_remote"] = [V, V, c_int, c_int, c_size_t, c_int, V]
    sigs["moe_halo_repack"] = [V, V, c_int, c_int, c_size_t, V]
    sigs["moe_halo_unpack"] = [V, V, V, c_int, c_int, c_size_t, c_int, V]
    sigs["moe_load_accumulate"] = [V, V, c_int]
    sigs["moe_load_imbalance"] = [V, c_int, c_int, V, POINTER(ctypes.c_double)]
    sigs["moe_rebalance_experts"] = [V, c_int, c_int, V, c_int, POINTER(ctypes.c_int32), V]
    for name, args in sigs.items():
        fn = getattr(lib, name)
        fn.restype = c_int
        fn.argtypes = args
    _lib = lib
    return lib


def status_str(status: int) -> str:
    return load_library().moe_status_str(int(status)).decode()


def abi_version() -> int:
    return int(load_library().moe_abi_version())


def workspace_bytes(shape) -> int:
    return int(load_library().moe_workspace_bytes(ctypes.byref(Shape.of(shape)._c)))


def profile_enable(on: bool) -> None:
    _check("moe_profile_enable", load_library().moe_profile_enable(int(bool(on))))


def profile_reset() -> None:
    _check("moe_profile_reset", load_library().moe_profile_reset())


def profile_records():
    """[(label, milliseconds)] of every launch recorded since the last reset (synchronises on each)."""
    lib = load_library()
    out = []
    for i in range(lib.moe_profile_count()):
        name = c_char_p()
        ms = ctypes.c_float()
        _check("moe_profile_get", lib.moe_profile_get(i, ctypes.byref(name), ctypes.byref(ms)))
        out.append((name.value.decode(), float(ms.value)))
    return out


# ------------------------------------------------------------------------------------------------------------
# marshalling helpers
# ------------------------------------------------------------------------------------------------------------

def _ptr(t, dtype=None, numel: Optional[int] = None, name: str = "tensor"):
    """Device pointer of a contiguous CUDA(HIP) tensor, after checking dtype and element count."""
    if t is None:
        return None
    import torch
    if not t.is_cuda:
        raise ValueError(f"{name}: expected a device tensor")
    if not t.is_contiguous():
        raise ValueError(f"{name}: expected a contiguous tensor")
    if dtype is not None:
        ok = t.dtype in dtype if isinstance(dtype, (tuple, list)) else t.dtype == dtype
        if not ok:
            raise ValueError(f"{name}: dtype {t.dtype}, expected {dtype}")
    if numel is not None and t.numel() < numel:
        raise ValueError(f"{name}: {t.numel()} elements, need {numel}")
    return t.data_ptr()


def _stream(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return c_void_p(s.cuda_stream)


def _check(fn: str, rc: int):
    if rc != 0:
        raise MoeError(fn, rc)


def _bf16_types():
    import torch
    return (torch.bfloat16, torch.int16, torch.uint16)


# ------------------------------------------------------------------------------------------------------------
# entry points (same names and argument order as include/moe.h)
# ------------------------------------------------------------------------------------------------------------

def moe_route_topk(shape, logits, topk_idx, topk_w, probs_save=None, stream=None):
    import torch
    s = Shape.of(shape)
    rc = load_library().moe_route_topk(
        ctypes.byref(s._c), _ptr(logits, torch.float32, s.T * s.E, "logits"),
        _ptr(topk_idx, torch.int32, s.N, "topk_idx"), _ptr(topk_w, torch.float32, s.N, "topk_w"),
        _ptr(probs_save, torch.float32, s.T * s.E, "probs_save"), _stream(stream))
    _check("moe_route_topk", rc)


def moe_route_topk_bwd(shape, dtopk_w, topk_idx, topk_w, probs_save, dlogits, stream=None):
    import torch
    s = Shape.of(shape)
    rc = load_library().moe_route_topk_bwd(
        ctypes.byref(s._c), _ptr(dtopk_w, torch.float32, s.N, "dtopk_w"), _ptr(topk_idx, torch.int32, s.N, "topk_idx"),
        _ptr(topk_w, torch.float32, s.N, "topk_w"), _ptr(probs_save, torch.float32, s.T * s.E, "probs_save"),
        _ptr(dlogits, torch.float32, s.T * s.E, "dlogits"), _stream(stream))
    _check("moe_route_topk_bwd", rc)


def moe_permute(shape, x, topk_idx, x_perm, counts, offsets, row_of_slot, slot_of_row, ws, stream=None):
    import torch
    s = Shape.of(shape)
    bf = _bf16_types()
    rc = load_library().moe_permute(
        ctypes.byref(s._c), _ptr(x, bf, s.T * s.d_model, "x"), _ptr(topk_idx, torch.int32, s.N, "topk_idx"),
        _ptr(x_perm, bf, s.N * s.d_model, "x_perm"), _ptr(counts, torch.int32, s.E_total, "counts"),
        _ptr(offsets, torch.int32, s.E_total + 1, "offsets"), _ptr(row_of_slot, torch.int32, s.N, "row_of_slot"),
        _ptr(slot_of_row, torch.int32, s.N, "slot_of_row"), _ptr(ws, None, None, "ws"),
        ws.numel() * ws.element_size(), _stream(stream))
    _check("moe_permute", rc)


def moe_permute_noalloc(shape, x, topk_idx, x_perm, counts, offsets, row_of_slot, slot_of_row, stream=None):
    import torch
    s = Shape.of(shape)
    bf = _bf16_types()
    rc = load_library().moe_permute_noalloc(
        ctypes.byref(s._c), _ptr(x, bf, s.T * s.d_model, "x"), _ptr(topk_idx, torch.int32, s.N, "topk_idx"),
        _ptr(x_perm, bf, s.N * s.d_model, "x_perm"), _ptr(counts, torch.int32, s.E_total, "counts"),
        _ptr(offsets, torch.int32, s.E_total + 1, "offsets"), _ptr(row_of_slot, torch.int32, s.N, "row_of_slot"),
        _ptr(slot_of_row, torch.int32, s.N, "slot_of_row"), _stream(stream))
    _check("moe_permute_noalloc", rc)


def moe_permute_bwd(shape, dx_perm, row_of_slot, dx, stream=None):
    import torch
    s = Shape.of(shape)
    bf = _bf16_types()
    rc = load_library().moe_permute_bwd(
        ctypes.byref(s._c), _ptr(dx_perm, bf, s.N * s.d_model, "dx_perm"),
        _ptr(row_of_slot, torch.int32, s.N, "row_of_slot"), _ptr(dx, bf, s.T * s.d_model, "dx"), _stream(stream))
    _check("moe_permute_bwd", rc)


def moe_permute_bwd_add(shape, dx_perm, row_of_slot, dx_addend, dx, stream=None):
    import torch
    s = Shape.of(shape)
    bf = _bf16_types()
    rc = load_library().moe_permute_bwd_add(
        ctypes.byref(s._c), _ptr(dx_perm, bf, s.N * s.d_model, "dx_perm"),
        _ptr(row_of_slot, torch.int32, s.N, "row_of_slot"), _ptr(dx_addend, bf, s.T * s.d_model, "dx_addend"),
        _ptr(dx, bf, s.T * s.d_model, "dx"), _stream(stream))
    _check("moe_permute_bwd_add", rc)


def moe_router_fwd(shape, x, w_router, logits, ws, stream=None):
    import torch
    s = Shape.of(shape)
    bf = _bf16_types()
    rc = load_library().moe_router_fwd(
        ctypes.byref(s._c), _ptr(x, bf, s.T * s.d_model, "x"), _ptr(w_router, bf, s.E * s.d_model, "w_router"),
        _ptr(logits, torch.float32, s.T * s.E, "logits"), _ptr(ws, None, None, "ws"), ws.numel() * ws.element_size(),
        _stream(stream))
    _check("moe_router_fwd", rc)


def moe_router_bwd(shape, x, w_router, dlogits, dx_router, dw_router, accumulate, ws, stream=None):
    import torch
    s = Shape.of(shape)
    bf = _bf16_types()
    rc = load_library().moe_router_bwd(
        ctypes.byref(s._c), _ptr(x, bf, s.T * s.d_model, "x"), _ptr(w_router, bf, s.E * s.d_model, "w_router"),
        _ptr(dlogits, torch.float32, s.T * s.E, "dlogits"), _ptr(dx_router, bf, s.T * s.d_model, "dx_router"),
        _ptr(dw_router, torch.float32, s.E * s.d_model, "dw_router"), int(bool(accumulate)),
        _ptr(ws, None, None, "ws"), ws.numel() * ws.element_size(), _stream(stream))
    _check("moe_router_bwd", rc)


def moe_grouped_ffn_fwd(shape, x_perm, offsets, w_gate, w_up, w_down, y_perm, save_g, save_u, ws, stream=None):
    import torch
    s = Shape.of(shape)
    bf = _bf16_types()
    nw = s.E_total * s.d_model * s.d_ffn
    rc = load_library().moe_grouped_ffn_fwd(
        ctypes.byref(s._c), _ptr(x_perm, bf, s.N * s.d_model, "x_perm"), _ptr(offsets, torch.int32, s.E_total + 1, "offsets"),
        _ptr(w_gate, bf, nw, "w_gate"), _ptr(w_up, bf, nw, "w_up"), _ptr(w_down, bf, nw, "w_down"),
        _ptr(y_perm, bf, s.N * s.d_model, "y_perm"),
        None if save_g is None else _ptr(save_g, bf, s.N * s.d_ffn, "save_g"),
        None if save_u is None else _ptr(save_u, bf, s.N * s.d_ffn, "save_u"), _ptr(ws, None, None, "ws"),
        ws.numel() * ws.element_size(), _stream(stream))
    _check("moe_grouped_ffn_fwd", rc)


def moe_grouped_ffn_bwd_recompute(shape, dy_perm, x_perm, offsets, w_gate, w_up, w_down, dx_perm, dw_gate, dw_up, dw_down,
                                  accumulate, ws, stream=None):
    import torch
    s = Shape.of(shape)
    bf = _bf16_types()
    nw = s.E_total * s.d_model * s.d_ffn
    rc = load_library().moe_grouped_ffn_bwd_recompute(
        ctypes.byref(s._c), _ptr(dy_perm, bf, s.N * s.d_model, "dy_perm"), _ptr(x_perm, bf, s.N * s.d_model, "x_perm"),
        _ptr(offsets, torch.int32, s.E_total + 1, "offsets"), _ptr(w_gate, bf, nw, "w_gate"), _ptr(w_up, bf, nw, "w_up"),
        _ptr(w_down, bf, nw, "w_down"), _ptr(dx_perm, bf, s.N * s.d_model, "dx_perm"),
        _ptr(dw_gate, torch.float32, nw, "dw_gate"), _ptr(dw_up, torch.float32, nw, "dw_up"),
        _ptr(dw_down, torch.float32, nw, "dw_down"), int(bool(accumulate)), _ptr(ws, None, None, "ws"),
        ws.numel() * ws.element_size(), _stream(stream))
    _check("moe_grouped_ffn_bwd_recompute", rc)


def moe_grouped_ffn_bwd(shape, dy_perm, x_perm, offsets, w_gate, w_up, w_down, save_g, save_u, dx_perm,
                        dw_gate, dw_up, dw_down, accumulate, ws, stream=None):
    import torch
    s = Shape.of(shape)
    bf = _bf16_types()
    nw = s.E_total * s.d_model * s.d_ffn
    rc = load_library().moe_grouped_ffn_bwd(
        ctypes.byref(s._c), _ptr(dy_perm, bf, s.N * s.d_model, "dy_perm"), _ptr(x_perm, bf, s.N * s.d_model, "x_perm"),
        _ptr(offsets, torch.int32, s.E_total + 1, "offsets"), _ptr(w_gate, bf, nw, "w_gate"), _ptr(w_up, bf, nw, "w_up"),
        _ptr(w_down, bf, nw, "w_down"), _ptr(save_g, bf, s.N * s.d_ffn, "save_g"), _ptr(save_u, bf, s.N * s.d_ffn, "save_u"),
        _ptr(dx_perm, bf, s.N * s.d_model, "dx_perm"), _ptr(dw_gate, torch.float32, nw, "dw_gate"),
        _ptr(dw_up, torch.float32, nw, "dw_up"), _ptr(dw_down, torch.float32, nw, "dw_down"), int(bool(accumulate)),
        _ptr(ws, None, None, "ws"), ws.numel() * ws.element_size(), _stream(stream))
    _check("moe_grouped_ffn_bwd", rc)


def moe_unpermute_combine(shape, y_perm, row_of_slot, topk_w, out, stream=None):
    import torch
    s = Shape.of(shape)
    bf = _bf16_types()
    rc = load_library().moe_unpermute_combine(
        ctypes.byref(s._c), _ptr(y_perm, bf, s.N * s.d_model, "y_perm"), _ptr(row_of_slot, torch.int32, s.N, "row_of_slot"),
        _ptr(topk_w, torch.float32, s.N, "topk_w"), _ptr(out, bf, s.T * s.d_model, "out"), _stream(stream))
    _check("moe_unpermute_combine", rc)


def moe_unpermute_combine_bwd(shape, dout, y_perm, row_of_slot, topk_w, dy_perm, dtopk_w, stream=None):
    import torch
    s = Shape.of(shape)
    bf = _bf16_types()
    rc = load_library().moe_unpermute_combine_bwd(
        ctypes.byref(s._c), _ptr(dout, bf, s.T * s.d_model, "dout"), _ptr(y_perm, bf, s.N * s.d_model, "y_perm"),
        _ptr(row_of_slot, torch.int32, s.N, "row_of_slot"), _ptr(topk_w, torch.float32, s.N, "topk_w"),
        _ptr(dy_perm, bf, s.N * s.d_model, "dy_perm"), _ptr(dtopk_w, torch.float32, s.N, "dtopk_w"), _stream(stream))
    _check("moe_unpermute_combine_bwd", rc)


# ---- single-GPU steps of the hierarchical all-to-all (device tensors; rows of any dtype, 16-byte multiples) -----

def _rows(t, n_rows, what):
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{what}: expected a contiguous CUDA tensor")
    nbytes = t.numel() * t.element_size()
    if n_rows == 0:
        return ctypes.c_void_p(t.data_ptr()), 0
    if nbytes % n_rows:
        raise ValueError(f"{what}: {nbytes} bytes do not split into {n_rows} rows")
    return ctypes.c_void_p(t.data_ptr()), nbytes // n_rows


def moe_halo_pack_remote(S, F2s, num_nodes, R, node_id, stream=None):
    ps, rb = _rows(S, num_nodes * R, "S")
    pd, rb2 = _rows(F2s, (num_nodes - 1) * R, "F2s")
    if num_nodes > 1 and rb != rb2:
        raise ValueError("S and F2s differ in row size")
    _check("moe_halo_pack_remote", load_library().moe_halo_pack_remote(ps, pd, int(num_nodes), int(R), rb, int(node_id), _stream(stream)))


def moe_halo_repack(F2r, F3s, M, R, stream=None):
    ps, rb = _rows(F2r, M * R, "F2r")
    pd, rb2 = _rows(F3s, M * R, "F3s")
    if rb != rb2:
        raise ValueError("F2r and F3s differ in size")
    _check("moe_halo_repack", load_library().moe_halo_repack(ps, pd, int(M), int(R), rb if M else 16, _stream(stream)))


def moe_halo_unpack(P1, F3r, O, num_nodes, R, node_id, stream=None):
    p1, rb = _rows(P1, R, "P1")
    po, rb2 = _rows(O, num_nodes * R, "O")
    if rb != rb2:
        raise ValueError("P1 and O differ in row size")
    p3 = None
    if num_nodes > 1:
        p3, rb3 = _rows(F3r, R * (num_nodes - 1), "F3r")
        if rb3 != rb:
            raise ValueError("F3r and O differ in row size")
    _check("moe_halo_unpack", load_library().moe_halo_unpack(p1, p3, po, int(num_nodes), int(R), rb, int(node_id), _stream(stream)))


# ---- host-side load statistics and rebalancing (NumPy arrays; nothing here touches the GPU) ------------------

def _np(a, dtype, what):
    import numpy as np
    if not isinstance(a, np.ndarray) or a.dtype != dtype or not a.flags["C_CONTIGUOUS"]:
        raise ValueError(f"{what}: expected a C-contiguous numpy array of {np.dtype(dtype).name}")
    return a.ctypes.data_as(ctypes.c_void_p)


def load_accumulate(running, counts):
    """running[e] += counts[e] in place (running int64 [E], counts int32 [E], both on the host)."""
    import numpy as np
    if running.shape != counts.shape:
        raise ValueError("running and counts differ in shape")
    _check("moe_load_accumulate", load_library().moe_load_accumulate(_np(running, np.int64, "running"), _np(counts, np.int32, "counts"),
                                                                     int(running.size)))


def load_imbalance(load, groups) -> float:
    """max group load / mean group load for a placement `groups` (int32 [n_groups, experts per group])."""
    import numpy as np
    r = ctypes.c_double(0.0)
    _check("moe_load_imbalance", load_library().moe_load_imbalance(_np(load, np.int64, "load"), int(load.size), int(groups.shape[0]),
                                                                   _np(groups, np.int32, "groups"), ctypes.byref(r)))
    return float(r.value)


def rebalance_experts(load, groups, max_iters=100):
    """Algorithm 2 on a copy of `groups`; returns (new groups, swaps) with swaps an int32 [n, 2] array."""
    import numpy as np
    out = np.ascontiguousarray(groups, dtype=np.int32).copy()
    swaps = np.zeros((max(int(max_iters), 1), 2), dtype=np.int32)
    n = ctypes.c_int32(0)
    _check("moe_rebalance_experts", load_library().moe_rebalance_experts(
        _np(load, np.int64, "load"), int(load.size), int(out.shape[0]), _np(out, np.int32, "groups"), int(max_iters),
        ctypes.byref(n), _np(swaps, np.int32, "swaps")))
    return out, swaps[:n.value].copy()
