"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol include/moe.h declares,
and rejects bad arguments before anything is launched."""
import ctypes
import os
import re

import pytest

import paper_2605_05049_amd as moe
from paper_2605_05049_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    return moe.load_library()


def test_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "moe.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(moe_[a-z_0-9]+)\s*\(", header))
    assert declared == set(moe.EXPORTED_SYMBOLS)
    for name in declared:
        assert hasattr(lib, name), name
    assert moe.abi_version() == 1


def test_status_strings(lib):
    assert moe.status_str(0) == "ok"
    for code in (-1, -2, -3, -4, -5):
        assert moe.status_str(code) not in ("ok", "unknown status")
    assert moe.status_str(-99) == "unknown status"


def test_workspace_bytes_follows_the_shape(lib):
    s = moe.Shape(256, 512, 1024, 8, 2)
    n = moe.workspace_bytes(s)
    # three [N,f] bf16 intermediates (H, dG, dU) plus the fixed 80 MiB of partial tiles of split contractions
    assert 3 * s.N * s.d_ffn * 2 + (80 << 20) <= n <= 3 * s.N * s.d_ffn * 2 + (82 << 20) and n % 256 == 0
    assert moe.workspace_bytes(moe.Shape(512, 512, 1024, 8, 2)) > n
    assert moe.workspace_bytes(moe.Shape(256, 500, 1024, 8, 2)) == 0       # d not a multiple of 64
    assert moe.workspace_bytes(moe.Shape(256, 512, 1024, 8, 9)) == 0       # k > E
    assert moe.workspace_bytes(moe.Shape(256, 512, 1024, 2000, 2)) == 0    # E over the limit
    assert moe.workspace_bytes(moe.Shape(2 ** 30, 512, 1024, 8, 2)) == 0   # T*K' >= 2^31
    assert moe.workspace_bytes(moe.Shape(1, 2 ** 22, 64, 8, 2)) > 0        # the widest rows the GEMM loads can address
    assert moe.workspace_bytes(moe.Shape(1, 2 ** 22 + 64, 64, 8, 2)) == 0  # beyond: the 32-bit row offsets would wrap
    assert moe.workspace_bytes(moe.Shape(1, 64, 2 ** 22 + 64, 8, 2)) == 0


def _shape(**kw):
    base = dict(T=256, d_model=512, d_ffn=1024, E=8, k=2, E_shared=0, renorm=1)
    base.update(kw)
    return moe.Shape(**base)


FAKE = ctypes.c_void_p(0x10000)        # aligned, never dereferenced: every call below fails its host checks first
ODD = ctypes.c_void_p(0x10004)


def test_argument_checks_run_before_any_launch(lib):
    s = _shape()
    sp = ctypes.byref(s._c)
    bad = ctypes.byref(_shape(k=0)._c)
    assert lib.moe_route_topk(sp, None, FAKE, FAKE, None, None) == -1
    assert lib.moe_route_topk(bad, FAKE, FAKE, FAKE, None, None) == -2
    assert lib.moe_route_topk(sp, ODD, FAKE, FAKE, None, None) == -3
    assert lib.moe_route_topk(None, FAKE, FAKE, FAKE, None, None) == -1
    assert lib.moe_route_topk_bwd(sp, FAKE, FAKE, FAKE, None, None, None) == -1
    nr = ctypes.byref(_shape(renorm=0)._c)
    assert lib.moe_route_topk_bwd(nr, FAKE, FAKE, FAKE, None, FAKE, None) == -1    # probs needed without renorm
    assert lib.moe_permute(sp, FAKE, None, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 1 << 40, None) == -1
    assert lib.moe_permute(sp, FAKE, FAKE, None, FAKE, FAKE, FAKE, FAKE, FAKE, 1 << 40, None) == -1   # x without x_perm
    assert lib.moe_permute(sp, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 16, None) == -4
    assert lib.moe_permute(sp, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, ctypes.c_void_p(0x10010), 1 << 40, None) == -3
    assert lib.moe_permute_bwd(sp, FAKE, None, FAKE, None) == -1
    assert lib.moe_grouped_ffn_fwd(sp, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 16, None) == -4
    assert lib.moe_grouped_ffn_fwd(sp, FAKE, FAKE, FAKE, None, FAKE, FAKE, FAKE, FAKE, FAKE, 1 << 40, None) == -1
    assert lib.moe_grouped_ffn_fwd(bad, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 1 << 40, None) == -2
    wide = ctypes.byref(_shape(d_model=2 ** 22 + 64)._c)
    assert lib.moe_grouped_ffn_fwd(wide, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 1 << 40, None) == -2
    assert lib.moe_grouped_ffn_bwd(sp, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None, 0,
                                   FAKE, 1 << 40, None) == -1
    assert lib.moe_grouped_ffn_bwd(sp, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 0,
                                   FAKE, 16, None) == -4
    assert lib.moe_grouped_ffn_fwd(sp, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None, FAKE, FAKE, 1 << 40, None) == -1   # G without U
    assert lib.moe_grouped_ffn_bwd_recompute(sp, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 0, FAKE, 16, None) == -4
    assert lib.moe_grouped_ffn_bwd_recompute(sp, FAKE, None, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 0, FAKE, 1 << 40, None) == -1
    assert lib.moe_grouped_ffn_bwd_recompute(sp, None, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 0, FAKE, 1 << 40, None) == -1
    assert lib.moe_unpermute_combine(sp, FAKE, FAKE, None, FAKE, None) == -1
    assert lib.moe_unpermute_combine(sp, FAKE, FAKE, ODD, FAKE, None) == -3
    assert lib.moe_unpermute_combine_bwd(sp, FAKE, FAKE, FAKE, FAKE, FAKE, None, None) == -1
    assert lib.moe_permute_bwd_add(sp, FAKE, FAKE, None, FAKE, None) == -1
    assert lib.moe_permute_bwd_add(sp, FAKE, FAKE, ODD, FAKE, None) == -3
    assert lib.moe_router_fwd(sp, FAKE, None, FAKE, FAKE, 1 << 40, None) == -1
    assert lib.moe_router_fwd(sp, FAKE, FAKE, FAKE, FAKE, 16, None) == -4
    assert lib.moe_router_fwd(bad, FAKE, FAKE, FAKE, FAKE, 1 << 40, None) == -2
    assert lib.moe_router_bwd(sp, FAKE, FAKE, FAKE, FAKE, None, 0, FAKE, 1 << 40, None) == -1
    assert lib.moe_router_bwd(sp, FAKE, FAKE, ODD, FAKE, FAKE, 0, FAKE, 1 << 40, None) == -3
    assert lib.moe_router_bwd(sp, FAKE, FAKE, FAKE, FAKE, FAKE, 0, None, 0, None) == -1


def test_binding_rejects_host_tensors(lib):
    import torch
    s = _shape(T=4)
    with pytest.raises(ValueError):
        moe.moe_route_topk(s, torch.zeros(4, 8), torch.zeros(4, 2, dtype=torch.int32), torch.zeros(4, 2))


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "_LIB_NAME", "libmoe_does_not_exist.so")
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        B.load_library()
