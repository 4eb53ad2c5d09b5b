"""moe_permute_noalloc (the entry point for callers that cannot allocate or bring a workspace) against moe_permute:
every output bit for bit, on two calls in a row, the second with a smaller input (the shared static scratch keeps
the first call's contents)."""
import numpy as np
import pytest
import torch

import workloads as W

pytestmark = pytest.mark.gpu


def _case(T, d, E, k, Es, seed):
    rng = np.random.default_rng(seed)
    keys = rng.gumbel(size=(T, E)) - 1.2 * np.log(np.arange(1, E + 1))[None, :]
    idx = np.empty((T, k + Es), dtype=np.int32)
    idx[:, :k] = np.argsort(-keys, axis=1)[:, :k]
    for j in range(Es):
        idx[:, k + j] = E + j
    xb = W.make_tokens(W.MoEShape(T, d, 64, E, k, Es), seed=seed)
    return idx, xb


def _run(moe, fn, s, d_x, d_idx, *extra):
    Et, N = s.E_total, s.N
    outs = [torch.full((Et,), -1, dtype=torch.int32, device="cuda"), torch.full((Et + 1,), -1, dtype=torch.int32, device="cuda"),
            torch.full((N,), -1, dtype=torch.int32, device="cuda"), torch.full((N,), -1, dtype=torch.int32, device="cuda")]
    xp = torch.zeros((N, s.d_model), dtype=torch.bfloat16, device="cuda")
    fn(s, d_x, d_idx, xp, *outs, *extra)
    torch.cuda.synchronize()
    return outs + [xp.view(torch.int16)]


def test_noalloc_permute_matches_permute_twice(moe):
    # first a larger input (40 rank blocks, 130 expert ids), then a smaller one of another shape
    for T, d, E, k, Es, seed in ((10000, 256, 128, 4, 2, 1), (777, 128, 16, 2, 0, 2)):
        idx, xb = _case(T, d, E, k, Es, seed)
        s = moe.Shape(T, d, 64, E, k, Es, 1)
        d_idx = torch.from_numpy(idx).cuda()
        d_x = torch.from_numpy(xb.view(np.int16)).cuda().view(torch.bfloat16)
        ws = torch.empty(moe.workspace_bytes(s), dtype=torch.uint8, device="cuda")
        ref = _run(moe, moe.moe_permute, s, d_x, d_idx, ws)
        got = _run(moe, moe.moe_permute_noalloc, s, d_x, d_idx)
        for name, a, b in zip(("counts", "offsets", "row_of_slot", "slot_of_row", "x_perm"), ref, got):
            assert torch.equal(a, b), (T, name)


def test_noalloc_permute_rejects_what_does_not_fit(moe):
    import ctypes
    lib = moe.load_library()
    fake = ctypes.c_void_p(0x10000)
    big = moe.Shape(1 << 19, 64, 64, 8, 4)                 # T*K' = 2^21 slots
    assert lib.moe_permute_noalloc(ctypes.byref(big._c), fake, fake, fake, fake, fake, fake, fake, None) == -4
    wide = moe.Shape(1 << 18, 64, 64, 1024, 4)             # 1024 rank blocks x 1024 experts = 2^20: fits exactly
    wider = moe.Shape((1 << 18) + 256, 64, 64, 1024, 4)    # one rank block more: does not
    assert lib.moe_permute_noalloc(ctypes.byref(wider._c), fake, fake, fake, fake, fake, fake, fake, None) == -4
    assert lib.moe_permute_noalloc(ctypes.byref(wide._c), None, fake, fake, fake, fake, fake, fake, None) == -1
