"""The single-GPU steps of the hierarchical all-to-all (Section V, Algorithm 1).

CPU: the oracle's three local steps are pinned by running the whole three-phase algorithm over all ranks (exchanges
done by plain host indexing) and comparing with the definition of an all-to-all, O_g[j] = S_j[g], plus loop
definitions of each step.  GPU: the kernels against the oracle, bit for bit (they only move bytes)."""
import ctypes

import numpy as np
import pytest

import paper_2605_05049_amd as moe
from oracle import moe_oracle as O


@pytest.mark.parametrize("num_nodes,R,D", [(1, 4, 3), (2, 8, 5), (3, 2, 4), (4, 3, 2), (5, 1, 6)])
def test_oracle_steps_compose_to_an_all_to_all(num_nodes, R, D):
    Wn = num_nodes * R
    rng = np.random.default_rng(num_nodes * 100 + R)
    send = [rng.integers(0, 1 << 30, size=(Wn, D)) for _ in range(Wn)]
    out = O.halo_all_to_all_reference(send, num_nodes, R)
    for g in range(Wn):
        for j in range(Wn):
            assert np.array_equal(out[g][j], send[j][g]), (g, j)


def test_oracle_steps_match_loop_definitions():
    num_nodes, R, D, node_id = 4, 3, 2, 2
    M = num_nodes - 1
    S = np.arange(num_nodes * R * D).reshape(num_nodes * R, D)
    F2s = O.halo_pack_remote(S, num_nodes, R, node_id)
    rem = [0, 1, 3]
    assert O.halo_remote_nodes(num_nodes, node_id) == rem
    for i, n in enumerate(rem):
        for r in range(R):
            assert np.array_equal(F2s[i * R + r], S[n * R + r])
    F2r = np.arange(M * R * D).reshape(M * R, D) + 500
    F3s = O.halo_repack_phase3(F2r, M, R)
    assert F3s.shape == (R, M * D)
    for r in range(R):
        for i in range(M):
            assert np.array_equal(F3s[r, i * D:(i + 1) * D], F2r[i * R + r])
    P1 = np.arange(R * D).reshape(R, D) + 900
    F3r = np.arange(R * M * D).reshape(R, M * D) + 2000
    Oo = O.halo_unpack_output(P1, F3r, num_nodes, R, node_id)
    for r in range(R):
        assert np.array_equal(Oo[node_id * R + r], P1[r])
    for i, n in enumerate(rem):
        for p in range(R):
            assert np.array_equal(Oo[n * R + p], F3r[p, i * D:(i + 1) * D])


def test_host_argument_checks():
    lib = moe.load_library()
    FAKE, ODD = ctypes.c_void_p(0x10000), ctypes.c_void_p(0x10004)
    assert lib.moe_halo_pack_remote(FAKE, FAKE, 0, 8, 64, 0, None) == -2          # no nodes
    assert lib.moe_halo_pack_remote(FAKE, FAKE, 4, 8, 24, 0, None) == -2          # rows not a multiple of 16 bytes
    assert lib.moe_halo_pack_remote(FAKE, FAKE, 4, 8, 64, 4, None) == -2          # node_id out of range
    assert lib.moe_halo_pack_remote(None, FAKE, 4, 8, 64, 1, None) == -1
    assert lib.moe_halo_pack_remote(FAKE, ODD, 4, 8, 64, 1, None) == -3
    assert lib.moe_halo_pack_remote(None, None, 1, 8, 64, 0, None) == 0           # a single node has nothing remote
    assert lib.moe_halo_repack(FAKE, None, 3, 8, 64, None) == -1
    assert lib.moe_halo_unpack(FAKE, None, FAKE, 3, 8, 64, 0, None) == -1         # F3r needed with remote nodes
    assert lib.moe_halo_unpack(None, None, FAKE, 1, 8, 64, 0, None) == -1


HALO_CASES = [
    # num_nodes, R, row elements (bf16), node_id
    (4, 8, 4096, 1), (2, 8, 8 * 1024, 0), (1, 8, 512, 0), (5, 3, 24, 4), (16, 8, 8, 7), (3, 1, 100 * 8, 2),
]


@pytest.mark.gpu
@pytest.mark.parametrize("num_nodes,R,D,node_id", HALO_CASES)
def test_kernels_match_oracle(num_nodes, R, D, node_id):
    import torch
    M = num_nodes - 1
    rng = np.random.default_rng(num_nodes * 1000 + R * 10 + node_id)
    mk = lambda rows: rng.integers(0, 1 << 16, size=(rows, D), dtype=np.uint16)  # noqa: E731
    up = lambda a: torch.from_numpy(a.view(np.int16)).cuda()                     # noqa: E731
    S, F2r, P1, F3r = mk(num_nodes * R), mk(M * R), mk(R), mk(R * M).reshape(R, M * D)
    F2s = torch.full((M * R, D), -1, dtype=torch.int16, device="cuda")
    moe.moe_halo_pack_remote(up(S), F2s, num_nodes, R, node_id)
    assert np.array_equal(F2s.cpu().numpy().view(np.uint16), O.halo_pack_remote(S, num_nodes, R, node_id))
    F3s = torch.full((R, M * D), -1, dtype=torch.int16, device="cuda")
    moe.moe_halo_repack(up(F2r), F3s, M, R)
    if M:
        assert np.array_equal(F3s.cpu().numpy().view(np.uint16), O.halo_repack_phase3(F2r, M, R))
    Oo = torch.full((num_nodes * R, D), -1, dtype=torch.int16, device="cuda")
    moe.moe_halo_unpack(up(P1), up(F3r) if M else None, Oo, num_nodes, R, node_id)
    assert np.array_equal(Oo.cpu().numpy().view(np.uint16), O.halo_unpack_output(P1, F3r, num_nodes, R, node_id))
