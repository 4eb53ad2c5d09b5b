"""Host-side checks of bench.py's bookkeeping (no GPU): the HBM traffic it reports for the dominant kernel is read from
the committed rocprofv3 summary, so the two cannot drift apart, and its algorithmic FLOP / byte counts follow the
definitions stated next to them."""
import os
import re

import bench
import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_traffic_comes_from_the_committed_profile():
    path = os.path.join(ROOT, "profiles", "grouped_gemm_mixtral_hbm_traffic.txt")
    text = open(path).read()
    got = bench.measured_traffic_bytes("mixtral")
    assert set(got) == {"ffn_fwd_gate_up_swiglu", "ffn_fwd_down", "ffn_bwd_dh_dswiglu", "ffn_bwd_dx", "ffn_bwd_dw_down",
                        "ffn_bwd_dw_gate_up"}
    # the file prints, per kernel, the two raw counters (KiB per dispatch) and the GB they scale to; the parsed byte
    # count must be the sum of those two GB columns
    for line in text.splitlines():
        f = line.split()
        if len(f) == 8 and f[0] in got:
            assert abs(got[f[0]] / 1e9 - (float(f[2]) + float(f[5]))) < 0.02, f[0]
    assert bench.measured_traffic_bytes("no_such_workload") == {}


def test_flop_and_byte_counts():
    sh = W.WORKLOADS["mixtral"].shape
    unit = 2 * sh.d_model * sh.d_ffn * sh.N
    total = sum(bench.gemm_flops_per_launch(k, sh) for k in ("ffn_fwd_gate_up_swiglu", "ffn_fwd_down", "ffn_bwd_dh_dswiglu",
                                                             "ffn_bwd_dx", "ffn_bwd_dw_down", "ffn_bwd_dw_gate_up"))
    assert total == 9 * unit == sh.flops_fwd_bwd()
    # weight gradients: operands once + fp32 dW of every expert
    by = bench.gemm_bytes_per_launch("ffn_bwd_dw_gate_up", sh, sh.E_total)
    assert by == sh.N * sh.d_model * 2 + 2 * sh.N * sh.d_ffn * 2 + 2 * sh.E_total * sh.d_model * sh.d_ffn * 4
    # the Mixtral-shaped GEMMs are MFMA-bound, the expert shard's are HBM-bound (weights streamed for ~128 rows each)
    assert bench.gemm_roofline("ffn_fwd_gate_up_swiglu", sh, 8, 2.0)["bound"] == "mfma"
    shard = W.WORKLOADS["shard"].shape
    r = bench.gemm_roofline("ffn_bwd_dw_gate_up", shard, 32, 1.0)
    assert r["bound"] == "hbm" and r["unit"] == "GB/s"
    assert bench.gemm_roofline("ffn_fwd_gate_up_swiglu", shard, 32, 1.0)["bound"] == "hbm"
