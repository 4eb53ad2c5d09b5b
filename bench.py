#!/usr/bin/env python3
"""Benchmark of the MoE expert layer on one MI355X: one step = one forward + backward pass of the whole hot path
(route -> permute -> grouped FFN -> combine, then combine_bwd -> grouped FFN bwd -> permute_bwd -> route_bwd) over one
batch of seeded synthetic input already resident in HBM.

Prints ONE JSON line.  `value` is fwd+bwd TFLOP/s with FLOPs = 18*d*f*N (three 2*d*f GEMMs per permuted row forward,
twice that backward; padded rows and empty experts are never counted).  `roofline` prices the slowest kernel of the
step against the bf16 dense MFMA peak from per-launch HIP-event timings taken live in a second, instrumented pass.
`permute_combine` reports the streaming kernels' HBM rate on the imbalance workload, `workloads` the same step on the
other three full-size workloads (each GEMM priced against the larger of its MFMA and its HBM time), `calibration` what
plain device copies, fills and reductions reach on the same box.  `cpu_baseline` times the fp64 oracle on a bounded
sample of the same workload on the host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_MFMA_TFLOPS = 2500.0   # MI355X dense bf16 MFMA, published
PEAK_HBM_GBS = 8000.0            # MI355X HBM3E, published

PROFILE_DIR = os.path.join(ROOT, "profiles")


def measured_traffic_bytes(workload):
    """HBM-side bytes per launch (read + written) of the grouped GEMM kernels, from the committed summary of the two
    rocprofv3 counter runs (FETCH_SIZE, WRITE_SIZE in KiB per dispatch, each scaled by what the same counter read for a
    plain copy of known size): profiles/grouped_gemm_<workload>_hbm_traffic.txt.  Counters cannot be read from inside
    this script; a workload without such a summary reports null."""
    path = os.path.join(PROFILE_DIR, f"grouped_gemm_{workload}_hbm_traffic.txt")
    if not os.path.exists(path):
        return {}
    import re
    text = open(path).read()
    m = re.search(r"scale factors ([0-9.]+) \(fetch\), ([0-9.]+) \(write\)", text)
    if not m:
        return {}
    sf, sw = float(m.group(1)), float(m.group(2))
    out = {}
    for line in text.splitlines():
        f = line.split()
        if len(f) == 8 and f[0].startswith("ffn_"):
            out[f[0]] = int((float(f[1]) * sf + float(f[4]) * sw) * 1024)
    return out


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="mixtral", help="mixtral (headline) | tiny | finegrained | shard | imbalance")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-streaming", action="store_true", help="skip the permute/combine bandwidth measurement")
    ap.add_argument("--no-calibration", action="store_true",
                    help="skip the plain 512 MiB device copy / fill / reduction (what this box's HBM reaches; the copy is also "
                         "the reference for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--no-workloads", action="store_true", help="skip the brief runs of the other full-size workloads")
    ap.add_argument("--cpu-sample-tokens", type=int, default=0, help="tokens of the workload the oracle is timed on (0 = auto)")
    return ap.parse_args()


def dev_bf16(bits):
    import numpy as np
    import torch
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def gemm_flops_per_launch(label, shape):
    """Algorithmic FLOPs of one launch of each grouped-GEMM kernel: 2*d*f per row and matrix."""
    unit = 2.0 * shape.d_model * shape.d_ffn * shape.N
    return {"ffn_fwd_gate_up_swiglu": 2 * unit, "ffn_fwd_down": unit, "ffn_bwd_dh_dswiglu": unit,
            "ffn_bwd_dx": 2 * unit, "ffn_bwd_dw_down": unit, "ffn_bwd_dw_gate_up": 2 * unit}.get(label)


def gemm_bytes_per_launch(label, shape, n_active):
    """Algorithmic HBM bytes of one launch of each grouped-GEMM kernel: every operand read once, every output written
    once; weights only of the n_active experts that have rows; the fp32 weight gradients of all E' experts (empty ones
    are zero-filled)."""
    d, f, N, Et = shape.d_model, shape.d_ffn, shape.N, shape.E_total
    act_d, act_f, w1 = N * d * 2, N * f * 2, n_active * d * f * 2
    return {"ffn_fwd_gate_up_swiglu": act_d + 2 * w1 + 3 * act_f, "ffn_fwd_down": act_f + w1 + act_d,
            "ffn_bwd_dh_dswiglu": act_d + w1 + 2 * act_f + 3 * act_f, "ffn_bwd_dx": 2 * act_f + 2 * w1 + act_d,
            "ffn_bwd_dw_down": act_f + act_d + Et * d * f * 4, "ffn_bwd_dw_gate_up": act_d + 2 * act_f + 2 * Et * d * f * 4}.get(label)


def gemm_roofline(label, shape, n_active, avg_ms):
    """A GEMM launch against the larger of its two lower bounds: FLOPs at the dense bf16 MFMA peak, algorithmic bytes
    at the HBM peak."""
    fl, by = gemm_flops_per_launch(label, shape), gemm_bytes_per_launch(label, shape, n_active)
    t_mfma, t_hbm = fl / (PEAK_BF16_MFMA_TFLOPS * 1e12), by / (PEAK_HBM_GBS * 1e9)
    t = avg_ms * 1e-3
    if t_hbm > t_mfma:
        return {"bound": "hbm", "achieved": round(by / t / 1e9, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(t_hbm / t, 4)}
    return {"bound": "mfma", "achieved": round(fl / t / 1e12, 2), "peak": PEAK_BF16_MFMA_TFLOPS, "unit": "TFLOP/s", "frac": round(t_mfma / t, 4)}


def stream_bytes_per_launch(label, shape):
    """Algorithmic HBM bytes of one launch of each streaming kernel (bf16 rows + int32 maps + fp32 weights)."""
    T, d, N = shape.T, shape.d_model, shape.N
    return {
        "perm_scatter_gather": T * d * 2 + N * d * 2 + N * 4 * 4,       # read x once, write x_perm, idx+rank in, 2 maps out
        "unpermute_combine": N * d * 2 + N * 8 + T * d * 2,
        "unpermute_combine_bwd": T * d * 2 + 2 * N * d * 2 + N * 12,
        "permute_bwd": N * d * 2 + N * 4 + T * d * 2,
    }.get(label)


def run_layer_bench(moe, W, args):
    import torch
    wl = W.WORKLOADS[args.workload]
    sh = wl.shape
    t0 = time.time()
    inp = W.make_layer_inputs(wl, seed=args.seed)
    gen_s = time.time() - t0
    s = moe.Shape.of(sh)
    buf = moe.MoeLayerBuffers(s)
    x, dout = dev_bf16(inp["x"]), dev_bf16(inp["dout"])
    wg, wu, wd = dev_bf16(inp["w_gate"]), dev_bf16(inp["w_up"]), dev_bf16(inp["w_down"])
    if "logits" in inp:
        logits = torch.from_numpy(inp["logits"]).cuda()
    else:
        logits = None
        buf.topk_idx.copy_(torch.from_numpy(inp["topk_idx"]).cuda())
        buf.topk_w.copy_(torch.from_numpy(inp["topk_w"]).cuda())

    def step():
        moe.layer_forward(buf, x, wg, wu, wd, logits)
        moe.layer_backward(buf, dout, wg, wu, wd, accumulate=False, with_router=logits is not None)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    # forward and backward on their own (HIP events on the launch stream, median and minimum over single steps)
    def per_step_ms(fn, n):
        out = []
        for _ in range(n):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            e1.synchronize()
            out.append(e0.elapsed_time(e1))
        out.sort()
        return {"median_ms": round(out[len(out) // 2], 4), "min_ms": round(out[0], 4)}
    n_split = max(3, min(args.steps, 10))
    split = {"fwd": per_step_ms(lambda: moe.layer_forward(buf, x, wg, wu, wd, logits), n_split),
             "bwd": per_step_ms(lambda: moe.layer_backward(buf, dout, wg, wu, wd, accumulate=False,
                                                           with_router=logits is not None), n_split),
             "fwd_bwd": per_step_ms(step, n_split)}

    # instrumented pass: per-launch HIP events on the launch stream
    moe.profile_reset()
    moe.profile_enable(True)
    prof_steps = max(1, min(args.steps, 5))
    for _ in range(prof_steps):
        step()
    torch.cuda.synchronize()
    moe.profile_enable(False)
    recs = moe.profile_records()
    moe.profile_reset()
    per_kernel = {}
    for name, ms in recs:
        per_kernel.setdefault(name, []).append(ms)
    kernels = {k: {"launches_per_step": len(v) // prof_steps, "avg_ms": sum(v) / len(v)} for k, v in per_kernel.items()}
    counts = buf.counts.cpu().numpy()
    load = {"experts_with_rows": int((counts > 0).sum()), "rows_min": int(counts.min()), "rows_median": int(sorted(counts)[len(counts) // 2]),
            "rows_max": int(counts.max())}
    return inp, sh, elapsed, kernels, gen_s, split, load


def run_workload_brief(moe, W, name, steps, seed):
    """One of the other full-size workloads, briefly: the same whole step (route -> ... -> route_bwd) on the workload's
    own routing input and seeded tokens; the expert weights are drawn on the device (N(0, 0.02), bf16) instead of on the
    host to keep the run short.  Reports ms per step, TFLOP/s and every GEMM against its own bound."""
    import torch
    wl = W.WORKLOADS[name]
    sh = wl.shape
    inp = W.make_layer_inputs(wl, seed=seed, with_weights=False)
    s = moe.Shape.of(sh)
    buf = moe.MoeLayerBuffers(s)
    x, dout = dev_bf16(inp["x"]), dev_bf16(inp["dout"])
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    Et, d, f = sh.E_total, sh.d_model, sh.d_ffn
    wg = (torch.randn((Et, d, f), generator=g, device="cuda") * 0.02).to(torch.bfloat16)
    wu = (torch.randn((Et, d, f), generator=g, device="cuda") * 0.02).to(torch.bfloat16)
    wd = (torch.randn((Et, f, d), generator=g, device="cuda") * 0.02).to(torch.bfloat16)
    if "logits" in inp:
        logits = torch.from_numpy(inp["logits"]).cuda()
    else:
        logits = None
        buf.topk_idx.copy_(torch.from_numpy(inp["topk_idx"]).cuda())
        buf.topk_w.copy_(torch.from_numpy(inp["topk_w"]).cuda())

    def step():
        moe.layer_forward(buf, x, wg, wu, wd, logits)
        moe.layer_backward(buf, dout, wg, wu, wd, accumulate=False, with_router=logits is not None)

    for _ in range(2):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        step()
    e1.record()
    e1.synchronize()
    ms = e0.elapsed_time(e1) / steps
    moe.profile_reset()
    moe.profile_enable(True)
    for _ in range(2):
        step()
    torch.cuda.synchronize()
    moe.profile_enable(False)
    per = {}
    for kn, t in moe.profile_records():
        per.setdefault(kn, []).append(t)
    moe.profile_reset()
    counts = buf.counts.cpu().numpy()
    n_active = int((counts > 0).sum())
    gemms, t_bound = {}, 0.0
    for kn, v in per.items():
        if gemm_flops_per_launch(kn, sh):
            avg = sum(v) / len(v)
            r = gemm_roofline(kn, sh, n_active, avg)
            gemms[kn] = {"avg_ms": round(avg, 4), "bound": r["bound"], "frac": r["frac"]}
            t_bound += r["frac"] * avg
    dom = max(gemms, key=lambda k: gemms[k]["avg_ms"])
    flops = sh.flops_fwd_bwd()
    out = {"config": f"T={sh.T} d_model={sh.d_model} d_ffn={sh.d_ffn} E={sh.E}+{sh.E_shared} shared top-{sh.k} (N={sh.N} rows)",
           "ms_per_step": round(ms, 4), "TFLOPs": round(flops / (ms * 1e-3) / 1e12, 1),
           "frac_bf16_mfma_peak": round(flops / (ms * 1e-3) / 1e12 / PEAK_BF16_MFMA_TFLOPS, 4),
           "gemm_ms": round(sum(e["avg_ms"] for e in gemms.values()), 4),
           "gemm_frac_of_own_bounds": round(t_bound / sum(e["avg_ms"] for e in gemms.values()), 4),
           "dominant": dict(kernel=dom, **gemms[dom]), "gemms": gemms,
           "rows_per_expert": {"with_rows": n_active, "min": int(counts.min()), "median": int(sorted(counts)[len(counts) // 2]), "max": int(counts.max())}}
    del buf, wg, wu, wd
    torch.cuda.empty_cache()
    return out


def run_streaming_bench(moe, W, steps):
    """permute / combine family on the imbalance workload's shape (working set 671 MB per kernel, larger than the
    256 MB last-level cache).  Each kernel is timed in its own loop over three rotating buffer sets, so no launch
    finds in cache what an earlier launch touched."""
    import numpy as np
    import torch
    wl = W.WORKLOADS["imbalance"]
    sh = wl.shape
    s = moe.Shape.of(sh)
    logits, _ = W.make_forced_imbalance_logits(sh, seed=0)
    d_logits = torch.from_numpy(logits).cuda()
    N, T, d, Kp, Et = s.N, s.T, s.d_model, s.K_slots, s.E_total
    sets = []
    for i in range(3):
        sets.append(dict(
            x=dev_bf16(W.make_tokens(sh, seed=i)), dout=dev_bf16(W.make_dout(sh, seed=i)),
            x_perm=torch.empty((N, d), dtype=torch.bfloat16, device="cuda"),
            y_perm=torch.randn((N, d), device="cuda").to(torch.bfloat16),
            dy_perm=torch.empty((N, d), dtype=torch.bfloat16, device="cuda"),
            out=torch.empty((T, d), dtype=torch.bfloat16, device="cuda"),
            dx=torch.empty((T, d), dtype=torch.bfloat16, device="cuda"),
            dtw=torch.empty((T, Kp), dtype=torch.float32, device="cuda")))
    idx = torch.empty((T, Kp), dtype=torch.int32, device="cuda")
    w = torch.empty((T, Kp), dtype=torch.float32, device="cuda")
    counts = torch.empty((Et,), dtype=torch.int32, device="cuda")
    offsets = torch.empty((Et + 1,), dtype=torch.int32, device="cuda")
    ros = torch.empty((N,), dtype=torch.int32, device="cuda")
    sor = torch.empty((N,), dtype=torch.int32, device="cuda")
    ws = torch.empty(moe.workspace_bytes(s), dtype=torch.uint8, device="cuda")
    moe.moe_route_topk(s, d_logits, idx, w, None)
    calls = {
        "moe_permute": lambda b: moe.moe_permute(s, b["x"], idx, b["x_perm"], counts, offsets, ros, sor, ws),
        "moe_unpermute_combine": lambda b: moe.moe_unpermute_combine(s, b["y_perm"], ros, w, b["out"]),
        "moe_unpermute_combine_bwd": lambda b: moe.moe_unpermute_combine_bwd(s, b["dout"], b["y_perm"], ros, w, b["dy_perm"], b["dtw"]),
        "moe_permute_bwd": lambda b: moe.moe_permute_bwd(s, b["y_perm"], ros, b["dx"]),
    }
    calls["moe_permute"](sets[0])      # the maps the other calls use
    torch.cuda.synchronize()
    out = {"workload": "imbalance: T=16384 d=4096 E=128 top-4 (N=65536)", "peak_GBs": PEAK_HBM_GBS, "kernels": {}}
    for call, fn in calls.items():
        for i in range(3):
            fn(sets[i])
        torch.cuda.synchronize()
        moe.profile_reset()
        moe.profile_enable(True)
        for i in range(steps):
            fn(sets[i % 3])
        torch.cuda.synchronize()
        moe.profile_enable(False)
        per = {}
        for name, ms in moe.profile_records():
            per.setdefault(name, []).append(ms)
        moe.profile_reset()
        for name, v in per.items():
            avg = sum(v) / len(v)
            b = stream_bytes_per_launch(name, sh)
            ent = {"avg_us": round(avg * 1e3, 2)}
            if b:
                ent["algorithmic_MB"] = round(b / 1e6, 1)
                ent["GBs"] = round(b / (avg * 1e-3) / 1e9, 1)
                ent["frac_hbm_peak"] = round(b / (avg * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)
            out["kernels"][name] = ent
        if call == "moe_permute":
            # the whole call (its three launches back to back, nothing recorded between them): one pair of events around
            # a run of calls on rotating buffers
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for i in range(steps):
                fn(sets[i % 3])
            e1.record()
            e1.synchronize()
            tot = e0.elapsed_time(e1) / steps
            b = stream_bytes_per_launch("perm_scatter_gather", sh)
            out["moe_permute_total"] = {"avg_us": round(tot * 1e3, 2), "GBs": round(b / (tot * 1e-3) / 1e9, 1),
                                        "frac_hbm_peak": round(b / (tot * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                                        "sum_of_launches_us": round(sum(sum(v) / len(v) for v in per.values()) * 1e3, 2)}
    del sets
    torch.cuda.empty_cache()
    return out


def run_router_bench(moe, W, workload, steps):
    """The router's three GEMMs (logits = x W_r^T, its dx term, dW_r) on the workload's shape, each call timed in its
    own loop; they are skinny (E columns), so the bound is the HBM traffic of x, not the matrix cores."""
    import numpy as np
    import torch
    sh = W.WORKLOADS[workload].shape
    s = moe.Shape.of(sh)
    T, d, E = s.T, s.d_model, s.E
    x = dev_bf16(W.make_tokens(sh, seed=0))
    wr = dev_bf16(W.make_router_weight(sh, seed=0))
    dl = torch.from_numpy((np.random.default_rng(5).standard_normal((T, E)) * 0.1).astype(np.float32)).cuda()
    logits = torch.empty((T, E), dtype=torch.float32, device="cuda")
    dxr = torch.empty((T, d), dtype=torch.bfloat16, device="cuda")
    dwr = torch.empty((E, d), dtype=torch.float32, device="cuda")
    ws = torch.empty(moe.workspace_bytes(s), dtype=torch.uint8, device="cuda")
    calls = {"moe_router_fwd": lambda: moe.moe_router_fwd(s, x, wr, logits, ws),
             "moe_router_bwd": lambda: moe.moe_router_bwd(s, x, wr, dl, dxr, dwr, 0, ws)}
    alg = {"router_fwd": T * d * 2 + E * d * 2 + T * E * 4,                    # read x and W_r, write logits
           "router_bwd_dx": T * E * 4 + E * d * 2 + T * d * 2,                 # read dlogits and W_r, write dx
           "router_bwd_dw": T * E * 4 + T * d * 2 + E * d * 4}                 # read dlogits and x, write dW_r
    out = {"workload": f"{workload}: T={T} d={d} E={E}", "calls": {}, "kernels": {}}
    for name, fn in calls.items():
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        out["calls"][name] = {"avg_us": round(e0.elapsed_time(e1) / steps * 1e3, 1)}
        moe.profile_reset()
        moe.profile_enable(True)
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        moe.profile_enable(False)
        per = {}
        for kn, ms in moe.profile_records():
            per.setdefault(kn, []).append(ms)
        moe.profile_reset()
        for kn, v in per.items():
            avg = sum(v) / len(v)
            ent = {"avg_us": round(avg * 1e3, 1), "launches": len(v) // steps}
            if kn in alg:
                ent["algorithmic_MB"] = round(alg[kn] / 1e6, 1)
                ent["GBs"] = round(alg[kn] / (avg * 1e-3) / 1e9, 1)
                ent["frac_hbm_peak"] = round(alg[kn] / (avg * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)
            out["kernels"][kn] = ent
    return out


def run_graph_bench(moe, W, steps):
    """The launch-bound end of the range: the tiny workload's whole step (about 20 kernels) issued call by call and
    replayed as one captured HIP graph."""
    import torch
    wl = W.WORKLOADS["tiny"]
    inp = W.make_layer_inputs(wl, seed=0)
    s = moe.Shape.of(wl.shape)
    x, dout = dev_bf16(inp["x"]), dev_bf16(inp["dout"])
    wg, wu, wd = dev_bf16(inp["w_gate"]), dev_bf16(inp["w_up"]), dev_bf16(inp["w_down"])
    logits = torch.from_numpy(inp["logits"]).cuda()
    buf = moe.MoeLayerBuffers(s)

    def eager():
        moe.layer_forward(buf, x, wg, wu, wd, logits)
        moe.layer_backward(buf, dout, wg, wu, wd)

    step = moe.CapturedLayerStep(buf, x, dout, wg, wu, wd, logits=logits)
    out = {"workload": wl.name}
    for label, fn in (("eager_ms", eager), ("graph_ms", step.replay)):
        for _ in range(5):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        out[label] = round(e0.elapsed_time(e1) / steps, 4)
    return out


def run_halo_bench(moe, steps):
    """The three single-GPU steps of the hierarchical all-to-all on an 8-node x 8-rank layout with 8 MiB per
    destination (512 MiB send buffer: larger than the last-level cache), two rotating buffer sets."""
    import torch
    nodes, R, row = 8, 8, 8 << 20
    M = nodes - 1
    sets = []
    for _ in range(2):
        sets.append(dict(S=torch.empty(nodes * R * row, dtype=torch.uint8, device="cuda").random_(0, 255),
                         F2=torch.empty(M * R * row, dtype=torch.uint8, device="cuda").random_(0, 255),
                         F3=torch.empty(M * R * row, dtype=torch.uint8, device="cuda"),
                         P1=torch.empty(R * row, dtype=torch.uint8, device="cuda").random_(0, 255),
                         O=torch.empty(nodes * R * row, dtype=torch.uint8, device="cuda")))
    calls = {"halo_pack_remote": (lambda b: moe.moe_halo_pack_remote(b["S"], b["F3"], nodes, R, 3), 2 * M * R * row),
             "halo_repack": (lambda b: moe.moe_halo_repack(b["F2"], b["F3"], M, R), 2 * M * R * row),
             "halo_unpack": (lambda b: moe.moe_halo_unpack(b["P1"], b["F2"], b["O"], nodes, R, 3), 2 * nodes * R * row)}
    out = {"layout": "8 nodes x 8 ranks, 8 MiB per destination", "peak_GBs": PEAK_HBM_GBS, "kernels": {}}
    for name, (fn, nbytes) in calls.items():
        for i in range(2):
            fn(sets[i])
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(steps):
            fn(sets[i % 2])
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / steps
        out["kernels"][name] = {"avg_us": round(ms * 1e3, 1), "algorithmic_MB": round(nbytes / 1e6, 1),
                                "GBs": round(nbytes / (ms * 1e-3) / 1e9, 1), "frac_hbm_peak": round(nbytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)}
    del sets
    torch.cuda.empty_cache()
    return out


def run_calibration():
    """What plain streaming reaches on this machine (torch is only the allocator here, but its copy and fill are the simplest
    yard sticks at hand): a 512 MiB device-to-device copy (also the
    reference the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run are scaled by) and a 512 MiB fill (write
    only), each 5 launches."""
    import torch
    n = 512 * 1024 * 1024
    a = torch.empty(n, dtype=torch.uint8, device="cuda").fill_(3)
    b = torch.empty_like(a)
    torch.cuda.synchronize()

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            fn()
        e1.record()
        e1.synchronize()
        return e0.elapsed_time(e1) / 5
    t_copy, t_fill = timed(lambda: b.copy_(a)), timed(lambda: b.fill_(1))
    gbs = lambda nbytes, ms: round(nbytes / (ms * 1e-3) / 1e9, 1)  # noqa: E731
    return {"bytes": n, "launches": 5,
            "copy": {"avg_us": round(t_copy * 1e3, 1), "GBs_read_plus_write": gbs(2 * n, t_copy), "frac_hbm_peak": round(gbs(2 * n, t_copy) / PEAK_HBM_GBS, 4)},
            "fill": {"avg_us": round(t_fill * 1e3, 1), "GBs_written": gbs(n, t_fill), "frac_hbm_peak": round(gbs(n, t_fill) / PEAK_HBM_GBS, 4)}}


def run_cpu_baseline(W, inp, sh, sample_tokens):
    """The fp64 oracle, as it stands, on the first `sample_tokens` tokens of the same workload (all experts, same
    routing): forward + backward of the per-token definition.  Rate = algorithmic FLOPs of the sample / wall time."""
    import numpy as np
    from oracle import moe_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    f = W.bf16_bits_to_f32
    n = min(sample_tokens, sh.T)
    x, dout = f(inp["x"][:n]), f(inp["dout"][:n])
    if "logits" in inp:
        idx, w, _ = O.route_topk(inp["logits"][:n], sh.k, sh.E_shared, True)
    else:
        idx, w = inp["topk_idx"][:n], inp["topk_w"][:n].astype(np.float64)
    t0 = time.perf_counter()
    wg, wu, wd = f(inp["w_gate"]), f(inp["w_up"]), f(inp["w_down"])
    out, _ = O.layer_forward(x, idx, w, wg, wu, wd)
    g = O.layer_backward(x, idx, w, wg, wu, wd, dout)
    dt = time.perf_counter() - t0
    flops = 18.0 * sh.d_model * sh.d_ffn * n * sh.K_slots
    return {"value": round(flops / dt / 1e12, 5), "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
            "sample": f"fp64 NumPy oracle fwd+bwd on the first {n} of {sh.T} tokens of the same workload "
                      f"(all {sh.E_total} experts, {n * sh.K_slots} slots, {flops / 1e12:.3f} TFLOP) in {dt:.1f} s",
            "seconds": round(dt, 2)}


def main():
    args = parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py measures one GPU's MoE expert layer; this build has no multi-GPU path "
              "(run with --gpus 1).", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2605_05049_amd as moe
    import workloads as W
    moe.load_library()      # raises if the HIP library is missing: no fallback
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)

    inp, sh, elapsed, kernels, gen_s, split, load = run_layer_bench(moe, W, args)
    flops = sh.flops_fwd_bwd()
    ms_per_step = elapsed / args.steps * 1e3
    tflops = flops / (ms_per_step * 1e-3) / 1e12

    # roofline of the dominant kernel (largest total time per step)
    dom = max(kernels, key=lambda k: kernels[k]["avg_ms"] * kernels[k]["launches_per_step"])
    dom_flops = gemm_flops_per_launch(dom, sh)
    if dom_flops:
        roofline = gemm_roofline(dom, sh, load["experts_with_rows"], kernels[dom]["avg_ms"])
        roofline.update({"traffic": measured_traffic_bytes(args.workload).get(dom), "kernel": dom,
                         "avg_ms": round(kernels[dom]["avg_ms"], 4), "flops_per_launch": dom_flops,
                         "bytes_per_launch": gemm_bytes_per_launch(dom, sh, load["experts_with_rows"])})
    else:
        b = stream_bytes_per_launch(dom, sh) or 0
        ach = b / (kernels[dom]["avg_ms"] * 1e-3) / 1e9
        roofline = {"bound": "hbm", "achieved": round(ach, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": round(ach / PEAK_HBM_GBS, 4), "traffic": None, "kernel": dom,
                    "avg_ms": round(kernels[dom]["avg_ms"], 4)}
    kern_out = {}
    for k, v in sorted(kernels.items(), key=lambda kv: -kv[1]["avg_ms"] * kv[1]["launches_per_step"]):
        ent = {"avg_ms": round(v["avg_ms"], 4), "launches_per_step": v["launches_per_step"]}
        fl = gemm_flops_per_launch(k, sh)
        if fl:
            ent["TFLOPs"] = round(fl / (v["avg_ms"] * 1e-3) / 1e12, 1)
            ent["frac_mfma_peak"] = round(ent["TFLOPs"] / PEAK_BF16_MFMA_TFLOPS, 4)
            r = gemm_roofline(k, sh, load["experts_with_rows"], v["avg_ms"])
            ent["bound"], ent["frac_of_bound"] = r["bound"], r["frac"]
        kern_out[k] = ent

    res = {
        "metric": "MoE layer fwd+bwd TFLOP/s", "value": round(tflops, 2), "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.workload}: T={sh.T} d_model={sh.d_model} d_ffn={sh.d_ffn} E={sh.E}"
                               f"+{sh.E_shared} shared top-{sh.k} (N={sh.N} rows), fwd+bwd, seed {args.seed}",
                   "flops_per_step": flops},
        "frac_bf16_mfma_peak": round(tflops / PEAK_BF16_MFMA_TFLOPS, 4),
        "roofline": roofline,
        "rows_per_expert": load,
        "phases": split,
        "kernels": kern_out,
    }
    if not args.no_streaming:
        res["permute_combine"] = run_streaming_bench(moe, W, steps=20)
    if not args.no_streaming and args.workload != "shard":
        res["router"] = run_router_bench(moe, W, args.workload, steps=20)
    if not args.no_streaming and args.workload == "mixtral":
        res["halo_pack"] = run_halo_bench(moe, steps=10)
        res["graph_replay"] = run_graph_bench(moe, W, steps=200)
    if not args.no_streaming and args.workload == "mixtral":
        res["router_imbalance"] = run_router_bench(moe, W, "imbalance", steps=20)
    if not args.no_workloads and args.workload == "mixtral":
        res["workloads"] = {name: run_workload_brief(moe, W, name, steps=5, seed=args.seed)
                            for name in ("finegrained", "shard", "imbalance")}
    if not args.no_calibration:
        res["calibration"] = run_calibration()
    if not args.no_cpu_baseline:
        n = args.cpu_sample_tokens
        if n <= 0:
            # about 10-30 s of fp64 work: ~1 TFLOP at the ~50-100 GFLOP/s the host cores give NumPy
            per_token = 18.0 * sh.d_model * sh.d_ffn * sh.K_slots
            n = int(max(16, min(sh.T, 1.0e12 / per_token)))
        res["cpu_baseline"] = run_cpu_baseline(W, inp, sh, n)
    res["input_generation_s"] = round(gen_s, 1)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
