"""Expert-GEMM throughput sweep over (tokens per expert, expert dimensions, number of experts, imbalance): the
paper's "MoE GEMM Performance" micro-benchmark (Section IV, the expert-GEMM throughput study that feeds its
estimator), run through this library's grouped FFN entry points on one MI355X.

    python -m paper_2605_05049_amd.sweep [--tokens 128,512,2048] [--dims 4096x14336,2048x1408] [--experts 8]
                                         [--imbalance uniform,zipf] [--steps 5]

One JSON line per point: forward, backward and forward+backward TFLOP/s of the grouped FFN (18*d*f FLOP per row;
rows of padding are never counted) and the per-kernel times.  Inputs are random bf16 tensors made on the device;
`tokens` is the mean number of rows per expert, `zipf` draws the per-expert row counts from a Zipf(1.2) law with
the same total.  Only marshals arguments and times: every computation is a C-ABI call.
"""
from __future__ import annotations

import argparse
import json
import sys


def expert_counts(n_experts: int, mean_rows: int, kind: str, seed: int):
    import numpy as np
    total = n_experts * mean_rows
    if kind == "uniform":
        return np.full(n_experts, mean_rows, dtype=np.int64)
    if kind == "zipf":
        rng = np.random.default_rng(seed)
        p = 1.0 / np.arange(1, n_experts + 1, dtype=np.float64) ** 1.2
        p = rng.permutation(p / p.sum())
        c = np.floor(p * total).astype(np.int64)
        c[np.argmax(c)] += total - c.sum()
        return c
    raise ValueError(kind)


def run_point(moe, d, f, n_experts, mean_rows, kind, steps, seed=0):
    import torch
    counts = expert_counts(n_experts, mean_rows, kind, seed)
    N = int(counts.sum())
    # the shape's T*k only sizes the buffers here: rows enter at the grouped FFN, already grouped by expert
    s = moe.Shape(N, d, f, n_experts, 1)
    offsets = torch.zeros(n_experts + 1, dtype=torch.int32)
    offsets[1:] = torch.from_numpy(counts).cumsum(0).to(torch.int32)
    offsets = offsets.cuda()
    g = torch.Generator(device="cuda").manual_seed(seed)
    rnd = lambda *sz, std=1.0: (torch.randn(*sz, device="cuda", generator=g) * std).to(torch.bfloat16)  # noqa: E731
    x, dy = rnd(N, d), rnd(N, d)
    wg, wu, wd = rnd(n_experts, d, f, std=0.02), rnd(n_experts, d, f, std=0.02), rnd(n_experts, f, d, std=0.02)
    y = torch.empty(N, d, dtype=torch.bfloat16, device="cuda")
    sg = torch.empty(N, f, dtype=torch.bfloat16, device="cuda")
    su = torch.empty_like(sg)
    dx = torch.empty_like(y)
    dwg = torch.empty(n_experts, d, f, dtype=torch.float32, device="cuda")
    dwu = torch.empty_like(dwg)
    dwd = torch.empty(n_experts, f, d, dtype=torch.float32, device="cuda")
    ws = torch.empty(moe.workspace_bytes(s), dtype=torch.uint8, device="cuda")

    def fwd():
        moe.moe_grouped_ffn_fwd(s, x, offsets, wg, wu, wd, y, sg, su, ws)

    def bwd():
        moe.moe_grouped_ffn_bwd(s, dy, x, offsets, wg, wu, wd, sg, su, dx, dwg, dwu, dwd, 0, ws)

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / steps

    fwd()
    t_f, t_b = timed(fwd), timed(bwd)
    moe.profile_reset()
    moe.profile_enable(True)
    fwd()
    bwd()
    torch.cuda.synchronize()
    moe.profile_enable(False)
    kern = {name: round(ms * 1e3, 1) for name, ms in moe.profile_records() if name.startswith("ffn_") and name != "ffn_schedule"}
    moe.profile_reset()
    unit = 2.0 * d * f * N
    return {"d_model": d, "d_ffn": f, "experts": n_experts, "mean_rows_per_expert": mean_rows, "imbalance": kind,
            "rows": N, "max_rows": int(counts.max()), "min_rows": int(counts.min()),
            "fwd_ms": round(t_f, 4), "bwd_ms": round(t_b, 4),
            "fwd_TFLOPs": round(3 * unit / (t_f * 1e-3) / 1e12, 1), "bwd_TFLOPs": round(6 * unit / (t_b * 1e-3) / 1e12, 1),
            "fwd_bwd_TFLOPs": round(9 * unit / ((t_f + t_b) * 1e-3) / 1e12, 1), "kernel_us": kern}


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--tokens", default="64,256,1024,4096", help="mean rows per expert, comma separated")
    ap.add_argument("--dims", default="4096x14336,2048x1408,7168x2048", help="d_model x d_ffn pairs")
    ap.add_argument("--experts", default="8", help="experts per point, comma separated")
    ap.add_argument("--imbalance", default="uniform,zipf")
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--max-gb", type=float, default=40.0, help="skip points whose tensors would exceed this")
    args = ap.parse_args(argv)
    import torch
    from . import binding as moe
    moe.load_library()
    if not torch.cuda.is_available():
        print("the sweep needs a GPU", file=sys.stderr)
        return 2
    for dim in args.dims.split(","):
        d, f = (int(v) for v in dim.lower().split("x"))
        for ne in (int(v) for v in args.experts.split(",")):
            for rows in (int(v) for v in args.tokens.split(",")):
                gb = (ne * d * f * (3 * 2 + 3 * 4) + ne * rows * (4 * d + 5 * f) * 2) / 1e9
                if gb > args.max_gb:
                    continue
                for kind in args.imbalance.split(","):
                    print(json.dumps(run_point(moe, d, f, ne, rows, kind, args.steps)), flush=True)
                    torch.cuda.empty_cache()
    return 0


if __name__ == "__main__":
    sys.exit(main())
