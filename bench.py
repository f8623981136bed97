#!/usr/bin/env python3
"""Benchmark of the EasyQuant quantization hot path on one MI355X.

One "step" = one eq_quantize_batch call over a whole synthetic LLaMA-shaped weight set that
is already resident in HBM (outlier isolation, all range-optimisation iterations, packed
codes, scales, zero-points and the sorted outlier list for every matrix).

Prints ONE JSON line: metric = GB/s of 16-bit weights quantized (and seconds per model), a
`roofline` object for the dominant kernel and a `cpu_baseline` object (the CPU oracle timed
on a bounded sample of the same workload on this machine's host cores).
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

HBM_PEAK = 8.0e12                               # B/s, MI355X HBM3E
ALU_PEAK = 256 * 4 * 16 * 2.4e9                 # lane-operations/s: 256 CUs x 4 SIMD x 16 lanes x 2.4 GHz

WORKLOADS = {
    # name: (model shapes, recipe key, 16-bit type, bits, note)
    "llama65b_f16_w4g128": ("llama65b", "c5", "f16", 4),
    "llama7b_bf16_w4g128": ("llama7b", "c4", "bf16", 4),
}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def build_workload(name, layers, device):
    import torch
    import eq_inputs
    which, rkey, dt, bits = WORKLOADS[name]
    recipe = eq_inputs.with_dtype(eq_inputs.RECIPES[rkey], dt)
    Ws, names = [], []
    t0 = time.time()
    for layer, nm, W in eq_inputs.iter_model(which, recipe, device, base_seed=0, layers=layers):
        Ws.append(W)
        names.append((layer, nm))
        if nm == "down":
            torch.cuda.synchronize()
            log(f"[gen] layer {layer} done, {sum(w.numel() for w in Ws) * 2 / 1e9:.1f} GB resident, {time.time() - t0:.0f}s")
    return Ws, names, bits, dt


def algorithmic_bytes(Ws, bits, n_outliers, group_size=128):
    """HBM bytes the path must move: read W once; write codes, scale + zero-point, outliers (col + value) and row_ptr."""
    elems = sum(w.numel() for w in Ws)
    rows = sum(w.shape[0] for w in Ws)
    units = elems // group_size if group_size else rows
    return elems * 2 + elems * bits // 8 + units * 5 + n_outliers * 6 + (rows + len(Ws)) * 4


def measured_traffic(workload, iters, kernel="quantize_units128"):
    """HBM bytes per step of the main kernels from the committed counter summary (rocprofv3 --pmc
    FETCH_SIZE / WRITE_SIZE, scaled by a copy of known size), if one exists for this workload."""
    path = os.path.join(ROOT, "profiles", f"{kernel}_{workload}_hbm_traffic.txt")
    if workload is None or not os.path.exists(path):
        return None
    vals = {}
    for line in open(path):
        if "=" in line and not line.startswith("#"):
            k, v = line.split("=", 1)
            vals[k.strip()] = v.strip()
    try:
        if int(vals.get("iters", -1)) != iters:
            return None
        return float(vals["fetch_bytes_per_step"]) + float(vals["write_bytes_per_step"])
    except (KeyError, ValueError):
        return None


def cpu_baseline(Ws, gp_kwargs, sample_rows):
    """The oracle, as it stands, on the first `sample_rows` rows of the first matrix."""
    import numpy as np
    from oracle import easyquant_oracle as eqo
    W = Ws[0][:sample_rows]
    raw = W.cpu().contiguous().view(__import__("torch").int16).numpy().view(np.uint16)
    p = eqo.Params(**gp_kwargs)
    t0 = time.perf_counter()
    eqo.quantize_matrix(raw, p)
    dt = time.perf_counter() - t0
    return raw.size * 2 / dt / 1e9, dt, raw.shape


def bench_dequantize(args):
    """Secondary measurement: eq_dequantize (Eq. 4) on the shape of the paper's latency paragraph
    (the first FFN layer of BLOOM-176B, 14336 x 57344; the paper prints 14336 x 53746), 4-bit,
    per-channel, with synthetic outlier lists of the ratios of the paper's Table 4."""
    import torch
    import paper_2403_02775_amd as eqg
    dev = "cuda:0"
    rows, cols = 14336, 57344
    G = args.matvec_group                            # 0: one range per row (the paper's setting)
    upr = cols // G if G else 1
    gp = eqg.Params(dtype=eqg.EQ_F16, bits=4, group_size=G)
    g = torch.Generator(device=dev)
    g.manual_seed(0)
    codes = torch.randint(-2 ** 31, 2 ** 31 - 1, (rows, cols * 4 // 32), dtype=torch.int32, device=dev, generator=g)
    scales = torch.rand((rows, upr), device=dev, generator=g) * 0.01 + 0.001
    zps = torch.full((rows, upr), 7, dtype=torch.uint8, device=dev)
    out = torch.empty((rows, cols), dtype=torch.float16, device=dev)
    res = {}
    for ratio in (0.0, 1e-4, 1e-3, 5e-3, 1e-2, 5e-2, 1e-1):
        k = int(round(cols * ratio))
        col = torch.randint(cols, (rows, max(k, 1)), device=dev, generator=g, dtype=torch.int32)[:, :k].sort(dim=1).values.contiguous()
        rp = (torch.arange(rows + 1, device=dev, dtype=torch.int64) * k).to(torch.int32)
        q = eqg.QMatrix(codes=codes, scales=scales, zero_points=zps, out_row_ptr=rp, out_col=col.view(-1),
                        out_val=torch.zeros(rows * k, dtype=torch.int16, device=dev), status=torch.zeros(1, dtype=torch.int32, device=dev))
        for _ in range(2):
            eqg.eq_dequantize(q, rows, cols, gp, out)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            eqg.eq_dequantize(q, rows, cols, gp, out)
        e1.record()
        torch.cuda.synchronize()
        res[f"{ratio:.4%}"] = e0.elapsed_time(e1) / args.steps
    dense_ms = res["0.0000%"]
    traffic = rows * cols * 2.5 + rows * upr * 5
    print(json.dumps({"metric": "eq_dequantize ms (14336x57344, int4 -> fp16, %s)" % ("one range per row" if not G else "groups of %d" % G),
                      "value": dense_ms, "unit": "ms",
                      "n_gpus": 1, "steps": args.steps, "higher_is_better": False, "data": "synthetic",
                      "dense_GBps": traffic / (dense_ms * 1e-3) / 1e9, "dense_hbm_frac": traffic / (dense_ms * 1e-3) / HBM_PEAK,
                      "outlier_overhead_ms": {k: v - dense_ms for k, v in res.items() if k != "0.0000%"},
                      "paper_context_A100": {"dequant_ms": 5.0, "outlier_ms": {"0.01%": 0.027, "0.10%": 0.055, "0.50%": 0.093,
                                                                           "1%": 0.117, "5%": 0.186, "10%": 0.212}}}), flush=True)


def bench_matvec(args):
    """Secondary measurement: eq_dequant_matvec (Eq. 4 fused with a matrix-vector product) on the
    same BLOOM-176B FFN shape, 4-bit per-channel, 1 % outliers, against torch's fp16 matrix-vector
    product on the dequantized matrix (which reads 2 bytes per weight)."""
    import torch
    import paper_2403_02775_amd as eqg
    dev = "cuda:0"
    rows, cols = 14336, 57344
    G = args.matvec_group                            # 0: one range per row (the paper's setting)
    upr = cols // G if G else 1
    gp = eqg.Params(dtype=eqg.EQ_F16, bits=4, group_size=G)
    g = torch.Generator(device=dev)
    g.manual_seed(0)
    codes = torch.randint(-2 ** 31, 2 ** 31 - 1, (rows, cols * 4 // 32), dtype=torch.int32, device=dev, generator=g)
    scales = torch.rand((rows, upr), device=dev, generator=g) * 0.01 + 0.001
    zps = torch.full((rows, upr), 7, dtype=torch.uint8, device=dev)
    k = max(1, int(round(cols * args.outlier_pct / 100.0)))
    stride = cols // k                              # one outlier in every stride-wide stretch: ascending, no duplicates
    col = (torch.arange(k, device=dev, dtype=torch.int32) * stride).view(1, -1) + \
        torch.randint(stride, (rows, k), device=dev, generator=g, dtype=torch.int32)
    col = col.contiguous()
    rp = (torch.arange(rows + 1, device=dev, dtype=torch.int64) * k).to(torch.int32)
    # the format's invariant: an outlier's slot holds the zero level (code = zero-point)
    by = codes.view(torch.uint8).view(rows, cols // 2)
    rr = torch.arange(rows, device=dev).view(-1, 1).expand(-1, k)
    cl = col.long()
    for nib, keep, put in ((0, 0xF0, 0x07), (1, 0x0F, 0x70)):
        m = (cl % 2) == nib
        r_, b_ = rr[m], cl[m] // 2
        by[r_, b_] = (by[r_, b_] & keep) | put
    vals = (torch.randn(rows * k, device=dev, generator=g) * 0.3).half().view(torch.int16)
    q = eqg.QMatrix(codes=codes, scales=scales, zero_points=zps, out_row_ptr=rp, out_col=col.view(-1),
                    out_val=vals, status=torch.zeros(1, dtype=torch.int32, device=dev))
    x = torch.randn(cols, device=dev, generator=g).half()
    y = torch.empty(rows, dtype=torch.float32, device=dev)
    W = torch.empty((rows, cols), dtype=torch.float16, device=dev)
    eqg.eq_dequantize(q, rows, cols, gp, W)

    def timed(fn):
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / args.steps

    fused_ms = timed(lambda: eqg.eq_dequant_matvec(q, rows, cols, gp, x, y))
    dense_ms = timed(lambda: torch.mv(W, x))
    y_ref = torch.mv(W.float(), x.float())
    rel = float((y - y_ref).abs().max() / y_ref.abs().max())
    traffic = rows * cols * 0.5 + rows * upr * 5 + rows * 4 + rows * k * 6 + cols * 2
    print(json.dumps({"metric": f"eq_dequant_matvec ms (14336x57344, int4 x fp16 vector, {args.outlier_pct:g} % outliers, "
                                f"{'one range per row' if not G else 'groups of %d' % G})", "value": fused_ms, "unit": "ms",
                      "n_gpus": 1, "steps": args.steps, "higher_is_better": False, "data": "synthetic",
                      "GBps": traffic / (fused_ms * 1e-3) / 1e9, "hbm_frac": traffic / (fused_ms * 1e-3) / HBM_PEAK,
                      "torch_fp16_mv_on_dequantized_ms": dense_ms, "speedup_vs_fp16_mv": dense_ms / fused_ms,
                      "max_rel_diff_vs_fp32_mv": rel}), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="llama65b_f16_w4g128", choices=sorted(WORKLOADS))
    ap.add_argument("--layers", type=int, default=-1, help="limit the number of layers (debugging; changes the workload)")
    ap.add_argument("--iters", type=int, default=100, help="Adam steps T on the range")
    ap.add_argument("--lr", type=float, default=1e-3)
    ap.add_argument("--bits", type=int, default=0, help="code width (default: the workload's, 4)")
    ap.add_argument("--group-size", type=int, default=128, help="0 = one range per output channel (secondary measurement)")
    ap.add_argument("--stat-scope", choices=["row", "matrix"], default="row",
                    help="scope of mean / sigma in the outlier criterion; matrix = Eq. 3 as printed (secondary measurement)")
    ap.add_argument("--select", choices=["best", "last"], default="best",
                    help="which iterate is kept; last = the paper's wording (secondary measurement)")
    ap.add_argument("--capacity-frac", type=float, default=0.02, help="outlier capacity per matrix as a fraction of its elements")
    ap.add_argument("--cpu-rows", type=int, default=3072, help="rows of the first matrix given to the CPU oracle (0 = skip)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 4 GiB device-to-device copy (torch's copy kernel) so that a counter run "
                         "(rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE) has a kernel of known traffic to scale by")
    ap.add_argument("--dequant", action="store_true", help="measure eq_dequantize instead (secondary benchmark, own JSON line)")
    ap.add_argument("--outlier-pct", type=float, default=1.0, help="outlier ratio in percent for --matvec")
    ap.add_argument("--matvec-group", type=int, default=0, help="group size for --dequant and --matvec (0 = one range per row)")
    ap.add_argument("--matvec", action="store_true", help="measure eq_dequant_matvec instead (secondary benchmark, own JSON line)")
    args = ap.parse_args()
    if args.dequant:
        return bench_dequantize(args)
    if args.matvec:
        return bench_matvec(args)
    if args.gpus != 1:
        sys.exit("bench.py: this build measures one GPU only (matrices, rows and groups are independent: the path needs no communication between GPUs); run with --gpus 1")

    import torch
    import paper_2403_02775_amd as eqg

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    torch.cuda.set_device(0)
    Ws, names, bits, dt = build_workload(args.workload, args.layers, dev)
    if args.bits:
        bits = args.bits
    gp = eqg.Params(dtype=eqg.EQ_F16 if dt == "f16" else eqg.EQ_BF16, bits=bits, group_size=args.group_size, mode=eqg.EQ_SYMMETRIC,
                    stat_scope=eqg.EQ_STAT_ROW if args.stat_scope == "row" else eqg.EQ_STAT_MATRIX, n_sigma=3.0,
                    iters=args.iters, lr=args.lr, select=eqg.EQ_SELECT_BEST if args.select == "best" else eqg.EQ_SELECT_LAST)
    caps = [int(w.numel() * args.capacity_frac) for w in Ws]
    outs = [eqg.alloc_outputs(w.shape[0], w.shape[1], gp, c, dev) for w, c in zip(Ws, caps)]
    ws_bytes = eqg.eq_workspace_bytes([w.shape[0] for w in Ws], [w.shape[1] for w in Ws], caps, gp)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()
    log(f"[mem] inputs {sum(w.numel() for w in Ws) * 2 / 1e9:.1f} GB, workspace {ws_bytes / 1e9:.1f} GB, "
        f"allocated {torch.cuda.memory_allocated() / 1e9:.1f} GB")

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.int32, device=dev).fill_(7)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        log("[calibration] copied 4 GiB (reads 4 GiB, writes 4 GiB)")
        del src, dst

    def step():
        eqg.eq_quantize_batch(Ws, gp, outs, ws)

    for i in range(args.warmup):
        step()
        torch.cuda.synchronize()
        log(f"[warmup] {i + 1}/{args.warmup}")
    eqg.eq_profile_enable(True)
    eqg.eq_profile_read()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev0.record()
    for _ in range(args.steps):
        step()
    ev1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    gpu_ms = ev0.elapsed_time(ev1)
    kern_ms, launches = eqg.eq_profile_read()
    eqg.eq_profile_enable(False)

    status = [int(o.status.item()) for o in outs]
    assert not any(status), f"device status words: {sorted(set(status))}"
    n_out = sum(int(o.out_row_ptr[-1].item()) & 0xFFFFFFFF for o in outs)
    elems = sum(w.numel() for w in Ws)
    ms_per_step = gpu_ms / args.steps
    weight_gbs = elems * 2 / (ms_per_step * 1e-3) / 1e9
    # T evaluations, one more for best-iterate selection, and the emitting pass
    passes = (args.iters + (2 if args.select == "best" else 1)) if args.iters else 1
    lane_ops = elems * (5 * passes + 12)          # useful lane-operations: 5 per element and pass, 12 fixed
    kern_s = kern_ms * 1e-3 / args.steps          # main kernels per step (one launch per row-length class)
    alg_bytes = algorithmic_bytes(Ws, bits, n_out, args.group_size)
    alu_frac = lane_ops / kern_s / ALU_PEAK
    hbm_frac = alg_bytes / kern_s / HBM_PEAK
    if alu_frac >= hbm_frac:
        roof = {"bound": "alu", "achieved": lane_ops / kern_s / 1e12, "peak": ALU_PEAK / 1e12, "unit": "Tlaneop/s",
                "frac": alu_frac, "traffic": None}
    else:
        roof = {"bound": "hbm", "achieved": alg_bytes / kern_s / 1e9, "peak": HBM_PEAK / 1e9, "unit": "GB/s",
                "frac": hbm_frac, "traffic": None}
    kernel = "quantize_rtn128" if args.group_size == 128 and args.iters == 0 else "quantize_units128" if args.group_size == 128 else "quantize_channels" if args.group_size == 0 else "quantize_rows_generic"
    roof["traffic"] = measured_traffic(args.workload if args.layers < 0 else None, args.iters, kernel)
    roof.update({"kernel": kernel, "launches_per_step": launches / args.steps,
                 "kernel_ms_per_step": kern_ms / args.steps, "avg_launch_ms": kern_ms / max(launches, 1),
                 "algorithmic_bytes": alg_bytes, "hbm_frac": hbm_frac, "alu_frac": alu_frac,
                 "lane_ops_per_element": 5 * passes + 12})

    out = {
        "metric": "fp16 weight GB/s quantized (fraction of HBM peak); s per 65B-shaped model",
        "value": weight_gbs, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32",                              # levels in binary32; the sums are exact integers, the recurrence binary64
        "data": "synthetic",
        "config": {"workload": args.workload + ("" if args.layers < 0 else f"[first {args.layers} layers]"),
                   "matrices": len(Ws), "elements": elems, "bits": bits, "group_size": args.group_size, "mode": "symmetric",
                   "n_sigma": 3.0, "stat_scope": args.stat_scope, "iters": args.iters, "lr": args.lr, "select": args.select,
                   "weights_dtype": dt,
                   "parallelism": "1 GPU, one batch call"},
        "seconds_per_model": ms_per_step * 1e-3,
        "weight_hbm_frac": weight_gbs * 1e9 / HBM_PEAK,
        "outlier_fraction": n_out / elems,
        "wall_s_per_step": wall / args.steps,
        "roofline": roof,
    }
    if args.cpu_rows > 0 and args.stat_scope == "row":       # (a sample of rows has no whole-matrix statistics)
        kw = dict(dtype=gp.dtype, bits=bits, group_size=args.group_size, mode=0, stat_scope=0, n_sigma=3.0, iters=args.iters,
                  lr=args.lr, select=0 if args.select == "best" else 1)
        gbs, secs, shape = cpu_baseline(Ws, kw, args.cpu_rows)
        out["cpu_baseline"] = {"value": gbs, "unit": "GB/s", "cores": 1, "kind": "oracle",
                               "sample": f"first {shape[0]} rows x {shape[1]} cols of layer 0 q_proj ({secs:.1f} s, NumPy, "
                                         f"single thread; host has {os.cpu_count()} logical CPUs)",
                               "seconds_per_model_extrapolated": elems * 2 / (gbs * 1e9)}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
