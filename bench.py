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


def measured_issue(workload, iters, kernel="quantize_units128"):
    """Shader-sequencer figures of the main kernels from the committed counter summary (rocprofv3 --pmc
    SQ_*), if one exists for this workload and step count: VALU instructions per element, share of
    cycles in which the vector ALUs issue, and VALU issue slots used (wavefront instructions x 4
    cycles / SIMDs / busy cycles).  Read like `traffic`: a counter run cannot share the timed run."""
    path = os.path.join(ROOT, "profiles", f"{kernel}_{workload}_sq_issue.txt")
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
        return {k: float(vals[k]) for k in ("valu_insts_per_element", "valu_busy", "issue_frac")}
    except (KeyError, ValueError):
        return None


PAPER_CONTEXT = {
    # the paper's own wall-clock figures, other hardware: context, not a target
    "quantization": "1-10 min per model for every evaluated model (BLOOM up to 176B, LLaMA up to 65B), 4-bit, per channel, "
                    "100-500 Adam steps, 8 x A100, one weight per GPU (Sec. 5, Implementation)",
    "quantization_175B": "within 10 minutes (Abstract, Sec. 6)",
    "dequantization_A100_ms": {"int4_dequantize_14336x53746": 5.0, "fp16_matmul_bs1_seq1024": 83.0},
    "outlier_isolation_A100_ms_by_ratio": {"0.01%": 0.027, "0.10%": 0.055, "0.50%": 0.093, "1%": 0.117, "5%": 0.186,
                                           "10%": 0.212},
}


def cpu_baseline_start_pool(workers):
    """The oracle's worker processes; to be called before anything touches the GPU."""
    from oracle.rowpool import RowPool
    return RowPool(workers)


def cpu_baseline_pooled(pool, Ws, gp_kwargs, single_rows, pool_rows):
    """The oracle, as it stands, on the first rows of the first matrix: `single_rows` rows in this
    process (one thread), then `pool_rows` rows as blocks of 32 rows over the worker processes."""
    import numpy as np
    import torch
    from oracle import easyquant_oracle as eqo
    p = eqo.Params(**gp_kwargs)
    raw = Ws[0][:max(single_rows, pool_rows)].cpu().contiguous().view(torch.int16).numpy().view(np.uint16)
    t0 = time.perf_counter()
    for a in range(0, single_rows, 32):
        eqo.quantize_matrix(raw[a:a + 32], p)
    t_single = time.perf_counter() - t0
    t0 = time.perf_counter()
    pool.quantize_blocks([raw[a:a + 32] for a in range(0, pool_rows, 32)], p, keep=("scales",))
    t_pool = time.perf_counter() - t0
    cols = raw.shape[1]
    return {"single_GBps": single_rows * cols * 2 / t_single / 1e9, "single_s": t_single,
            "pool_GBps": pool_rows * cols * 2 / t_pool / 1e9, "pool_s": t_pool, "cols": cols}


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
    if args.matvec_lookup:
        eqg.set_override(eqg.OVR_MATVEC_LOOKUP, args.matvec_lookup)
    g = torch.Generator(device=dev)
    g.manual_seed(0)
    codes = torch.randint(-2 ** 31, 2 ** 31 - 1, (rows, cols * 4 // 32), dtype=torch.int32, device=dev, generator=g)
    scales = torch.rand((rows, upr), device=dev, generator=g) * 0.01 + 0.001
    zps = torch.full((rows, upr), 7, dtype=torch.uint8, device=dev)
    k = int(round(cols * args.outlier_pct / 100.0)) if args.outlier_pct > 0 else 0   # 0: no outlier list at all
    k = max(1, k) if args.outlier_pct > 0 else 0
    stride = cols // max(k, 1)                      # one outlier in every stride-wide stretch: ascending, no duplicates
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
    ap.add_argument("--channel-evaluation", choices=["auto", "direct", "sorted"], default="auto",
                    help="rows with one range each (--group-size 0): element-by-element kernels, or the evaluation from sorted rows "
                         "(auto: the library's choice, sorted from 60 to 65 steps on for rows of 8192 and longer)")
    ap.add_argument("--class-streams", choices=["auto", "sequential"], default="auto",
                    help="sequential: the row-length classes of a batch one after the other also without optimisation steps "
                         "(auto: side by side then), so that per-kernel counters and durations do not overlap")
    ap.add_argument("--stat-scope", choices=["row", "matrix"], default="row",
                    help="scope of mean / sigma in the outlier criterion; matrix = Eq. 3 as printed (secondary measurement)")
    ap.add_argument("--select", choices=["best", "last"], default="best",
                    help="which iterate is kept; last = the paper's wording (secondary measurement)")
    ap.add_argument("--capacity-frac", type=float, default=0.02, help="outlier capacity per matrix as a fraction of its elements")
    ap.add_argument("--cpu-rows", type=int, default=1024,
                    help="rows of the first matrix the CPU oracle recomputes in one thread; the all-core sample is this "
                         "times half the number of worker processes (0 = skip)")
    ap.add_argument("--no-sweep", dest="sweep", action="store_false",
                    help="skip the secondary configurations timed after the headline (T = 0, 1, 10, 500; per channel)")
    ap.add_argument("--sweep-steps", type=int, default=3)
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 4 GiB device-to-device copy (torch's copy kernel) so that a counter run "
                         "(rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE) has a kernel of known traffic to scale by")
    ap.add_argument("--dequant", action="store_true", help="measure eq_dequantize instead (secondary benchmark, own JSON line)")
    ap.add_argument("--outlier-pct", type=float, default=1.0, help="outlier ratio in percent for --matvec")
    ap.add_argument("--matvec-group", type=int, default=0, help="group size for --dequant and --matvec (0 = one range per row)")
    ap.add_argument("--matvec-lookup", type=int, default=0,
                    help="measurement override for --matvec with one range per row: 1 = half of the weight pairs from the "
                         "table of pairs, half from the table of single values, 2 = table of single values only "
                         "(default 0: the library's choice, the table of pairs)")
    ap.add_argument("--matvec", action="store_true", help="measure eq_dequant_matvec instead (secondary benchmark, own JSON line)")
    args = ap.parse_args()
    if args.dequant:
        return bench_dequantize(args)
    if args.matvec:
        return bench_matvec(args)
    if args.gpus != 1:
        sys.exit("bench.py: this build measures one GPU only (matrices, rows and groups are independent: the path needs no communication between GPUs); run with --gpus 1")

    # The oracle's worker processes (the cpu_baseline leg) are started before anything touches the GPU.
    pool = None
    if args.cpu_rows > 0 and args.stat_scope == "row":
        pool = cpu_baseline_start_pool(min(16, os.cpu_count() or 1))
        log(f"[cpu] oracle pool of {pool.workers} worker processes")

    import torch
    import paper_2403_02775_amd as eqg

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    torch.cuda.set_device(0)
    Ws, names, bits, dt = build_workload(args.workload, args.layers, dev)
    if args.bits:
        bits = args.bits
    elems = sum(w.numel() for w in Ws)

    def params(iters, group_size, lr):
        return eqg.Params(dtype=eqg.EQ_F16 if dt == "f16" else eqg.EQ_BF16, bits=bits, group_size=group_size, mode=eqg.EQ_SYMMETRIC,
                          stat_scope=eqg.EQ_STAT_ROW if args.stat_scope == "row" else eqg.EQ_STAT_MATRIX, n_sigma=3.0,
                          iters=iters, lr=lr, select=eqg.EQ_SELECT_BEST if args.select == "best" else eqg.EQ_SELECT_LAST)

    gp = params(args.iters, args.group_size, args.lr)
    # secondary configurations timed on the same resident weights after the headline (the sweep of
    # step counts, and one range per output channel): (label, iters, group size, lr)
    sweep_cfgs = []
    if args.sweep and args.group_size == 128 and args.iters == 100:
        sweep_cfgs = [("T=0", 0, 128, args.lr), ("T=1", 1, 128, args.lr), ("T=10", 10, 128, args.lr),
                      ("T=500, lr=1e-4 (the paper's LLaMA setting)", 500, 128, 1e-4),
                      ("per channel, T=100 (the paper's granularity)", 100, 0, args.lr),
                      ("per channel, T=500, lr=1e-4 (the paper's LLaMA setting at its granularity)", 500, 0, 1e-4)]
    # test hooks of the library: same results, other kernels (set before the workspace is sized: it depends on them)
    if args.class_streams == "sequential":
        eqg.set_override(eqg.OVR_CLASS_STREAMS, 1)
    if args.channel_evaluation != "auto":
        eqg.set_override(eqg.OVR_SORTED_ROWS, 1 if args.channel_evaluation == "direct" else 2)
    caps = [int(w.numel() * args.capacity_frac) for w in Ws]
    outs = [eqg.alloc_outputs(w.shape[0], w.shape[1], gp, c, dev) for w, c in zip(Ws, caps)]
    shape_r, shape_c = [w.shape[0] for w in Ws], [w.shape[1] for w in Ws]
    ws_bytes = max(eqg.eq_workspace_bytes(shape_r, shape_c, caps, q)
                   for q in [gp] + [params(t, g, lr) for _, t, g, lr in sweep_cfgs])
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()
    log(f"[mem] inputs {elems * 2 / 1e9:.1f} GB, workspace {ws_bytes / 1e9:.1f} GB, "
        f"allocated {torch.cuda.memory_allocated() / 1e9:.1f} GB")

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.int32, device=dev).fill_(7)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        log("[calibration] copied 4 GiB (reads 4 GiB, writes 4 GiB)")
        del src, dst

    def kernel_name(q):
        # one range per row, at most 4 bits, steps x (columns - 960) >= 57 x columns (bf16: 80 x): Adam runs on the sorted rows
        # (sorted_prepare, sorted_iterate), the kernel without optimisation steps emits
        return ("quantize_rtn128" if q.iters == 0 and q.group_size in (0, 128) else "quantize_units128" if q.group_size == 128
                else ("sorted_rows" if args.channel_evaluation != "direct" and q.bits <= 4 and q.iters > 0 and
                      (q.iters * (max(w.shape[1] for w in Ws) - 960) >= (57 if dt == "f16" else 80) * max(w.shape[1] for w in Ws)
                       or args.channel_evaluation == "sorted")
                      else "quantize_channels") if q.group_size == 0
                else "quantize_rows_generic")

    def timed(q, q_outs, steps, warmup, label):
        """`steps` calls of eq_quantize_batch over the whole set; timing by events on the stream the
        calls are made on (torch's current stream); the main kernels are bracketed by the library."""
        for i in range(warmup):
            eqg.eq_quantize_batch(Ws, q, q_outs, ws)
            torch.cuda.synchronize()
            if warmup <= 5 or (i + 1) % 10 == 0:
                log(f"[warmup] {label} {i + 1}/{warmup}")
        eqg.eq_profile_enable(True)
        eqg.eq_profile_read()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ev0.record()
        for _ in range(steps):
            eqg.eq_quantize_batch(Ws, q, q_outs, ws)
        ev1.record()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        gpu_ms = ev0.elapsed_time(ev1)
        kern_ms, launches = eqg.eq_profile_read()
        eqg.eq_profile_enable(False)
        status = [int(o.status.item()) for o in q_outs]
        assert not any(status), f"device status words: {sorted(set(status))}"
        n_out = sum(int(o.out_row_ptr[-1].item()) & 0xFFFFFFFF for o in q_outs)
        ms_per_step = gpu_ms / steps
        # T evaluations, one more for best-iterate selection, and the emitting pass
        passes = (q.iters + (2 if args.select == "best" else 1)) if q.iters else 1
        lane_ops = elems * (5 * passes + 12)          # useful lane-operations: 5 per element and pass, 12 fixed
        kern_s = kern_ms * 1e-3 / steps               # main kernels per step (one launch per row-length class)
        alg_bytes = algorithmic_bytes(Ws, bits, n_out, q.group_size)
        return {"ms_per_step": ms_per_step, "wall_s_per_step": wall / steps, "kernel_ms_per_step": kern_ms / steps,
                "launches_per_step": launches / steps, "avg_launch_ms": kern_ms / max(launches, 1), "n_out": n_out,
                "passes": passes, "lane_ops": lane_ops, "alg_bytes": alg_bytes,
                "weight_GBps": elems * 2 / (ms_per_step * 1e-3) / 1e9,
                # whole step (every kernel of the call) against the two peaks
                "step_hbm_frac": alg_bytes / (ms_per_step * 1e-3) / HBM_PEAK,
                "step_useful_op_frac": lane_ops / (ms_per_step * 1e-3) / ALU_PEAK,
                # main kernels only
                "kernel_hbm_frac": alg_bytes / kern_s / HBM_PEAK, "kernel_useful_op_frac": lane_ops / kern_s / ALU_PEAK}

    m = timed(gp, outs, args.steps, args.warmup, "headline")
    ms_per_step, weight_gbs, n_out = m["ms_per_step"], m["weight_GBps"], m["n_out"]
    kern_s = m["kernel_ms_per_step"] * 1e-3
    kernel = kernel_name(gp)
    workload_key = args.workload if args.layers < 0 else None
    sq = measured_issue(workload_key, args.iters, kernel)
    # Without optimisation steps the useful-operation count (17 per element) overstates the kernel, which
    # issues 8.5 vector instructions per element at 43 % VALU busy: that end of the path is HBM-bound.
    if args.iters > 0 and m["kernel_useful_op_frac"] >= m["kernel_hbm_frac"]:
        # `frac` counts USEFUL lane-operations (5 per element and pass + 12, a definition fixed before the
        # kernel existed; the kernel issues about 4 per element and pass, so this can exceed what the issue
        # slots alone would allow); `issue_frac` is the measured share of VALU issue slots in use.
        roof = {"bound": "alu", "achieved": m["lane_ops"] / kern_s / 1e12, "peak": ALU_PEAK / 1e12, "unit": "Tlaneop/s",
                "frac": m["kernel_useful_op_frac"], "traffic": None}
    else:
        roof = {"bound": "hbm", "achieved": m["alg_bytes"] / kern_s / 1e9, "peak": HBM_PEAK / 1e9, "unit": "GB/s",
                "frac": m["kernel_hbm_frac"], "traffic": None}
    roof["traffic"] = measured_traffic(workload_key, args.iters, kernel)
    if kernel == "sorted_rows":
        # the lane-operations counted are those of an evaluation that visits every element in every pass; these
        # kernels take the sums from the sorted row, so the fraction compares with that evaluation at peak
        roof["note"] = ("frac = work of an element-by-element evaluation / time / ALU peak (can exceed 1: the sums come from "
                        "sorted rows); issue figures of the kernels: profiles/sorted_rows_*_sq_counters.txt")
    roof.update({"kernel": kernel, "launches_per_step": m["launches_per_step"],
                 "kernel_ms_per_step": m["kernel_ms_per_step"], "avg_launch_ms": m["avg_launch_ms"],
                 "algorithmic_bytes": m["alg_bytes"], "hbm_frac": m["kernel_hbm_frac"],
                 "useful_op_frac": m["kernel_useful_op_frac"], "lane_ops_per_element": 5 * m["passes"] + 12,
                 "issue_frac": sq["issue_frac"] if sq else None,
                 "valu_insts_per_element": sq["valu_insts_per_element"] if sq else None,
                 "valu_busy": sq["valu_busy"] if sq else None})

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
        "wall_s_per_step": m["wall_s_per_step"],
        "roofline": roof,
        "paper_context": PAPER_CONTEXT,
    }

    # ---- the sweep: same weights, same buffers, 3 timed steps each ----
    if sweep_cfgs:
        sweep = []
        chan_outs = None
        for label, iters, group, lr in sweep_cfgs:
            q = params(iters, group, lr)
            q_outs = outs
            if group == 0:                           # one scale and zero-point per row; everything else is shared
                if chan_outs is None:
                    chan_outs = [eqg.QMatrix(codes=o.codes, scales=torch.empty((w.shape[0], 1), dtype=torch.float32, device=dev),
                                             zero_points=torch.empty((w.shape[0], 1), dtype=torch.uint8, device=dev),
                                             out_row_ptr=o.out_row_ptr, out_col=o.out_col, out_val=o.out_val, status=o.status)
                                 for o, w in zip(outs, Ws)]
                q_outs = chan_outs
            # short steps need more of them: the first second or so of a configuration runs a few percent
            # slower than the steady state (clocks, address translation of 180 GB of buffers)
            n_steps, n_warm = (10 * args.sweep_steps, 30 if iters == 0 else 10) if iters <= 10 else (args.sweep_steps, 1)
            r = timed(q, q_outs, n_steps, n_warm, label)
            sweep.append({"config": label, "iters": iters, "group_size": group, "lr": lr, "steps": n_steps, "warmup": n_warm,
                          "ms_per_step": r["ms_per_step"], "seconds_per_model": r["ms_per_step"] * 1e-3,
                          "weight_GBps": r["weight_GBps"], "weight_hbm_frac": r["weight_GBps"] * 1e9 / HBM_PEAK,
                          "hbm_frac": r["step_hbm_frac"], "useful_op_frac": r["step_useful_op_frac"],
                          "bound": "hbm" if iters == 0 or r["step_hbm_frac"] >= r["step_useful_op_frac"] else "alu",
                          "kernel": kernel_name(q), "kernel_ms_per_step": r["kernel_ms_per_step"],
                          "kernel_hbm_frac": r["kernel_hbm_frac"], "algorithmic_bytes": r["alg_bytes"]})
            log(f"[sweep] {label}: {r['ms_per_step']:.2f} ms/step, {r['weight_GBps']:.0f} GB/s of weights, "
                f"hbm {r['step_hbm_frac']:.3f}, useful-op {r['step_useful_op_frac']:.3f}")
        out["sweep"] = sweep
        out["sweep_note"] = ("hbm_frac / useful_op_frac of a sweep entry are over the WHOLE step (every kernel of the call): "
                             "algorithmic bytes, resp. elements x (5 x passes + 12) lane-operations, over the step time and the peak. "
                             "The lane-operations are those of an evaluation that visits every element in every pass; the per-channel "
                             "entries (kernel sorted_rows) take the sums from the sorted row instead, so their useful_op_frac is the "
                             "work such an evaluation would have done over the time taken, and may exceed 1")

    if pool is not None:
        kw = dict(dtype=gp.dtype, bits=bits, group_size=args.group_size, mode=0, stat_scope=0, n_sigma=3.0, iters=args.iters,
                  lr=args.lr, select=0 if args.select == "best" else 1)
        single_rows = max(32, min(args.cpu_rows, Ws[0].shape[0]) // 32 * 32)
        pool_rows = max(32, min(args.cpu_rows * pool.workers // 2, Ws[0].shape[0]) // 32 * 32)
        c = cpu_baseline_pooled(pool, Ws, kw, single_rows, pool_rows)
        pool.close()
        out["cpu_baseline"] = {"value": c["pool_GBps"], "unit": "GB/s", "cores": pool.workers, "kind": "oracle",
                               "sample": f"first {pool_rows} rows x {c['cols']} cols of layer 0 q_proj in blocks of 32 rows over "
                                         f"{pool.workers} worker processes ({c['pool_s']:.1f} s, NumPy, one thread each; host "
                                         f"has {os.cpu_count()} logical CPUs)",
                               "seconds_per_model_extrapolated": elems * 2 / (c["pool_GBps"] * 1e9),
                               "single_thread": {"value": c["single_GBps"], "unit": "GB/s", "cores": 1,
                                                 "sample": f"first {single_rows} rows of the same matrix, blocks of 32 rows, in "
                                                           f"this process ({c['single_s']:.1f} s)",
                                                 "seconds_per_model_extrapolated": elems * 2 / (c["single_GBps"] * 1e9)}}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
