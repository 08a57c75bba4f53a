#!/usr/bin/env python3
"""Benchmark of the sensitive-sparse ZO step on one MI355X.

A "step" is one pass of the whole hot path over the whole stack of the chosen
workload: for every matrix a +eps and a -eps forward (int4 dequant + sparse
scatter with the Gaussian regenerated in-kernel + MFMA product), the MSE loss
of each, the SPSA scalar g, and the sparse update of every matrix.  Inputs are
seeded, synthetic and already resident in HBM when the clock starts.

Prints ONE JSON line: metric, value (ZO steps/s), ms_per_step, the roofline of the dominant kernel
(achieved vs peak, from per-launch events recorded by the library) and the CPU oracle as a baseline.
"""
import argparse
import json
import os
import platform
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_MFMA_16BIT_TFLOPS = 2500.0      # MI355X dense fp16/bf16 matrix peak
PEAK_HBM_GBS = 8000.0                # MI355X HBM3E
# HBM bytes per launch of the dominant kernel, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this
# script scaled by a plain copy of known size (profiles/*.md give the commands and the raw readings).
# Only valid for the unmodified workloads; anything else reports null.
MEASURED_TRAFFIC_BYTES = {"c3": 1.4187e11, "c3m16": 3.632e9}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def algorithmic_bytes_fwd(m, fused=True):
    """Bytes one pass over a matrix must move: codes + scales + sparse (idx, val) + x, and either
    the bf16 target (loss fused into the kernel) or the fp32 y it writes."""
    side = 32 * m.N if m.lut is not None else 2 * m.N * (m.K // m.group)    # per-row table | group scales
    return (m.N * m.K // 2 + side + 8 * m.nnz + 2 * m.M * m.K + (2 if fused else 4) * m.M * m.N)


def few_token_path(M, two_sets=False):
    """The library's rule for the few-token path (slices of 16 / 32 token rows instead of 256-row tiles):
    at most 15 slices of 32 rows (16 with two activation sets), and fewer than 7.5 of them per row of
    tiles.  Only used to label the kernel and to pick default step counts."""
    rows = 16 if two_sets else 32
    slices, tile_rows = (M + rows - 1) // rows, (M + 255) // 256
    return slices <= 15 and 2 * slices < 15 * tile_rows


def cpu_baseline(cfg, args, total_flops_per_step):
    """The oracle, as it stands, on a bounded sample of the same workload."""
    import numpy as np
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from helpers import make_oracle_matrix
    from oracle import zo as ozo
    from paper_2406_02913_amd import synth
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count()
    M = args.m or cfg["M"]
    done_flops, t_spent, used = 0.0, 0.0, []
    layers = args.layers or cfg["layers"]
    for layer in range(layers):                 # whole matrices, in stack order, until the time budget is used
        for i, (name, N, K) in enumerate(cfg["block"]):
            m = make_oracle_matrix(synth.matrix_seed(args.data_seed, layer, i), M, N, K, cfg["group"],
                                   cfg["density"], cfg["mask"], fmt=args.format)
            t0 = time.perf_counter()
            ozo.zo_step([m], args.seed, 0, cfg["eps"], cfg["lr"])
            t_spent += time.perf_counter() - t0
            done_flops += 2 * 2.0 * M * N * K
            used.append(f"L{layer}.{name}")
            if t_spent >= args.cpu_seconds:
                break
        if t_spent >= args.cpu_seconds:
            break
    frac = done_flops / total_flops_per_step
    est_step_s = t_spent / frac
    return {"value": 1.0 / est_step_s, "unit": "ZO steps/s", "cores": int(threads), "kind": "oracle",
            "sample": f"full oracle ZO step (fp64) on the first {len(used)} matrices of the stack ({used[0]} .. {used[-1]}) "
                      f"at M={M}: {t_spent:.2f} s for {100 * frac:.3f}% of one step's FLOPs, extrapolated by FLOPs",
            "cpu": platform.processor() or platform.machine(), "os_cpu_count": os.cpu_count()}


def host_rebuild(args):
    """Dynamic-mask bookkeeping (the paper's variant that re-selects the mask every 100 steps) as a
    host-side throughput figure: everything libszo's host calls must redo when the mask of a matrix
    changes.  No GPU involved; the copy of the new arrays to the device is not included."""
    from paper_2406_02913_amd import synth, szo
    cfg = synth.WORKLOADS[args.workload]
    rows, total = [], 0.0
    for i, (name, N, K) in enumerate(cfg["block"]):
        W = synth.dense_weight(synth.matrix_seed(args.data_seed, 0, i), N, K)
        k = int(cfg["density"] * N * K + 0.5)
        t0 = time.perf_counter()
        flat = szo.szo_mask_generate(N, K, k, 0 if cfg["mask"] == "uniform" else 1, 4242 + i)
        t1 = time.perf_counter()
        tile_ptr, sp_idx, perm = szo.szo_tcsr_build(N, K, flat)
        t2 = time.perf_counter()
        q, scales, sp_val = szo.szo_quantize_pack(W, cfg["group"], sp_idx)
        t3 = time.perf_counter()
        szo.szo_layout_weights(q, scales, cfg["group"])
        t4 = time.perf_counter()
        rows.append({"matrix": name, "N": N, "K": K, "nnz": k, "mask_s": t1 - t0, "tile_order_s": t2 - t1,
                     "split_quantise_s": t3 - t2, "layout_s": t4 - t3})
        total += t4 - t0
    print(json.dumps({"host_rebuild_s_per_block": total, "blocks_per_s": 1.0 / total, "threads": os.cpu_count(),
                      "workload": args.workload, "per_matrix": rows}), flush=True)


def vendor_gemm(args):
    """Not part of the path: torch.matmul (hipBLASLt / rocBLAS) on x [M,K] times W^T with W [N,K] already
    in 16 bits, i.e. the dense product of the SparseAdd-then-DenseMM form without dequantisation, sparse
    add, loss or update."""
    import torch
    from paper_2406_02913_amd import synth
    cfg = synth.WORKLOADS[args.workload]
    M = args.m or cfg["M"]
    dt = torch.float16 if args.tile == "f16" else torch.bfloat16
    rows, total_us, total_flops = [], 0.0, 0.0
    torch.manual_seed(0)
    for name, N, K in cfg["block"]:
        for data in ("random", "zeros"):
            if data == "random":
                x = torch.randn(M, K, device="cuda").to(dt)
                w = (0.02 * torch.randn(N, K, device="cuda")).to(dt)
            else:
                x = torch.zeros(M, K, device="cuda", dtype=dt)
                w = torch.zeros(N, K, device="cuda", dtype=dt)
            for _ in range(30):
                y = x @ w.t()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(50):
                y = x @ w.t()
            e1.record()
            torch.cuda.synchronize()
            us = 1e3 * e0.elapsed_time(e1) / 50
            rows.append({"matrix": name, "M": M, "N": N, "K": K, "operands": data, "us": round(us, 1),
                         "tflops": round(2.0 * M * N * K / us / 1e6, 1)})
            if data == "random":
                total_us += us
                total_flops += 2.0 * M * N * K
            del x, w, y
    print(json.dumps({"vendor_dense_gemm": rows, "dtype": args.tile, "workload": args.workload,
                      "block_us_random": round(total_us, 1),
                      "block_tflops_random": round(total_flops / total_us / 1e6, 1)}), flush=True)


def operand_sensitivity(args):
    """Not the benchmark: the same fused step on a few blocks of the workload, timed with the synthetic
    operands and again after x and / or the codes have been overwritten with zeros.  Matrix cores draw
    power by the bits that toggle, so the difference is what the clock management takes; the all-zero
    figure is what the kernel's instruction schedule alone allows."""
    import torch
    from paper_2406_02913_amd import stack, synth, szo
    torch.cuda.set_device(0)
    szo.szo_set_tile_config(3 if args.tile_config == 0 else args.tile_config)
    dt = szo.TILE_F16 if args.tile == "f16" else szo.TILE_BF16
    mats, cfg = stack.build_stack(args.workload, args.data_seed, "cuda", M=args.m, layers=args.layers or 4,
                                  density=args.density)
    descs = szo.desc_array([m.desc(dt, with_y=False) for m in mats])
    ws = szo.new_workspace()
    scal = torch.zeros(3, dtype=torch.float64, device="cuda")
    flops = sum(2 * 2.0 * m.M * m.N * m.K for m in mats)
    rows = []

    def timed(tag):
        for s in range(5):
            szo.szo_zo_step(descs, args.seed, s, cfg["eps"], 0.0, scal, ws, szo.STEP_FUSED_LOSS)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for s in range(20):
            szo.szo_zo_step(descs, args.seed, s, cfg["eps"], 0.0, scal, ws, szo.STEP_FUSED_LOSS)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 20
        rows.append({"operands": tag, "ms_per_step": round(ms, 3), "tflops": round(flops / ms / 1e9, 1)})

    timed("synthetic x, synthetic codes")
    for m in mats:
        m.x.zero_()
    timed("zero x, synthetic codes")
    for m in mats:
        m.qweight.fill_(0x88)
    timed("zero x, zero codes")
    for m in mats:
        m.x.normal_()
    timed("random x, zero codes")
    print(json.dumps({"operand_sensitivity": rows, "workload": args.workload, "blocks": args.layers or 4,
                      "M": mats[0].M, "dtype": args.tile, "lr": 0.0}), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="timed steps (default 20; 200 for the few-token workloads)")
    ap.add_argument("--warmup", type=int, default=None, help="untimed steps first (default 3; 30 for the few-token workloads, "
                    "whose sub-millisecond steps otherwise end before the clocks have settled)")
    ap.add_argument("--workload", default="c3", help="c1|c2|c3|c4|c5|c3m16 (see synth.WORKLOADS)")
    ap.add_argument("--layers", type=int, default=None, help="override the number of decoder blocks")
    ap.add_argument("--m", type=int, default=None, help="override the token count")
    ap.add_argument("--density", type=float, default=None)
    ap.add_argument("--tile", default="f16", choices=["f16", "bf16"])
    ap.add_argument("--format", default="uniform", choices=["uniform", "lut"],
                    help="4-bit format of the frozen part: uniform codes with group scales (the workloads' format) or "
                         "the non-uniform one, a table of 16 fp16 centroids per output row")
    ap.add_argument("--unfused-loss", action="store_true", help="write y and run the separate loss kernel")
    ap.add_argument("--two-activation-sets", action="store_true",
                    help="give every layer a second, different set of activations for its -eps forward (desc.x_minus), "
                         "as inside a model; the few-token path then still reads the weights once for both signs")
    ap.add_argument("--one-dense-pass", action="store_true",
                    help="SZO_STEP_ONE_DENSE_PASS: the slicing path of the few-token case at any token count (the dense "
                         "product of a slice is computed once and serves both signs; valid because both forwards of a "
                         "layer see the same x in this benchmark).  Not the default: see include/szo.h")
    ap.add_argument("--tile-config", type=int, default=0, choices=[0, 1, 2, 3, 4, 5],
                    help="0: the library chooses (few-token path for small token counts); 1 / 2: force the tiled kernel with "
                         "128x128 / 256x256 workgroup tiles; 3: as 2, and always one grouped launch per step; 4: as 0 "
                         "with 32 token rows per pass of the few-token path wherever there are more than 16 (for comparisons)")
    ap.add_argument("--seed", type=int, default=2024)
    ap.add_argument("--data-seed", type=int, default=0)
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="budget of the oracle baseline leg (0 = skip)")
    ap.add_argument("--kernel-reps", type=int, default=None,
                    help="extra steps run with per-launch kernel timing switched on (default: as many as --steps)")
    ap.add_argument("--host-rebuild", action="store_true",
                    help="instead of the benchmark: time the host-side bookkeeping of a mask change (new mask -> tile "
                         "order -> re-split and re-quantise -> banded layout) for one block of the workload and exit")
    ap.add_argument("--vendor-gemm", action="store_true",
                    help="instead of the benchmark: time the vendor library's plain dense 16-bit GEMM (torch.matmul) on "
                         "the workload's shapes with random and with all-zero operands and exit (context for the "
                         "roofline: what a dense product on already materialised weights reaches on this machine)")
    ap.add_argument("--operand-sensitivity", action="store_true",
                    help="instead of the benchmark: time the fused step on --layers (default 4) blocks with the synthetic "
                         "operands and with x and / or the codes zeroed, and exit (how much of the step time is the "
                         "data-dependent power draw of the matrix cores, how much the kernel's own schedule)")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MIB",
                    help="instead of the benchmark: copy a buffer of this many MiB five times with a plain copy kernel "
                         "and exit (known traffic, to scale the FETCH_SIZE / WRITE_SIZE counters of a profiler run)")
    args = ap.parse_args()
    if args.copy_calibration:
        import torch
        n = args.copy_calibration << 20
        src = torch.ones(n, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_per_launch": n, "launches": 5}), flush=True)
        return
    if args.host_rebuild:
        host_rebuild(args)
        return
    if args.vendor_gemm:
        vendor_gemm(args)
        return
    if args.operand_sensitivity:
        operand_sensitivity(args)
        return
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        log("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1")
        sys.exit(2)

    import torch
    from paper_2406_02913_amd import stack, synth, szo

    few_default = few_token_path(args.m or synth.WORKLOADS[args.workload]["M"], args.two_activation_sets)
    if args.steps is None:
        args.steps = 200 if few_default else 20
    if args.warmup is None:
        args.warmup = 30 if few_default else 3
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dt = szo.TILE_F16 if args.tile == "f16" else szo.TILE_BF16
    flags = 0 if args.unfused_loss else szo.STEP_FUSED_LOSS
    if args.one_dense_pass and flags:
        flags |= szo.STEP_ONE_DENSE_PASS

    t0 = time.perf_counter()
    count = [0]

    def progress(lin):
        count[0] += 1
        if count[0] % 28 == 0:
            log(f"[bench] built {count[0]} matrices ({time.perf_counter() - t0:.1f} s)")

    mats, cfg = stack.build_stack(args.workload, args.data_seed, "cuda", M=args.m, layers=args.layers,
                                  density=args.density, progress=progress, fmt=args.format)
    if args.density is not None:
        cfg["density"] = args.density
    torch.cuda.synchronize()
    log(f"[bench] {len(mats)} matrices resident after {time.perf_counter() - t0:.1f} s, "
        f"{torch.cuda.memory_allocated() / 2**30:.1f} GiB")

    if args.two_activation_sets:
        gen = torch.Generator(device="cuda").manual_seed(args.data_seed + 7)
        for m in mats:
            m.x_minus = torch.randn(m.x.shape, device="cuda", generator=gen).to(torch.bfloat16)
    szo.szo_set_tile_config(args.tile_config)
    descs = szo.desc_array([m.desc(dt, with_y=bool(args.unfused_loss)) for m in mats])
    ws = szo.new_workspace()
    scal = torch.zeros(3, dtype=torch.float64, device="cuda")
    eps, lr = cfg["eps"], cfg["lr"]
    stream = torch.cuda.current_stream()

    def one_step(s):
        szo.szo_zo_step(descs, args.seed, s, eps, lr, scal, ws, flags, stream.cuda_stream)

    for s in range(args.warmup):
        one_step(s)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    w0 = time.perf_counter()
    ev0.record(stream)
    for s in range(args.warmup, args.warmup + args.steps):
        one_step(s)
    ev1.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - w0
    ms_per_step = ev0.elapsed_time(ev1) / args.steps
    lp, lm, g = scal.cpu().tolist()
    log(f"[bench] {ms_per_step:.3f} ms/step (events), {1e3 * wall / args.steps:.3f} ms/step (wall); "
        f"last step L+={lp:.6f} L-={lm:.6f} g={g:.4e}")

    # ---- the dominant kernel alone: the library brackets every forward-kernel launch of a few more
    #      steps with events on the launch stream (szo_kernel_timing) ----
    fwd_flops = sum(2.0 * m.M * m.N * m.K for m in mats)
    few = (all((few_token_path(m.M, args.two_activation_sets) or args.one_dense_pass) and m.K % 128 == 0 for m in mats) and dt == szo.TILE_F16
           and args.tile_config in (0, 4, 5) and bool(flags))                            # the library's few-token path
    reps = args.steps if args.kernel_reps is None else max(1, args.kernel_reps)
    szo.szo_kernel_timing(True)
    for s in range(reps):
        one_step(args.warmup + args.steps + s)
    (k_total_ms, launches), (u_total_ms, u_launches) = szo.szo_kernel_timing_read2()
    szo.szo_kernel_timing(False)
    k_ms = k_total_ms / launches
    if few:
        # one launch streams every matrix once and serves both signs
        kernel = "small_m_kernel"
        launch_bytes = float(sum(algorithmic_bytes_fwd(m, fused=bool(flags)) for m in mats)) * reps / launches
        launch_flops = 2 * fwd_flops * reps / launches
    else:
        # large fused steps run every forward of the step in one table-driven launch
        kernel = "linear_fwd_table_kernel" if launches == reps else "linear_fwd_kernel"
        launch_bytes = float(sum(algorithmic_bytes_fwd(m, fused=bool(flags)) for m in mats)) * 2 * reps / launches
        launch_flops = 2 * fwd_flops * reps / launches
    tflops = launch_flops / (k_ms * 1e-3) / 1e12
    gbs = launch_bytes / (k_ms * 1e-3) / 1e9
    mfma_bound = (launch_flops / launch_bytes) > (PEAK_MFMA_16BIT_TFLOPS * 1e12) / (PEAK_HBM_GBS * 1e9)
    if mfma_bound:
        roof = {"bound": "mfma", "achieved": round(tflops, 2), "peak": PEAK_MFMA_16BIT_TFLOPS, "unit": "TFLOP/s",
                "frac": round(tflops / PEAK_MFMA_16BIT_TFLOPS, 4), "traffic": None}
    else:
        roof = {"bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": round(gbs / PEAK_HBM_GBS, 4), "traffic": None}
    if (args.layers is None and args.m is None and args.density is None and flags and dt == szo.TILE_F16
            and args.tile_config == 0 and args.format == "uniform"):
        roof["traffic"] = MEASURED_TRAFFIC_BYTES.get(args.workload)
    roof.update({"kernel": kernel, "avg_launch_us": round(1e3 * k_ms, 2), "launches_timed": launches,
                 "flops_per_launch": launch_flops, "bytes_per_launch": launch_bytes})
    # the sparse update: 8 bytes per sensitive entry (fp32 value read and written); z is regenerated
    upd = None
    if u_launches:
        u_ms = u_total_ms / u_launches
        u_bytes = 8.0 * sum(m.nnz for m in mats) * reps / u_launches
        upd = {"kernel": "sparse_update", "avg_launch_us": round(1e3 * u_ms, 2), "launches_timed": u_launches,
               "bytes_per_launch": u_bytes, "achieved": round(u_bytes / (u_ms * 1e-3) / 1e9, 1), "unit": "GB/s",
               "frac_of_hbm_peak": round(u_bytes / (u_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)}
    step_flops = 2 * fwd_flops
    log(f"[bench] {kernel}: {1e3 * k_ms:.1f} us/launch avg over {launches} launches, {tflops:.1f} TFLOP/s, "
        f"{gbs:.1f} GB/s algorithmic")

    base = None
    if args.cpu_seconds > 0:
        base = cpu_baseline(cfg, args, step_flops)
        log(f"[bench] oracle baseline: {base['value']:.3e} steps/s on {base['cores']} threads")

    M = mats[0].M
    out = {
        "metric": "ZO steps/sec + % bf16 MFMA peak, int4+0.1%-sparse linears, Llama-2-7B shapes",
        "value": round(1e3 / ms_per_step, 4), "unit": "ZO steps/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None,
        "dtype": "f16" if dt == szo.TILE_F16 else "bf16", "data": "synthetic",
        "config": {"workload": f"{args.workload}: {len(mats)} matrices ({len(mats) // len(cfg['block'])} block(s) of "
                               f"{[b[0] for b in cfg['block']]}), M={M} tokens, "
                               + (f"int4 group {cfg['group']}, " if args.format == "uniform" else "4-bit table format, ") +
                               f"mask {cfg['density']:g} {cfg['mask']}, eps={eps}, lr={lr}",
                   "loss": "fused into the forward epilogue" if flags else "separate kernel",
                   "dense_product": ("once per sign" if (not few or args.two_activation_sets)
                                     else "once per slice of token rows, shared by both signs"),
                   "activations": "x for +eps, x_minus for -eps" if args.two_activation_sets else "one x for both signs",
                   "tile": args.tile, "format": args.format, "accumulate": "f32", "loss_accumulate": "f64"},
        "step_tflops": round(step_flops / (ms_per_step * 1e-3) / 1e12, 2),
        "step_frac_of_mfma_peak": round(step_flops / (ms_per_step * 1e-3) / 1e12 / PEAK_MFMA_16BIT_TFLOPS, 4),
        "roofline": roof,
        "sparse_update": upd,
        "cpu_baseline": base,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
