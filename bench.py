#!/usr/bin/env python3
"""Benchmark of the sensitive-sparse ZO step on one MI355X.

A "step" is one pass of the whole hot path over the whole stack of the chosen
workload: for every matrix a +eps and a -eps forward (int4 dequant + sparse
scatter with the Gaussian regenerated in-kernel + MFMA product), the MSE loss
of each, the SPSA scalar g, and the sparse update of every matrix.  Inputs are
seeded, synthetic and already resident in HBM when the clock starts.

Prints ONE JSON line: metric, value (ZO steps/s), ms_per_step, the roofline of the dominant kernel
(achieved vs peak, from per-launch events recorded by the library around the launches of the timed
steps themselves), the CPU oracle as a baseline with the parity of the GPU path on the same sample,
and -- in the default invocation -- the other workloads of the configuration list as extra keys:
`few_token` (the same stack at 16 tokens, HBM-bound), `c4` (a Mistral-7B block at 8192 tokens at three
mask densities) and `c5` (a 32-block OPT-6.7B stack at 1 / 16 / 64 tokens).
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
MEASURED_TRAFFIC_BYTES = {"c3": 7.44e10, "c3m16": 3.613e9,
                          # the extra legs of the default run (one Mistral block by density, 32 OPT blocks by token count)
                          "c4:0.0001": 4.329e9, "c4:0.001": 4.358e9, "c4:0.01": 4.604e9,
                          "c5:1": 3.447e9, "c5:16": 3.586e9, "c5:64": 4.237e9}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def algorithmic_bytes_fwd(m, M, fused=True):
    """Bytes one pass over a matrix must move: codes + scales + sparse (idx, val) + x, and either
    the bf16 target (loss fused into the kernel) or the fp32 y it writes."""
    side = 32 * m.N if m.lut is not None else 2 * m.N * (m.K // m.group)    # per-row table | group scales
    return (m.N * m.K // 2 + side + 8 * m.nnz + 2 * M * m.K + (2 if fused else 4) * M * m.N)


def few_token_path(M, two_sets=False):
    """The library's rule for the few-token path (slices of 16 / 32 token rows instead of 256-row tiles):
    at most 15 slices of 32 rows (16 with two activation sets), and fewer than 7.5 of them per row of
    tiles.  Only used to label the kernel and to pick default step counts."""
    rows = 16 if two_sets else 32
    slices, tile_rows = (M + rows - 1) // rows, (M + 255) // 256
    return slices <= 15 and 2 * slices < 15 * tile_rows


def time_steps(szo, torch, descs, seed, eps, lr, flags, steps, warmup, first_step=0):
    """`warmup` untimed steps, then `steps` timed ones between two events on the launch stream; the same
    timed steps have every forward-kernel and update-kernel launch bracketed by the library's own events."""
    ws = szo.new_workspace()
    scal = torch.zeros(3, dtype=torch.float64, device="cuda")
    stream = torch.cuda.current_stream()
    for s in range(first_step, first_step + warmup):
        szo.szo_zo_step(descs, seed, s, eps, lr, scal, ws, flags, stream.cuda_stream)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    szo.szo_kernel_timing(True)
    w0 = time.perf_counter()
    ev0.record(stream)
    for s in range(first_step + warmup, first_step + warmup + steps):
        szo.szo_zo_step(descs, seed, s, eps, lr, scal, ws, flags, stream.cuda_stream)
    ev1.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - w0
    (k_ms, k_n), (u_ms, u_n) = szo.szo_kernel_timing_read2()
    szo.szo_kernel_timing(False)
    lp, lm, g = scal.cpu().tolist()
    return {"ms_per_step": ev0.elapsed_time(ev1) / steps, "wall_ms_per_step": 1e3 * wall / steps,
            "fwd_ms": k_ms, "fwd_launches": k_n, "upd_ms": u_ms, "upd_launches": u_n,
            "steps": steps, "warmup": warmup, "last": (lp, lm, g)}


def rooflines(mats, M, t, few, fused, traffic=None):
    """Roofline entry of the dominant (forward) kernel and the figures of the sparse update, per launch."""
    steps = t["steps"]
    fwd_flops = sum(2.0 * M * m.N * m.K for m in mats)
    launches = t["fwd_launches"]
    k_ms = t["fwd_ms"] / launches
    one_pass = float(sum(algorithmic_bytes_fwd(m, M, fused) for m in mats))
    if few:       # one launch streams every matrix once and serves both signs
        kernel = "small_m_kernel"
        launch_bytes = one_pass * steps / launches
    else:         # large fused steps run every forward of the step in one table-driven launch
        kernel = "linear_fwd_table_kernel" if launches == steps else "linear_fwd_kernel"
        launch_bytes = one_pass * 2 * steps / launches
    launch_flops = 2 * fwd_flops * steps / launches
    tflops = launch_flops / (k_ms * 1e-3) / 1e12
    gbs = launch_bytes / (k_ms * 1e-3) / 1e9
    mfma_bound = (launch_flops / launch_bytes) > (PEAK_MFMA_16BIT_TFLOPS * 1e12) / (PEAK_HBM_GBS * 1e9)
    if mfma_bound:
        roof = {"bound": "mfma", "achieved": round(tflops, 2), "peak": PEAK_MFMA_16BIT_TFLOPS, "unit": "TFLOP/s",
                "frac": round(tflops / PEAK_MFMA_16BIT_TFLOPS, 4), "traffic": traffic}
    else:
        roof = {"bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": round(gbs / PEAK_HBM_GBS, 4), "traffic": traffic}
    roof.update({"kernel": kernel, "avg_launch_us": round(1e3 * k_ms, 2), "launches_timed": launches,
                 "flops_per_launch": launch_flops, "bytes_per_launch": launch_bytes,
                 "algorithmic_tflops": round(tflops, 2), "algorithmic_gbs": round(gbs, 1)})
    upd = None
    if t["upd_launches"]:       # 8 bytes per sensitive entry (fp32 value read and written); z is regenerated
        u_ms = t["upd_ms"] / t["upd_launches"]
        u_bytes = 8.0 * sum(m.nnz for m in mats) * steps / t["upd_launches"]
        upd = {"kernel": "sparse_update", "avg_launch_us": round(1e3 * u_ms, 2), "launches_timed": t["upd_launches"],
               "bytes_per_launch": u_bytes, "achieved": round(u_bytes / (u_ms * 1e-3) / 1e9, 1), "unit": "GB/s",
               "frac_of_hbm_peak": round(u_bytes / (u_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)}
    return roof, upd, 2 * fwd_flops


def descs_for(szo, mats, M, dt, with_y):
    """Descriptors of the stack at M tokens: the first M rows of every x and target (row-major, so a
    prefix of the resident arrays)."""
    out = []
    for m in mats:
        d = m.desc(dt, with_y=with_y)
        d.M = M
        out.append(d)
    return szo.desc_array(out)


def extra_workload(szo, torch, stack, name, seed, data_seed, dt, variants, steps=None, warmup=None, **build):
    """Builds `name` once per entry of `variants` that changes the stack (density) or once for all (token
    counts), times the fused step, and returns one summary per variant."""
    rows = []
    mats = cfg = None
    for v in variants:
        if mats is None or "density" in v:
            del mats
            torch.cuda.empty_cache()
            mats, cfg = stack.build_stack(name, data_seed, "cuda", density=v.get("density"), **build)
        M = v.get("M", mats[0].M)
        few = few_token_path(M)
        descs = descs_for(szo, mats, M, dt, with_y=False)
        t = time_steps(szo, torch, descs, seed, cfg["eps"], cfg["lr"], szo.STEP_FUSED_LOSS,
                       steps or (200 if few else 20), warmup if warmup is not None else (30 if few else 5))
        traffic = MEASURED_TRAFFIC_BYTES.get(f"{name}:{v['density']:g}" if "density" in v else f"{name}:{M}") if dt == szo.TILE_F16 else None
        roof, upd, step_flops = rooflines(mats, M, t, few, True, traffic)
        row = {"M": M, "density": v.get("density", cfg["density"]), "matrices": len(mats),
               "ms_per_step": round(t["ms_per_step"], 4), "steps": t["steps"], "warmup": t["warmup"],
               "step_tflops": round(step_flops / (t["ms_per_step"] * 1e-3) / 1e12, 2),
               "roofline": roof, "sparse_update": upd}
        log(f"[bench] {name} {v}: {t['ms_per_step']:.3f} ms/step, {roof['kernel']} {roof['achieved']} {roof['unit']} "
            f"({100 * roof['frac']:.1f} % of peak)")
        rows.append(row)
    del mats
    torch.cuda.empty_cache()
    return rows


def cpu_baseline_and_parity(szo, torch, mats, pristine, cfg, args, total_flops_per_step, dt):
    """The oracle, as it stands, on a bounded sample of the same workload (whole matrices in stack order,
    one full ZO step each, until the time budget is used), and the GPU path on the same sample (the same
    matrices with their initial sparse values, one single-matrix fused step each through the C ABI):
    the per-matrix losses and SPSA scalars of both sides, and the outputs of the first matrix, compared."""
    import numpy as np
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from helpers import make_oracle_matrix, rel_fro
    from oracle import zo as ozo, layer as olayer, philox as ophilox
    from paper_2406_02913_amd import synth
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count()
    M = mats[0].M
    done_flops, t_spent, used, ref = 0.0, 0.0, [], []
    nb = len(cfg["block"])
    y_rel = None
    for idx, dm in enumerate(mats):
        layer, i = divmod(idx, nb)
        name, N, K = cfg["block"][i]
        m = make_oracle_matrix(synth.matrix_seed(args.data_seed, layer, i), M, N, K, cfg["group"],
                               cfg["density"], cfg["mask"], nnz_base=dm.nnz_base, fmt=args.format)
        if idx == 0:          # outputs of one perturbed forward, element by element (not part of the timed baseline)
            z = ophilox.zbar(args.seed, 0, m.nnz_base, m.sp_idx.size)
            y_ref = olayer.linear_fwd(m.x_bits, m.codes, m.scales, m.group, m.sp_idx, m.sp_val, z, +1, cfg["eps"], lut=m.lut)
            dm.sp_val.copy_(pristine[0])
            y_buf = torch.empty((M, N), dtype=torch.float32, device="cuda")
            d = dm.desc(dt, with_y=False)
            d.y = y_buf.data_ptr()
            szo.szo_linear_fwd(d, args.seed, 0, +1, cfg["eps"])
            y_rel = rel_fro(y_buf.cpu().numpy(), y_ref)
            del y_buf, y_ref
        t0 = time.perf_counter()
        r = ozo.zo_step([m], args.seed, 0, cfg["eps"], cfg["lr"])
        t_spent += time.perf_counter() - t0
        ref.append((r["loss_plus"], r["loss_minus"], r["g"]))
        done_flops += 2 * 2.0 * M * N * K
        used.append(f"L{layer}.{name}")
        if t_spent >= args.cpu_seconds:
            break
    frac = done_flops / total_flops_per_step
    est_step_s = t_spent / frac
    base = {"value": 1.0 / est_step_s, "unit": "ZO steps/s", "cores": int(threads), "kind": "oracle",
            "sample": f"full oracle ZO step (fp64) on the first {len(used)} matrices of the stack ({used[0]} .. {used[-1]}) "
                      f"at M={M}: {t_spent:.2f} s for {100 * frac:.3f}% of one step's FLOPs, extrapolated by FLOPs",
            "cpu": platform.processor() or platform.machine(), "os_cpu_count": os.cpu_count()}
    # the GPU on the same sample
    ws = szo.new_workspace()
    scal = torch.zeros(3, dtype=torch.float64, device="cuda")
    got = []
    for idx in range(len(ref)):
        mats[idx].sp_val.copy_(pristine[idx])
        szo.szo_zo_step([mats[idx].desc(dt, with_y=False)], args.seed, 0, cfg["eps"], 0.0, scal, ws, szo.STEP_FUSED_LOSS)
        got.append(scal.cpu().tolist())
    ref, got = np.array(ref), np.array(got)
    parity = {"y_rel": y_rel,
              "loss_rel": float(np.max(np.abs(got[:, :2] - ref[:, :2]) / ref[:, :2])),
              "g_rel": float(np.linalg.norm(got[:, 2] - ref[:, 2]) / max(np.linalg.norm(ref[:, 2]), 1e-300)),
              "sample": f"the baseline's {len(ref)} matrices: y of one +eps forward of {used[0]} (relative Frobenius error), "
                        "per-matrix L+ and L- (largest relative error), per-matrix SPSA scalars g_i = (L+ - L-) / (2 eps) "
                        "(||g_gpu - g_oracle|| / ||g_oracle|| over the sample)",
              "tolerance": {"y_rel": 5e-3, "g_rel": 1e-2}}
    return base, parity


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
    ap.add_argument("--tile-config", type=int, default=0, choices=[0, 1, 2, 3, 4, 5, 6, 7],
                    help="0: the library chooses (few-token path for small token counts); 1 / 2: force the tiled kernel with "
                         "128x128 / 256x256 workgroup tiles; 3: as 2, and always one grouped launch per step; 4: as 0 "
                         "with 32 token rows per pass of the few-token path wherever there are more than 16 (for comparisons)")
    ap.add_argument("--seed", type=int, default=2024)
    ap.add_argument("--data-seed", type=int, default=0)
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="budget of the oracle baseline leg (0 = skip)")
    ap.add_argument("--no-extras", action="store_true",
                    help="default invocation only: skip the few-token, Mistral-block and OPT-stack legs (profiling runs)")
    ap.add_argument("--host-rebuild", action="store_true",
                    help="instead of the benchmark: time the host-side bookkeeping of a mask change (new mask -> tile "
                         "order -> re-split and re-quantise -> banded layout) for one block of the workload and exit")
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
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        log("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1")
        sys.exit(2)

    import torch
    from paper_2406_02913_amd import stack, synth, szo

    # the default invocation (the headline workload, untouched) also reports the other workloads
    default_run = (args.workload == "c3" and args.layers is None and args.m is None and args.density is None
                   and not args.unfused_loss and not args.two_activation_sets and not args.one_dense_pass
                   and args.tile == "f16" and args.tile_config == 0 and args.format == "uniform")
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
    pristine = [m.sp_val.clone() for m in mats]          # the parity leg starts from the initial sparse values

    if args.two_activation_sets:
        gen = torch.Generator(device="cuda").manual_seed(args.data_seed + 7)
        for m in mats:
            m.x_minus = torch.randn(m.x.shape, device="cuda", generator=gen).to(torch.bfloat16)
    szo.szo_set_tile_config(args.tile_config)
    M = mats[0].M
    descs = szo.desc_array([m.desc(dt, with_y=bool(args.unfused_loss)) for m in mats])
    eps, lr = cfg["eps"], cfg["lr"]

    t = time_steps(szo, torch, descs, args.seed, eps, lr, flags, args.steps, args.warmup)
    ms_per_step = t["ms_per_step"]
    lp, lm, g = t["last"]
    log(f"[bench] {ms_per_step:.3f} ms/step (events), {t['wall_ms_per_step']:.3f} ms/step (wall); "
        f"last step L+={lp:.6f} L-={lm:.6f} g={g:.4e}")
    few = (all((few_token_path(m.M, args.two_activation_sets) or args.one_dense_pass) and m.K % 128 == 0 for m in mats)
           and dt == szo.TILE_F16 and args.tile_config in (0, 4, 5) and bool(flags))        # the library's few-token path
    traffic = MEASURED_TRAFFIC_BYTES.get(args.workload) if (
        args.layers is None and args.m is None and args.density is None and flags and dt == szo.TILE_F16
        and args.tile_config == 0 and args.format == "uniform" and not args.two_activation_sets
        and not args.one_dense_pass) else None
    roof, upd, step_flops = rooflines(mats, M, t, few, bool(flags), traffic)
    log(f"[bench] {roof['kernel']}: {roof['avg_launch_us']:.1f} us/launch avg over {roof['launches_timed']} launches of the "
        f"timed steps, {roof['achieved']} {roof['unit']}")

    extras = {}
    d16 = None
    if default_run and not args.no_extras:
        # the second target: the same resident stack at 16 tokens (first 16 rows of every x and target)
        try:
            d16 = descs_for(szo, mats, 16, dt, with_y=False)
            t16 = time_steps(szo, torch, d16, args.seed, eps, lr, flags, 200, 30, first_step=1000)
            r16, u16, _ = rooflines(mats, 16, t16, True, True, MEASURED_TRAFFIC_BYTES.get("c3m16"))
            extras["few_token"] = {"workload": f"the same {len(mats)} matrices at M=16 tokens (the first 16 rows of every x and target)",
                                   "ms_per_step": round(t16["ms_per_step"], 4), "value": round(1e3 / t16["ms_per_step"], 2),
                                   "unit": "ZO steps/s", "steps": 200, "warmup": 30, "roofline": r16, "sparse_update": u16}
            log(f"[bench] few_token: {t16['ms_per_step']:.4f} ms/step, small_m_kernel {r16['achieved']} GB/s "
                f"({100 * r16['frac']:.1f} % of the HBM peak)")
        except Exception as e:      # noqa: BLE001 -- reported in the line instead of losing the headline
            extras["few_token"] = {"error": f"{type(e).__name__}: {e}"}
            log(f"[bench] few_token leg failed: {e}")

    base = parity = None
    if args.cpu_seconds > 0:
        try:
            base, parity = cpu_baseline_and_parity(szo, torch, mats, pristine, cfg, args, step_flops, dt)
            log(f"[bench] oracle baseline: {base['value']:.3e} steps/s on {base['cores']} threads; parity {parity['y_rel']:.2e} (y), "
                f"{parity['loss_rel']:.2e} (losses), {parity['g_rel']:.2e} (g)")
        except Exception as e:      # noqa: BLE001
            base = {"error": f"{type(e).__name__}: {e}"}
            log(f"[bench] oracle baseline leg failed: {e}")

    n_mats, n_blocks = len(mats), len(mats) // len(cfg["block"])
    if default_run and not args.no_extras:
        del mats, descs, pristine, d16
        torch.cuda.empty_cache()
        # the other workloads never take the headline line down with them
        for key, label, name, variants, build in (
                ("c4", "one Mistral-7B block (q, k, v, o, gate, up, down), M=8192 tokens, int4 group 128, uniform mask",
                 "c4", [{"density": 1e-4}, {"density": 1e-3}, {"density": 1e-2}], {}),
                ("c5", "32 OPT-6.7B blocks (q, k, v, o, fc1, fc2), int4 group 128, uniform mask 0.001",
                 "c5", [{"M": 1}, {"M": 16}, {"M": 64}], {"layers": 32, "M": 64})):
            try:
                extras[key] = {"workload": label,
                               "runs": extra_workload(szo, torch, stack, name, args.seed, args.data_seed, dt, variants, **build)}
            except Exception as e:      # noqa: BLE001 -- reported in the line instead
                extras[key] = {"workload": label, "error": f"{type(e).__name__}: {e}"}
                log(f"[bench] {key} leg failed: {e}")

    out = {
        "metric": "ZO steps/sec + % bf16 MFMA peak, int4+0.1%-sparse linears, Llama-2-7B shapes",
        "value": round(1e3 / ms_per_step, 4), "unit": "ZO steps/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None,
        "dtype": "f16" if dt == szo.TILE_F16 else "bf16", "data": "synthetic",
        "config": {"workload": f"{args.workload}: {n_mats} matrices ({n_blocks} block(s) of "
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
        "parity": parity,
    }
    out.update(extras)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
