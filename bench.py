#!/usr/bin/env python3
"""Benchmark of the HARP rotation hot path on one MI355X.

A step is one pass of the hot path over one batch of synthetic activations already resident
in device memory: ``harp_apply`` (load + signs, every stage on chip, store) followed by
``harp_apply_transpose`` on the same batch.  Each call transforms n rows, so a step counts
2 n row-transforms.  Batches rotate through a pool larger than the 256 MB Infinity Cache so
the timed launches read and write device memory, not a cache.

Prints ONE JSON line (metric: rotation rows/s and achieved HBM GB/s as a
fraction of the 8 TB/s peak), with a ``roofline`` object for the dominant kernel (timed
with HIP events on the launch stream) and a ``cpu_baseline`` object (the float64 oracle
timed on the host cores on a bounded sample of the same workload).
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

HBM_PEAK_GBS = 8000.0
KERNEL_SYMBOL = {"dpp_radix2": "harp_dpp_kernel",
                 "pipe_radix2": "harp_pipe_kernel", "tile_fused": "harp_tile_kernel",
                 "tile_generic": "harp_tile_kernel", "split_pipe_stream": "harp_pipe_kernel",
                 "split_chunk_stream": "harp_tile_kernel", "wave_radix2": "harp_wave_kernel",
                 "split_wave_stream": "harp_wave_kernel", "radix_tile": "harp_radix_kernel",
                 "split_radix_stream": "harp_radix_kernel", "radix_tile_int8": "harp_radix_kernel",
                 "split_radix_stream_int8": "harp_radix_kernel",
                 "split_dpp_stream_h16": "harp_dpp_kernel", "split_wave_stream_h16": "harp_wave_kernel"}


# kernels one call of harp_apply launches, by the path name harp_plan_kernel_name reports
KERNELS_OF = {"split_wave_stream": ["harp_wave_kernel", "harp_stream_mfma_kernel"],
              "split_pipe_stream": ["harp_pipe_kernel", "harp_stream_kernel"],
              "split_dpp_stream_h16": ["harp_dpp_kernel", "harp_stream_z16_kernel"],
              "split_wave_stream_h16": ["harp_wave_kernel", "harp_stream_z16_kernel"]}


def cpu_baseline(w, sample_rows: int):
    """The oracle as it stands (dense U by pushing the signed identity through the stages,
    then X @ U and X @ U^T), float64 numpy, on `sample_rows` rows of the workload."""
    import numpy as np
    from oracle import harp_oracle as ho
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    X = w["X"][:sample_rows].astype(np.float64)
    t0 = time.perf_counter()
    U = ho.build_U(w["d"], w["radices"], w["blocks"], w["signs"])
    t1 = time.perf_counter()
    Y = X @ U
    Z = X @ U.T
    t2 = time.perf_counter()
    assert Y.shape == Z.shape
    total = (t1 - t0) + (t2 - t1)
    # second CPU figure: the oracle's stage-by-stage form of the same method (float64 numpy,
    # validated against the dense form in the CPU tests), on the same rows
    ns = sample_rows
    t3 = time.perf_counter()
    Ys = ho.apply_staged(w["X"][:ns], w["d"], w["radices"], w["blocks"], w["signs"])
    Zs = ho.apply_transpose_staged(w["X"][:ns], w["d"], w["radices"], w["blocks"], w["signs"])
    t4 = time.perf_counter()
    assert Ys.shape == Zs.shape
    return {
        "value": 2 * sample_rows / total, "unit": "rows/s", "cores": int(cores), "kind": "oracle",
        "sample": f"{sample_rows} of {w['n']} rows, apply + transpose; build dense U once "
                  f"({t1 - t0:.2f} s) + two float64 matmuls ({t2 - t1:.2f} s)",
        "seconds": total,
        "staged": {"value": 2 * ns / (t4 - t3), "unit": "rows/s", "kind": "oracle, stage by stage",
                   "sample": f"{ns} of {w['n']} rows, apply + transpose", "seconds": t4 - t3},
    }


def warm_clocks(fn, seconds=0.08):
    """Run fn() repeatedly for about `seconds` of wall time: the shader clock needs tens of
    milliseconds of sustained load to settle, and host-side set-up lets it drop again."""
    import torch
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < seconds:
        for _ in range(20):
            fn()
        torch.cuda.synchronize()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # defaults: the shader clock needs a few hundred launches of sustained load to settle (40
    # warm-up steps read 12.6 us per launch, 400 read 11.6, 2000 and more 11.5)
    ap.add_argument("--steps", type=int, default=4000)
    ap.add_argument("--warmup", type=int, default=2000)
    ap.add_argument("--workload", default="llama7b_4096_r2")
    ap.add_argument("--rows", type=int, default=None, help="override n (default: the workload's)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--extra", action="store_true", help="also time the other shapes (stderr)")
    ap.add_argument("--decode", action="store_true",
                    help="also time the decode regime (n = 1..64 rows; stderr): median of 1000 "
                         "launches and the per-launch time of a HIP graph of 20 launches")
    ap.add_argument("--x8", action="store_true",
                    help="add roofline.at_8x_rows: the same step on the batch repeated 8 times "
                         "(off by default so that a profile of the default command holds "
                         "launches of one size only)")
    ap.add_argument("--shapes", action="store_true",
                    help="also time apply and apply_transpose (n = 2048, bf16 and f32) over the "
                         "layer widths of the Llama-2 / Llama-3 families under the radix-2 and "
                         "the greedy radix-8 schedules, and rotate_weight over their layer "
                         "shapes (stderr)")
    ap.add_argument("--int8", action="store_true",
                    help="only the int8-parameter lines of --shapes: blocks rebuilt at plan creation "
                         "against blocks rebuilt inside the kernel (stderr)")
    ap.add_argument("--settle-ms", type=float, default=100.0,
                    help="untimed set-up before the warm-up steps: the same step run for this many "
                         "milliseconds so that the shader clock has settled whatever --warmup is "
                         "(0 switches it off); reported as config.clock_settle_ms")
    ap.add_argument("--no-shapes-line", action="store_true",
                    help="skip the other widths in roofline.shapes (11008, 14336, 28672)")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also launch the library's plain copy kernel on one batch (known bytes), "
                         "the reference that scales rocprofv3 FETCH_SIZE / WRITE_SIZE readings")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (rows shard across GPUs with no "
              "communication; no multi-GPU figure is produced). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2605_29843_amd import harp, inputs as gi   # raises if libharp.so is missing

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    w = gi.workload(args.workload, n=args.rows)
    n, d, radices = w["n"], w["d"], w["radices"]
    bf16 = w["dtype"] == "bf16"
    esz = 2 if bf16 else 4
    plan = harp.Plan(d, radices, w["blocks"], w["signs"])

    def dev(a):
        if bf16:
            return torch.from_numpy(gi.bf16_bits(a).view(np.int16).copy()).view(torch.bfloat16).cuda()
        return torch.from_numpy(a).cuda()

    # pool of batches: same distribution, rows permuted per batch; > 512 MB in total
    batch_bytes = n * d * esz
    nbuf = max(2, int(np.ceil(640e6 / (3 * batch_bytes))))
    X0 = dev(w["X"])
    pool = []
    g = torch.Generator(device="cuda").manual_seed(0)
    for i in range(nbuf):
        Xi = X0 if i == 0 else X0[torch.randperm(n, device="cuda", generator=g)].contiguous()
        pool.append((Xi, torch.empty_like(Xi), torch.empty_like(Xi)))

    stream = torch.cuda.current_stream()

    def step(i):
        Xi, Yi, Zi = pool[i % nbuf]
        harp.harp_apply(plan, Xi, Yi, stream)
        harp.harp_apply_transpose(plan, Yi, Zi, stream)

    if args.settle_ms > 0:
        cnt0 = [0]

        def one0():
            step(cnt0[0])
            cnt0[0] += 1
        warm_clocks(one0, seconds=args.settle_ms * 1e-3)
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record(stream)
    for i in range(args.steps):
        step(args.warmup + i)
    ev1.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ev_ms = ev0.elapsed_time(ev1)

    # sanity of what was timed: round trip returns the input
    Xi, Yi, Zi = pool[(args.warmup + args.steps - 1) % nbuf]
    rt = float((Zi.float() - Xi.float()).abs().max() / Xi.float().abs().max())
    assert rt < (3e-2 if bf16 else 1e-4), f"round trip error {rt}"

    if args.calib_copy:
        for _ in range(3):   # harp_copy2d_kernel: reads and writes n*d*esz bytes each
            harp.harp_rotate_weight(None, None, pool[1][0], pool[1][1], stream=stream)
        torch.cuda.synchronize()

    def timed_us(fn, reps, settle=0.05):
        """Average duration of fn()'s launches, HIP events on the launch stream."""
        warm_clocks(fn, seconds=settle)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(reps):
            fn()
        e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / reps

    launches = 2 * args.steps
    kernel_us = ev_ms * 1e3 / launches                       # average launch duration (HIP events)
    param_bytes = plan.param_bytes()
    alg_bytes = n * d * 2 * esz + param_bytes                # per launch: read X, write Y, params once
    achieved = alg_bytes / (kernel_us * 1e-6) / 1e9
    ms_per_step = wall * 1e3 / args.steps
    rows_per_s = 2 * n * args.steps / wall

    out = {
        "metric": "HARP rotation rows/s (apply + apply_transpose), achieved HBM GB/s in roofline",
        "value": rows_per_s, "unit": "rows/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": args.workload, "n": n, "d": d, "radices": radices,
                   "io_dtype": w["dtype"], "kernel": plan.kernel_name(n), "batches_in_pool": nbuf,
                   "clock_settle_ms": args.settle_ms,
                   "step": "harp_apply + harp_apply_transpose on one batch"},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": None,
                     "kernel": KERNEL_SYMBOL.get(plan.kernel_name(n), plan.kernel_name(n)), "avg_launch_us": kernel_us,
                     "algorithmic_bytes_per_launch": alg_bytes, "param_bytes": param_bytes},
    }
    # Copy ceiling of this machine at this batch size: the library's plain copy kernel (reads and
    # writes n*d*esz bytes) on the same rotating batches, same event method.
    ccnt = [0]

    def copy_once():
        Xi, Yi, _ = pool[ccnt[0] % nbuf]
        harp.harp_rotate_weight(None, None, Xi, Yi, stream=stream)
        ccnt[0] += 1
    copy_us = timed_us(copy_once, 400)
    copy_gbs = 2 * n * d * esz / (copy_us * 1e-6) / 1e9
    out["roofline"]["copy_ceiling_gbs"] = copy_gbs
    out["roofline"]["copy_launch_us"] = copy_us
    out["roofline"]["frac_of_copy"] = achieved / copy_gbs
    out["roofline"]["shapes"] = {str(d): {
        "workload": args.workload, "n": n, "avg_launch_us": kernel_us, "achieved": achieved,
        "frac": achieved / HBM_PEAK_GBS, "kernels": [out["roofline"]["kernel"]], "launches_per_call": 1,
        "traffic_ratio": None}}
    if not args.no_shapes_line and args.rows is None and args.workload == "llama7b_4096_r2":
        # The other widths of the target: 2048 x 11008 = 2^8 * 43 (the second width the headline
        # metric is quoted at), 2048 x 14336 = 2^11 * 7 and 4096 x 28672 = 2^12 * 7, bf16, apply and
        # apply_transpose on rotating batches (> 640 MB of inputs and outputs).
        for wname in ("down_11008_r2x8_43", "ffn_14336_r2x11_7", "ffn70b_28672_r2x12_7"):
            w2 = gi.workload(wname)
            p2 = harp.Plan(w2["d"], w2["radices"], w2["blocks"], w2["signs"])
            X2 = dev(w2["X"])
            nb2 = max(2, int(np.ceil(640e6 / (3 * X2.numel() * X2.element_size()))))
            pool2 = [(X2 if i == 0 else X2.roll(i, 0).contiguous(), torch.empty_like(X2), torch.empty_like(X2))
                     for i in range(nb2)]
            c2 = [0]

            def step2():
                Xi, Yi, Zi = pool2[c2[0] % nb2]
                harp.harp_apply(p2, Xi, Yi, stream)
                harp.harp_apply_transpose(p2, Yi, Zi, stream)
                c2[0] += 1
            us2 = timed_us(step2, 300 if w2["d"] < 20000 else 100, settle=0.08) / 2   # per call
            Xi, Yi, Zi = pool2[(c2[0] - 1) % nb2]
            rt2 = float((Zi.float() - Xi.float()).abs().max() / Xi.float().abs().max())
            assert rt2 < 3e-2, f"{wname} round trip error {rt2}"
            alg2 = w2["n"] * w2["d"] * 4 + p2.param_bytes()
            ach2 = alg2 / (us2 * 1e-6) / 1e9
            kname2 = p2.kernel_name(w2["n"])
            out["roofline"]["shapes"][str(w2["d"])] = {
                "workload": wname, "n": w2["n"], "avg_launch_us": us2, "achieved": ach2,
                "frac": ach2 / HBM_PEAK_GBS, "rows_per_s": w2["n"] / (us2 * 1e-6),
                "kernels": KERNELS_OF.get(kname2, [kname2]), "path": kname2,
                "algorithmic_bytes_per_call": alg2, "traffic_ratio": None}
            del pool2, X2, Xi, Yi, Zi
            p2.destroy()
            torch.cuda.empty_cache()
    if args.x8 and args.rows is None and n * 8 * d * esz * 6 < 4e9:
        # The same kernel on 8 n rows (the batch repeated): 8 times the rows per workgroup, so the
        # start-up of a launch weighs an eighth as much.  Context for `frac`, not the headline.
        nb8 = 2
        big = [(X0.repeat(8, 1), None, None) for _ in range(nb8)]
        big = [(x, torch.empty_like(x), torch.empty_like(x)) for x, _, _ in big]

        def step8(i):
            Xi, Yi, Zi = big[i % nb8]
            harp.harp_apply(plan, Xi, Yi, stream)
            harp.harp_apply_transpose(plan, Yi, Zi, stream)
        cnt8 = [0]

        def one8():
            step8(cnt8[0])
            cnt8[0] += 1
        warm_clocks(one8)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for i in range(200):
            step8(i)
        e1.record(stream)
        torch.cuda.synchronize()
        us8 = e0.elapsed_time(e1) * 1e3 / 400
        ach8 = (8 * n * d * 2 * esz + param_bytes) / (us8 * 1e-6) / 1e9
        out["roofline"]["at_8x_rows"] = {"n": 8 * n, "avg_launch_us": us8, "achieved": ach8,
                                         "frac": ach8 / HBM_PEAK_GBS}
        del big
    tpath = os.path.join(ROOT, "profiles", f"traffic_{args.workload}.json")
    if os.path.exists(tpath) and args.rows is None:
        with open(tpath) as f:
            tj = json.load(f)
        out["roofline"]["traffic"] = tj.get("traffic_bytes_per_launch")
        out["roofline"]["traffic_source"] = "profiles/" + os.path.basename(tpath)
        if out["roofline"]["traffic"]:
            out["roofline"]["shapes"][str(d)]["traffic_ratio"] = out["roofline"]["traffic"] / alg_bytes
    for key, sh in out["roofline"]["shapes"].items():
        tp = os.path.join(ROOT, "profiles", f"traffic_{sh['workload']}.json")
        if key != str(d) and os.path.exists(tp):
            with open(tp) as f:
                tj = json.load(f)
            if tj.get("traffic_bytes_per_launch"):
                sh["traffic_ratio"] = tj["traffic_bytes_per_launch"] / sh["algorithmic_bytes_per_call"]
                sh["traffic_source"] = "profiles/" + os.path.basename(tp)
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(w, sample_rows=min(n, 2048))
    if args.extra:
        for name in ("llama7b_4096_r8", "down_11008_r2x8_43", "ffn_14336_r2x11_7", "ffn70b_28672_r2x12_7",
                     "llama13b_5120_r2x10_5", "ffn13b_13824_r2x9_27", "hidden70b_8192_r2"):
            try:
                we = gi.workload(name)
                pe = harp.Plan(we["d"], we["radices"], we["blocks"], we["signs"])
                Xe = dev(we["X"])
                # rotate through > 640 MB of inputs and outputs, as the main measurement does
                nb = max(2, int(np.ceil(640e6 / (2 * Xe.numel() * Xe.element_size()))))
                Xs = [Xe] + [Xe.clone() for _ in range(nb - 1)]
                Ys = [torch.empty_like(Xe) for _ in range(nb)]
                cnt = [0]

                def one():
                    harp.harp_apply(pe, Xs[cnt[0] % nb], Ys[cnt[0] % nb], stream)
                    cnt[0] += 1
                warm_clocks(one)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                reps = 200
                for i in range(reps):
                    harp.harp_apply(pe, Xs[i % nb], Ys[i % nb], stream)
                e1.record(stream)
                torch.cuda.synchronize()
                del Xs, Ys
                us = e0.elapsed_time(e1) * 1e3 / reps
                gb = (we["n"] * we["d"] * 4 + pe.param_bytes()) / (us * 1e-6) / 1e9
                print(f"[extra] {name}: {us:.1f} us/apply, {gb:.0f} GB/s ({gb / HBM_PEAK_GBS:.1%}), "
                      f"{we['n'] / (us * 1e-6):.3e} rows/s", file=sys.stderr, flush=True)
                pe.destroy()
            except Exception as e:  # noqa: BLE001
                print(f"[extra] {name}: {e}", file=sys.stderr, flush=True)
        try:   # two-sided weight rotation at the 70B FFN shape (weights drawn on the device)
            do, di = 8192, 28672
            bu, su = gi.processor(do, [2] * 13, config=5, salt=1)
            bv, sv = gi.processor(di, [2] * 12 + [7], config=5, salt=2)
            pu, pv = harp.Plan(do, [2] * 13, bu, su), harp.Plan(di, [2] * 12 + [7], bv, sv)
            Wm = (torch.randn(do, di, device="cuda") * 0.02).to(torch.bfloat16)
            Wo = torch.empty_like(Wm)
            ws = torch.empty(harp.harp_rotate_weight_workspace_size(pu, pv, do, di, harp.HARP_BF16),
                             dtype=torch.uint8, device="cuda")
            for _ in range(8):
                harp.harp_rotate_weight(pu, pv, Wm, Wo, ws, stream)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(10):
                harp.harp_rotate_weight(pu, pv, Wm, Wo, ws, stream)
            e1.record(stream)
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / 10
            gb = 4 * do * di * 2 / (us * 1e-6) / 1e9   # two sides, each reads and writes W once
            print(f"[extra] rotate_weight 8192 x 28672 bf16: {us:.0f} us, {gb:.0f} GB/s "
                  f"({gb / HBM_PEAK_GBS:.1%})", file=sys.stderr, flush=True)
            e0.record(stream)
            for _ in range(10):
                harp.harp_rotate_weight_inverse(pu, pv, Wm, Wo, ws, stream)
            e1.record(stream)
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / 10
            print(f"[extra] rotate_weight_inverse 8192 x 28672 bf16: {us:.0f} us", file=sys.stderr, flush=True)
        except Exception as e:  # noqa: BLE001
            print(f"[extra] rotate_weight: {e}", file=sys.stderr, flush=True)
        try:   # gradient with respect to the blocks at the benchmark shape
            Gd = torch.randn(n, d, device="cuda").to(X0.dtype)
            wsz = harp.harp_grad_blocks_workspace_size(plan, n)
            wsg = torch.empty(wsz, dtype=torch.uint8, device="cuda")
            warm_clocks(lambda: harp.harp_grad_blocks(plan, X0, Gd, True, wsg, stream))
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(50):
                harp.harp_grad_blocks(plan, X0, Gd, True, wsg, stream)
            e1.record(stream)
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / 50
            # algorithmic bytes: read X and G, write dX (caller's type) and the block gradients
            gb = (3 * n * d * esz + sum(d * b for b in radices) * 4) / (us * 1e-6) / 1e9
            print(f"[extra] grad_blocks {n} x {d} {w['dtype']}: {us:.0f} us, {gb:.0f} GB/s algorithmic "
                  f"({gb / HBM_PEAK_GBS:.1%})", file=sys.stderr, flush=True)
        except Exception as e:  # noqa: BLE001
            print(f"[extra] grad_blocks: {e}", file=sys.stderr, flush=True)
        try:   # the same at 2048 x 11008 (eight radix-2 stages and the radix-43 stage)
            dg, rg = 11008, [2] * 8 + [43]
            bg, sg = gi.processor(dg, rg, config=2, salt=3)
            pg = harp.Plan(dg, rg, bg, sg)
            Xg = torch.randn(2048, dg, device="cuda").to(torch.bfloat16)
            Gg = torch.randn(2048, dg, device="cuda").to(torch.bfloat16)
            wsg = torch.empty(harp.harp_grad_blocks_workspace_size(pg, 2048), dtype=torch.uint8, device="cuda")
            for _ in range(5):
                harp.harp_grad_blocks(pg, Xg, Gg, True, wsg, stream)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(20):
                harp.harp_grad_blocks(pg, Xg, Gg, True, wsg, stream)
            e1.record(stream)
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / 20
            gb = (3 * 2048 * dg * 2 + sum(dg * b for b in rg) * 4) / (us * 1e-6) / 1e9
            print(f"[extra] grad_blocks 2048 x {dg} bf16: {us:.0f} us, {gb:.0f} GB/s algorithmic "
                  f"({gb / HBM_PEAK_GBS:.1%})", file=sys.stderr, flush=True)
            pg.destroy()
        except Exception as e:  # noqa: BLE001
            print(f"[extra] grad_blocks 11008: {e}", file=sys.stderr, flush=True)
    if args.shapes:
        r2 = {4096: [2] * 12, 5120: [2] * 10 + [5], 8192: [2] * 13, 11008: [2] * 8 + [43],
              13824: [2] * 9 + [3, 3, 3], 14336: [2] * 11 + [7], 28672: [2] * 12 + [7]}
        g8 = {4096: [8] * 4, 5120: [8, 8, 8, 5, 2], 8192: [8, 8, 8, 8, 2], 11008: [8, 8, 4, 43],
              13824: [8, 8, 8, 3, 3, 3], 14336: [8, 8, 8, 7, 4], 28672: [8, 8, 8, 8, 7]}
        rng = np.random.default_rng(0)

        def timed(fn, reps):
            warm_clocks(fn, seconds=0.03)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(reps):
                fn()
            e1.record(stream)
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) * 1e3 / reps

        for fam, sched in (("radix-2", r2), ("greedy-8", g8)):
            for dd, rr in sched.items():
                ps = harp.Plan(dd, rr, gi.make_blocks(dd, rr, "orth", rng), gi.make_signs(dd, rng))
                for tdt in (torch.bfloat16, torch.float32):
                    nb = max(2, min(8, int(400e6 / (2048 * dd * tdt.itemsize))))
                    Xs = [torch.randn(2048, dd, device="cuda").to(tdt) for _ in range(nb)]
                    Ys = [torch.empty_like(x) for x in Xs]
                    cnt = [0]

                    def fwd():
                        harp.harp_apply(ps, Xs[cnt[0] % nb], Ys[cnt[0] % nb], stream)
                        cnt[0] += 1

                    def trn():
                        harp.harp_apply_transpose(ps, Xs[cnt[0] % nb], Ys[cnt[0] % nb], stream)
                        cnt[0] += 1
                    tf, tt = timed(fwd, 100), timed(trn, 100)
                    gbs = 2 * 2048 * dd * tdt.itemsize / 1e3   # bytes read + written, per us -> GB/s
                    print(f"[shapes] {fam:8s} d={dd:6d} {str(tdt)[6:]:8s} apply {tf:7.1f} us "
                          f"({gbs / tf:5.0f} GB/s)  transpose {tt:7.1f} us ({gbs / tt:5.0f} GB/s)  "
                          f"[{ps.kernel_name(2048, harp.HARP_BF16 if tdt == torch.bfloat16 else harp.HARP_F32)}]",
                          file=sys.stderr, flush=True)
                    del Xs, Ys
                ps.destroy()
            for do, di in ((4096, 4096), (11008, 4096), (4096, 11008), (5120, 13824), (13824, 5120),
                           (14336, 4096), (4096, 14336), (8192, 28672), (28672, 8192)):
                pu = harp.Plan(do, sched[do], gi.make_blocks(do, sched[do], "orth", rng),
                               gi.make_signs(do, rng))
                pv = harp.Plan(di, sched[di], gi.make_blocks(di, sched[di], "orth", rng),
                               gi.make_signs(di, rng))
                Wm = (torch.randn(do, di, device="cuda") * 0.02).to(torch.bfloat16)
                Wo = torch.empty_like(Wm)
                ws = torch.empty(max(1, harp.harp_rotate_weight_workspace_size(pu, pv, do, di,
                                                                               harp.HARP_BF16)),
                                 dtype=torch.uint8, device="cuda")
                tf = timed(lambda: harp.harp_rotate_weight(pu, pv, Wm, Wo, ws, stream), 10)
                ti = timed(lambda: harp.harp_rotate_weight_inverse(pu, pv, Wm, Wo, ws, stream), 10)
                print(f"[shapes] {fam:8s} rotate_weight W[{do} x {di}] bf16 {tf:7.0f} us  "
                      f"inverse {ti:7.0f} us", file=sys.stderr, flush=True)
                del Wm, Wo, ws
                pu.destroy()
                pv.destroy()
    if args.shapes:
        # Kronecker fallback against Mixed-Radix (speed only; the paper compares their accuracy):
        # (H~_K / sqrt(K)) (x) T_{n2} as a plan with tied parameters, the same processor expanded to
        # an ordinary plan, and the Mixed-Radix radix-2 chain of the same width; bf16, n = 2048.
        rngk = np.random.default_rng(1)

        def timed2(fn, reps=100):
            warm_clocks(fn, seconds=0.03)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(reps):
                fn()
            e1.record(stream)
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) * 1e3 / reps

        for dd, K, n2, mixed in ((12288, 12, 1024, [2] * 12 + [3]), (14336, 28, 512, [2] * 11 + [7]),
                                 (28672, 28, 1024, [2] * 12 + [7])):
            r2k = [2] * int(np.log2(n2))
            b2 = gi.make_blocks(n2, r2k, "orth", rngk)
            sg = gi.make_signs(dd, rngk)
            Hk = gi.hadamard_table(K)
            rk, bk = harp.harp_kronecker_blocks(Hk, n2, r2k, b2)
            plans = (("kronecker tied", harp.Plan.kronecker(Hk, n2, r2k, b2, sg)),
                     ("kronecker expanded", harp.Plan(dd, rk, bk, sg)),
                     ("mixed-radix", harp.Plan(dd, mixed, gi.make_blocks(dd, mixed, "orth", rngk), sg)))
            nb = max(2, min(8, int(400e6 / (2048 * dd * 2))))
            Xs = [torch.randn(2048, dd, device="cuda").to(torch.bfloat16) for _ in range(nb)]
            Ys = [torch.empty_like(x) for x in Xs]
            cnt = [0]
            for nm, pk in plans:
                def fwd():
                    harp.harp_apply(pk, Xs[cnt[0] % nb], Ys[cnt[0] % nb], stream)
                    cnt[0] += 1

                def trn():
                    harp.harp_apply_transpose(pk, Xs[cnt[0] % nb], Ys[cnt[0] % nb], stream)
                    cnt[0] += 1
                tf, tt = timed2(fwd), timed2(trn)
                print(f"[shapes] d={dd:6d} = {K} x {n2} {nm:19s} apply {tf:7.1f} us  transpose {tt:7.1f} us  "
                      f"parameters {pk.param_bytes() / 1e6:6.2f} MB  [{pk.kernel_name(2048)}]",
                      file=sys.stderr, flush=True)
                pk.destroy()
            del Xs, Ys
    if args.shapes or args.int8:
        # Int8-stored parameters (appendix "Int8 storage of HARP parameters"): the same codes as a
        # plan whose blocks are rebuilt once on the host, and as a plan whose chain kernel
        # rebuilds them from the int8 image in every launch; bf16, n = 2048.
        rngq = np.random.default_rng(2)

        def timed3(fn, reps=100):
            warm_clocks(fn, seconds=0.03)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(reps):
                fn()
            e1.record(stream)
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) * 1e3 / reps

        for dd, rr in ((4096, [8] * 4), (8192, [8] * 4 + [2])):
            th = [(0.5 * rngq.standard_normal((dd // b, b * (b - 1) // 2))).astype(np.float32) for b in rr]
            cq, sq = harp.harp_theta_quantize_int8(dd, rr, th)
            sg = gi.make_signs(dd, rngq)
            Xs = [torch.randn(2048, dd, device="cuda").to(torch.bfloat16) for _ in range(8)]
            Ys = [torch.empty_like(x) for x in Xs]
            cnt = [0]
            for nm, fl in (("blocks rebuilt at plan creation", 0),
                           ("blocks rebuilt in the kernel", harp.HARP_THETA_IN_KERNEL)):
                pq = harp.Plan.from_theta_int8(dd, rr, cq, sq, None, sg, flags=fl)

                def fwd():
                    harp.harp_apply(pq, Xs[cnt[0] % 8], Ys[cnt[0] % 8], stream)
                    cnt[0] += 1

                def trn():
                    harp.harp_apply_transpose(pq, Xs[cnt[0] % 8], Ys[cnt[0] % 8], stream)
                    cnt[0] += 1
                tf, tt = timed3(fwd), timed3(trn)
                print(f"[shapes] int8 theta d={dd:6d} {str(rr):22s} {nm:32s} apply {tf:7.1f} us  "
                      f"transpose {tt:7.1f} us  [{pq.kernel_name(2048)}]", file=sys.stderr, flush=True)
                pq.destroy()
            del Xs, Ys
    if args.decode:
        for dd, rr in ((4096, [2] * 12), (12288, [2] * 12 + [3]), (14336, [2] * 11 + [7])):
            bb, ss = gi.processor(dd, rr, config=4)
            pd_ = harp.Plan(dd, rr, bb, ss)
            for nn in (1, 8, 32, 64):
                Xd = torch.randn(nn, dd, device="cuda").to(torch.bfloat16)
                Yd = torch.empty_like(Xd)
                for _ in range(20):
                    harp.harp_apply(pd_, Xd, Yd, stream)
                torch.cuda.synchronize()
                evs = [torch.cuda.Event(enable_timing=True) for _ in range(1001)]
                evs[0].record(stream)
                for i in range(1000):
                    harp.harp_apply(pd_, Xd, Yd, stream)
                    evs[i + 1].record(stream)
                torch.cuda.synchronize()
                med = float(np.median([evs[i].elapsed_time(evs[i + 1]) for i in range(1000)])) * 1e3
                tg = float("nan")
                try:
                    side = torch.cuda.Stream()
                    side.wait_stream(stream)
                    with torch.cuda.stream(side):
                        harp.harp_apply(pd_, Xd, Yd, side)    # warms the plan's intermediate on it
                    stream.wait_stream(side)
                    g = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(g, stream=side):      # capture on the warmed stream
                        for _ in range(20):
                            harp.harp_apply(pd_, Xd, Yd, side)
                    for _ in range(5):
                        g.replay()
                    torch.cuda.synchronize()
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                    for _ in range(50):
                        g.replay()
                    e1.record()
                    torch.cuda.synchronize()
                    tg = e0.elapsed_time(e1) * 1e3 / (50 * 20)
                except Exception as e:  # noqa: BLE001
                    print(f"[decode] graph capture failed: {str(e)[:100]}", file=sys.stderr, flush=True)
                byt = nn * dd * 4 + pd_.param_bytes()      # parameters dominate at these sizes
                print(f"[decode] d={dd} n={nn} {pd_.kernel_name(nn)}: median {med:.2f} us/call "
                      f"({byt / (med * 1e-6) / 1e9:.0f} GB/s incl. parameters), "
                      f"in a HIP graph {tg:.2f} us/launch", file=sys.stderr, flush=True)
            pd_.destroy()
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
