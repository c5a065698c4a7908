#!/usr/bin/env python3
"""Throughput of the fused permute + block-Hadamard + quantize path on one MI355X.

A step is one call of perq_permute_rotate_quant on a T-token batch already resident in HBM
(gather through the calibrated permutation, rotation, scale, round, pack).  The calibration
that produces the permutation (perq_colabs_mean on the device, the greedy on the host) runs
once before the timed region, as it does once per layer in the method, and is reported in
its own field.  Prints ONE JSON line on stdout.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, vendor figure

WORKLOADS = {
    # name: (generator key, b, fmt, use calibrated perm)
    "llama8b_d4096_b128_int4_perm": ("llama8b_d4096", 128, "int4", True),
    "llama8b_d4096_b4096_int4_perm": ("llama8b_d4096", 4096, "int4", True),
    "llama8b_d14336_b128_int4_perm": ("llama8b_d14336", 128, "int4", True),
    "llama8b_d14336_b2048_int4_perm": ("llama8b_d14336", 2048, "int4", True),
    # full-vector rotation at the Llama3 1B/3B width (Table 3, first row), on the d = 8192 workloads
    "calib_apply_full_mxfp4": ("calib_apply", 8192, "mxfp4", False),
    "llama1b_down_full_int4": ("llama1b_down", 8192, "int4", False),
    # full-vector rotation at the Llama3-8B width, 14336 = 2^9 * 28 (Appendix A.1); a permutation
    # does not change the bound of one block that spans the row, so P = I
    "llama8b_d14336_full_int4": ("llama8b_d14336", 14336, "int4", False),
    # the same at the Qwen3 8B and 4B widths, 12288 = 2^10 * 12 and 9728 = 2^7 * 76
    "qwen3_d12288_full_int4": ("qwen3_d12288", 12288, "int4", False),
    "qwen3_d9728_full_int4": ("qwen3_d9728", 9728, "int4", False),
    "llama1b_down_b32_int4_perm": ("llama1b_down", 32, "int4", True),
    "block_vs_full_b32_mxfp4": ("block_vs_full", 32, "mxfp4", False),
    "block_vs_full_b2048_mxfp4": ("block_vs_full", 2048, "mxfp4", False),
    "calib_apply_b32_mxfp4_perm": ("calib_apply", 32, "mxfp4", True),
    "calib_apply_b16_mxfp4_perm": ("calib_apply", 16, "mxfp4", True),
    "llama8b_d4096_b128_int4asym_perm": ("llama8b_d4096", 128, "int4_asym", True),
    "llama8b_d4096_b128_fp4token_perm": ("llama8b_d4096", 128, "fp4_token", True),
}
DEFAULT = "llama8b_d4096_b128_int4_perm"


def algorithmic_bytes(T: int, d: int, fmt: str) -> int:
    """What the method itself must move per launch: bf16 in, nibbles out, scales out."""
    scales = {"int4": 4 * T, "fp4_token": 4 * T, "int4_asym": 8 * T, "mxfp4": T * d // 32}[fmt]
    return T * d * 2 + T * d // 2 + scales


def read_traffic(name: str, algo: str = "auto", identity: bool = False, arranged: bool = False):
    """(HBM bytes per launch, where from) out of the committed rocprofv3 --pmc summary of this
    workload, if there is one: the figure is that of the profiled build, not of this run, so the
    file and the kernel line it was taken for are reported with it."""
    if identity:
        name = name.replace("_perm", "_identity")
    elif arranged:
        name = name.replace("_perm", "_perm_arranged")
    if algo == "butterfly":
        name += "_butterfly"
    rel = os.path.join("profiles", f"hbm_traffic_{name}.txt")
    path = os.path.join(ROOT, rel)
    if not os.path.exists(path):
        return None, None
    value, kernel = None, None
    for line in open(path):
        if line.startswith("HBM_BYTES_PER_LAUNCH="):
            value = float(line.split("=", 1)[1])
        if kernel is None and " calls " in line and "perq::" in line and "colabs" not in line:
            kernel = " ".join(line.split())
    return value, {"file": rel, "kernel_line": kernel, "note": "committed rocprofv3 summary, not measured in this run"}


def prepare_placement(perm_np, b, dev):
    """The form perq_perm_prepare writes for this permutation (host, once per layer: the operand offsets
    in the kernel's lane order and, for wide rows, the LDS placement): device copy, and what the
    placement does to the bank conflicts of the operand reads.  None where the shape's kernel has no
    such gather."""
    from paper_2601_22347_amd import binding
    h0 = time.perf_counter()
    try:
        table, before, after, reads = binding.perq_perm_prepare(perm_np, b)
    except binding.PerqError:
        return None, None
    ms = (time.perf_counter() - h0) * 1e3
    placed = perm_np.size > 8192        # narrower rows keep the fixed layout
    return binding.placement_to_device(table, dev), {"lds_passes_per_read": [before / reads, (after if placed else before) / reads],
                                                     "prepare_host_ms": ms}


# The configurations the bandwidth target (T >= 16384, d >= 4096) is quoted on: the headline and the
# five others, every one timed by the default invocation.
TARGET_SHAPES = ["llama8b_d4096_b128_int4_perm", "llama8b_d4096_b4096_int4_perm", "llama8b_d14336_b128_int4_perm",
                 "llama8b_d14336_b2048_int4_perm", "calib_apply_b32_mxfp4_perm", "calib_apply_b16_mxfp4_perm"]


def time_target_shape(name, steps, warmup, pool_bytes, algo, check, prepared=True):
    """One of the other target-size workloads: calibrate, time `steps` launches with HIP events over
    cycled buffer sets, compare sampled rows with the oracle.  Returns a dict for the report."""
    import torch
    from paper_2601_22347_amd import binding, synth
    key, b, fmt, use_perm = WORKLOADS[name]
    wl = synth.ALL[key]()
    T, d = wl.T, wl.d
    dev = torch.device("cuda:0")
    x_bits = wl.apply_rows_parallel()
    perm_np = perm_t = None
    place_t, place_info = None, None
    if use_perm:
        a_np = binding.perq_colabs_mean(binding.bits_to_device(wl.calib_rows())).cpu().numpy()
        perm_np = binding.perq_massdiff_perm(a_np, b)
        perm_t = torch.from_numpy(perm_np).to(dev)
        if prepared and algo == "auto":
            place_t, place_info = prepare_placement(perm_np, b, dev)
    per_set = T * d * 2 + T * d // 2
    nsets = max(2, int(np.ceil(pool_bytes / per_set)))
    x0 = binding.bits_to_device(x_bits, dev)
    xs = [x0] + [x0.clone() for _ in range(nsets - 1)]
    outs = [binding.alloc_outputs(T, d, fmt, dev) for _ in range(nsets)]
    stream = torch.cuda.current_stream()

    def step(i):
        k = i % nsets
        binding.perq_permute_rotate_quant(xs[k], perm_t, b, fmt, codes=outs[k][0], scales=outs[k][1],
                                          stream=stream, algo=algo, placement=place_t)
    t_ramp = time.perf_counter()
    while time.perf_counter() - t_ramp < 0.15:
        for i in range(20):
            step(i)
        torch.cuda.synchronize()
    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record(stream)
    for i in range(steps):
        step(i)
    ev1.record(stream)
    torch.cuda.synchronize()
    kern_ms = ev0.elapsed_time(ev1) / steps
    alg = algorithmic_bytes(T, d, fmt)
    res = {"workload": name, "T": T, "d": d, "b": b, "fmt": fmt, "placement": place_info, "kernel_ms": kern_ms, "algorithmic_bytes": alg,
           "achieved_GBs": alg / (kern_ms * 1e-3) / 1e9, "frac": alg / (kern_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
           "tokens_per_s": T / (kern_ms * 1e-3)}
    if check:
        import parity
        rng = np.random.default_rng(0)
        rows = np.unique(np.concatenate([np.arange(16), T - 1 - np.arange(16), rng.choice(T, size=32, replace=False)]))
        rt = torch.from_numpy(rows).to(dev)
        last = (steps - 1) % nsets
        rep = parity.compare_apply(x_bits[rows], perm_np, b, fmt, outs[last][0][rt].cpu().numpy(),
                                   outs[last][1][rt].cpu().numpy())
        res["check"] = dict(rep.summary(), rows=int(rows.size), ok=rep.ok())
    del xs, outs, x0
    torch.cuda.empty_cache()
    return res


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--workload", default=DEFAULT, choices=sorted(WORKLOADS))
    ap.add_argument("--algo", default="auto", choices=["auto", "butterfly", "mfma"])
    ap.add_argument("--pool-bytes", type=float, default=1.5e9,
                    help="input+output bytes cycled through so that no step re-reads cached data")
    ap.add_argument("--identity", action="store_true", help="run the workload with P = I (no gather)")
    ap.add_argument("--arranged", action="store_true",
                    help="time the calibrated permutation in the order perq_perm_arrange gives its blocks")
    ap.add_argument("--no-placement", action="store_true",
                    help="call the fused path without the prepared form of perq_perm_prepare")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-check", action="store_true")
    ap.add_argument("--no-context", action="store_true",
                    help="skip the single-buffer-set and device-copy figures and the other target-size workloads")
    ap.add_argument("--no-target-shapes", action="store_true",
                    help="skip timing the other target-size workloads after the headline")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (token rows would be sharded across GPUs "
              "with no exchange; nothing here uses a second device). Use --gpus 1.", file=sys.stderr)
        return 2

    import torch
    from paper_2601_22347_amd import binding, synth
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    binding.load()

    key, b, fmt, use_perm = WORKLOADS[args.workload]
    use_perm = use_perm and not args.identity
    wl = synth.ALL[key]()
    T, d = wl.T, wl.d
    dev = torch.device("cuda:0")

    t0 = time.perf_counter()
    x_bits = wl.apply_rows_parallel()
    gen_s = time.perf_counter() - t0

    # ---- calibration: colabs mean on the device, greedy on the host (once, untimed region) ----
    calib = None
    perm_np = perm_t = None
    place_t = None
    if use_perm:
        xc = binding.bits_to_device(wl.calib_rows())
        a_t = binding.perq_colabs_mean(xc)           # warm-up
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10):
            a_t = binding.perq_colabs_mean(xc, out=a_t)
        e1.record()
        torch.cuda.synchronize()
        a_np = a_t.cpu().numpy()
        h0 = time.perf_counter()
        perm_np = binding.perq_massdiff_perm(a_np, b)
        greedy_ms = (time.perf_counter() - h0) * 1e3
        assert binding.perq_perm_validate(perm_np)
        if args.arranged:
            perm_np = binding.perq_perm_arrange(perm_np, b)
            assert binding.perq_perm_validate(perm_np)
        perm_t = torch.from_numpy(perm_np).to(dev)
        calib = {"colabs_mean_tokens": wl.calib_tokens, "colabs_mean_ms": e0.elapsed_time(e1) / 10,
                 "greedy_host_ms": greedy_ms}
        if not args.no_placement and args.algo == "auto":
            place_t, place_info = prepare_placement(perm_np, b, dev)
            calib["placement"] = place_info
        del xc

    # ---- buffer pool larger than the last-level cache ----------------------------------------
    per_set = T * d * 2 + T * d // 2
    nsets = max(2, int(np.ceil(args.pool_bytes / per_set)))
    x0 = binding.bits_to_device(x_bits, dev)
    xs = [x0] + [x0.clone() for _ in range(nsets - 1)]
    outs = [binding.alloc_outputs(T, d, fmt, dev) for _ in range(nsets)]
    stream = torch.cuda.current_stream()

    def step(i):
        k = i % nsets
        binding.perq_permute_rotate_quant(xs[k], perm_t, b, fmt, codes=outs[k][0], scales=outs[k][1],
                                          stream=stream, algo=args.algo, placement=place_t)

    # The device needs some tens of milliseconds of load before its clocks settle (the first
    # ~100 launches run 1.1-2.5x slower); run it up on the same work before the warm-up steps so
    # that a small --warmup still times the steady state.  Not counted, not timed.
    t_ramp = time.perf_counter()
    while time.perf_counter() - t_ramp < 0.15:
        for i in range(50):
            step(i)
        torch.cuda.synchronize()
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    w0 = time.perf_counter()
    ev0.record(stream)
    for i in range(args.steps):
        step(i)
    ev1.record(stream)
    torch.cuda.synchronize()
    wall_s = time.perf_counter() - w0
    kern_ms = ev0.elapsed_time(ev1) / args.steps        # one kernel per step, back to back
    ms_per_step = wall_s * 1e3 / args.steps
    tokens_per_s = T / (ms_per_step * 1e-3)

    alg_bytes = algorithmic_bytes(T, d, fmt)
    achieved = alg_bytes / (kern_ms * 1e-3) / 1e9

    # ---- context figures (untimed region of the report): one buffer set only, which stays in the
    # 256 MB last-level cache when it is small enough, and the box's plain device copy ----------
    def timed(fn, n):
        for i in range(max(10, n // 10)):
            fn(i)
        torch.cuda.synchronize()
        a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a0.record(stream)
        for i in range(n):
            fn(i)
        a1.record(stream)
        torch.cuda.synchronize()
        return a0.elapsed_time(a1) / n
    context = None
    if not args.no_context:
        one_set_ms = timed(lambda i: binding.perq_permute_rotate_quant(xs[0], perm_t, b, fmt, codes=outs[0][0],
                                                                       scales=outs[0][1], stream=stream, algo=args.algo,
                                                                       placement=place_t),
                           min(args.steps, 300))
        if place_t is not None:
            # the same launch with the plain call (perm turned into addresses by every launch, fixed LDS
            # layout): all buffer sets, in turns
            def all_sets_pl(pl):
                return timed(lambda i: binding.perq_permute_rotate_quant(
                    xs[i % nsets], perm_t, b, fmt, codes=outs[i % nsets][0], scales=outs[i % nsets][1],
                    stream=stream, algo=args.algo, placement=pl), min(args.steps, 300))
            turns_pl = [(all_sets_pl(None), all_sets_pl(place_t)) for _ in range(3)]
            placement_ab = {"plain_call_kernel_ms": float(np.mean([t[0] for t in turns_pl])),
                            "prepared_kernel_ms": float(np.mean([t[1] for t in turns_pl]))}
        cp_src, cp_dst = xs[0].view(torch.uint8).reshape(-1), xs[1].view(torch.uint8).reshape(-1)
        copy_ms = timed(lambda i: cp_dst.copy_(cp_src), 50)
        context = {"placement_ab": placement_ab if place_t is not None else None,
                   "single_buffer_set_ms": one_set_ms,
                   "single_buffer_set_note": "same call on one input/output set (%.0f MB; cache resident if well under "
                                             "256 MB)" % (per_set / 1e6),
                   "device_copy_GBs": 2 * cp_src.numel() / (copy_ms * 1e-3) / 1e9}
        # Launch time against the number of rows (the first T' rows of every buffer set, in turns): the
        # fixed cost of a launch (start-up and drain, which no row accounts for) and the kernel's steady
        # rate, from a least-squares line through four points.  The last point is the full workload, so
        # the output buffers hold the timed configuration's results afterwards.
        if T >= 2048:
            pts = []
            for frac4 in (1, 2, 3, 4):
                Tp = T * frac4 // 4
                ms = timed(lambda i: binding.perq_permute_rotate_quant(
                    xs[i % nsets][:Tp], perm_t, b, fmt, codes=outs[i % nsets][0][:Tp], scales=outs[i % nsets][1][:Tp],
                    stream=stream, algo=args.algo, placement=place_t), min(args.steps, 300))
                pts.append((Tp, ms * 1e3))
            A = np.array([[1.0, tp] for tp, _ in pts])
            (fixed_us, us_per_row), *_ = np.linalg.lstsq(A, np.array([u for _, u in pts]), rcond=None)
            steady = algorithmic_bytes(T, d, fmt) / T / (us_per_row * 1e-6) / 1e9 if us_per_row > 0 else None
            context["launch_model"] = {"points_rows_us": [[int(tp), float(u)] for tp, u in pts],
                                       "fixed_us": float(fixed_us), "ns_per_row": float(us_per_row * 1e3),
                                       "steady_GBs": steady, "steady_frac": steady / HBM_PEAK_GBS if steady else None,
                                       "note": "time = fixed + rows * per-row: the fixed part is start-up and drain of a launch"}
        if perm_t is not None and not args.arranged:
            # the same blocks in the order perq_perm_arrange gives them (fewer LDS bank conflicts in
            # the operand gather): all buffer sets, as in the timed region; not the headline value
            arranged = binding.perq_perm_arrange(perm_np, b)
            if not np.array_equal(arranged, perm_np):
                arr_t = torch.from_numpy(arranged).to(dev)

                def all_sets(pt):
                    return timed(lambda i: binding.perq_permute_rotate_quant(
                        xs[i % nsets], pt, b, fmt, codes=outs[i % nsets][0], scales=outs[i % nsets][1],
                        stream=stream, algo=args.algo), min(args.steps, 300))
                # in turns, so that both see the same state of the device
                turns = [(all_sets(perm_t), all_sets(arr_t)) for _ in range(3)]
                as_is_ms = float(np.mean([t[0] for t in turns]))
                arr_ms = float(np.mean([t[1] for t in turns]))
                p0, r0 = binding.perq_perm_gather_cost(perm_np, b)
                p1, _ = binding.perq_perm_gather_cost(arranged, b)
                context["arranged_perm"] = {"kernel_ms": arr_ms, "as_given_kernel_ms": as_is_ms, "frac": alg_bytes / (arr_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                            "lds_passes_per_read": [p0 / r0, p1 / r0],
                                            "note": "perq_perm_arrange: same blocks, order inside a block chosen for the LDS gather"}
                # the output buffers hold the timed configuration's results again (they are compared
                # with the oracle below)
                for i in range(nsets):
                    step(i)
                torch.cuda.synchronize()

    # ---- the oracle on the host cores, bounded sample (the only part of this file that runs it):
    #      timed as the CPU baseline, and the timed launch configuration is compared with it on
    #      sampled rows ---------------------------------------------------------------------------
    cpu = None
    check = None
    if not args.no_cpu_baseline:
        from oracle import perq_oracle as orc
        if not args.no_check:
            import parity
            rng = np.random.default_rng(0)
            rows = np.unique(np.concatenate([np.arange(32), T - 1 - np.arange(32),
                                             rng.choice(T, size=64, replace=False), wl.massive_rows[:8]]))
            codes = outs[(args.steps - 1) % nsets][0][torch.from_numpy(rows).to(dev)].cpu().numpy()
            sc = outs[(args.steps - 1) % nsets][1][torch.from_numpy(rows).to(dev)].cpu().numpy()
            rep = parity.compare_apply(x_bits[rows], perm_np, b, fmt, codes, sc)
            check = dict(rep.summary(), rows=int(rows.size), ok=rep.ok())
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = 1
        n = 256
        c0 = time.perf_counter()
        orc.perq_apply(x_bits[:n], perm_np, b, fmt)
        per_row = (time.perf_counter() - c0) / n
        n2 = int(min(T, max(n, 12.0 / max(per_row, 1e-9))))
        c0 = time.perf_counter()
        for s in range(0, n2, 2048):
            orc.perq_apply(x_bits[s:min(n2, s + 2048)], perm_np, b, fmt)
        cpu_s = time.perf_counter() - c0
        pow2 = b & (b - 1) == 0
        how = "explicit H_b product" if pow2 else "explicit product, one Kronecker factor of H_b at a time"
        cpu = {"value": n2 / cpu_s, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
               "sample": f"first {n2} tokens of the workload, fp64 NumPy, {how}, {cpu_s:.1f} s"}
        if pow2 and b >= 2048:
            # the oracle's second evaluation (fp64 radix-2 butterflies) on the same rows, for scale:
            # the explicit product costs O(d b) per token, this one O(d log b)
            n3 = min(n2, 4096)
            c0 = time.perf_counter()
            for s in range(0, n3, 2048):
                orc.perq_apply(x_bits[s:min(n3, s + 2048)], perm_np, b, fmt, rotate=orc.fwht_f64)
            f_s = time.perf_counter() - c0
            cpu["butterfly_variant"] = {"value": n3 / f_s, "unit": "tokens/s",
                                        "sample": f"first {n3} tokens, fp64 radix-2 butterflies, {f_s:.1f} s"}

    traffic, traffic_source = read_traffic(args.workload, args.algo, args.identity, args.arranged and use_perm)

    # ---- the other target-size workloads, same number of steps each (context, not the value) ----
    if context is not None and not args.no_target_shapes and args.workload == DEFAULT and not (args.identity or args.arranged):
        del xs, outs, x0
        torch.cuda.empty_cache()
        shapes = [{"workload": args.workload, "T": T, "d": d, "b": b, "fmt": fmt, "kernel_ms": kern_ms,
                   "algorithmic_bytes": alg_bytes, "achieved_GBs": achieved, "frac": achieved / HBM_PEAK_GBS,
                   "tokens_per_s": T / (kern_ms * 1e-3), "check": check}]
        for name in TARGET_SHAPES:
            if name != args.workload:
                shapes.append(time_target_shape(name, args.steps, args.warmup, args.pool_bytes, args.algo,
                                                not (args.no_check or args.no_cpu_baseline)))
        context["target_shapes"] = shapes

    line = {
        "metric": "fused permute+block-Hadamard+quant tokens/s",
        "value": tokens_per_s,
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": args.workload, "T": T, "d": d, "b": b, "fmt": fmt,
                   "perm": ("greedy-calibrated, blocks arranged for the LDS gather, gather fused" if args.arranged
                            else "greedy-calibrated, gather fused") if use_perm else "identity",
                   "prepared_form": "perq_perm_prepare" if place_t is not None else "none",
                   "algo": args.algo, "buffer_sets": nsets, "input_gen_s": round(gen_s, 1)},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_source,
                     "algorithmic_bytes": alg_bytes, "kernel_ms": kern_ms},
        "cpu_baseline": cpu,
        "calibration": calib,
        "context": context,
        "check": check,
    }
    print(json.dumps(line))
    ok = check is None or check["ok"]
    for sh in (context or {}).get("target_shapes", []):
        ok = ok and (sh.get("check") is None or sh["check"]["ok"])
    return 0 if ok else 1


if __name__ == "__main__":
    sys.exit(main())
