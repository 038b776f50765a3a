#!/usr/bin/env python3
"""Benchmark: spherical-attention forward on one MI355X.

A step is one full forward pass (both N x N contractions, the row-norm
accumulation and the tail) over one batch of synthetic Gaussian Q/K/V already
resident in HBM.  Throughput uses the 4*B*H*N^2*d FLOP convention.  Prints one
JSON line.
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

# dense MFMA peaks of MI355X; the fp8-QK workload runs half its flops at the fp8 rate (5000)
# and half at the bf16 rate (2500): harmonic mean
PEAK_TFLOPS = {"bf16": 2500.0, "f16": 2500.0, "fp8qk_bf16v": 1.0 / (0.5 / 5000.0 + 0.5 / 2500.0), "f32": 157.3}
# HBM bytes per launch from rocprofv3 FETCH_SIZE / WRITE_SIZE, each scaled by the reading of a
# 256 MiB device copy in the same run.  These are stored readings of the profile named beside
# them, not measured by this process (counters need the profiler): `traffic` carries one only for
# the workload and kernel that profile covers, `traffic_source` says where it came from, and
# every other workload reports null.
MEASURED_HBM_BYTES = {
    "C1": (1.28e6, "profiles/fwd_f32_d64_C1.md"),
    "C2": (33.7e6, "profiles/fwd_pipelined_bf16_d64_C2.md"),
    "C3": (268.7e6, "profiles/fwd_pipelined_bf16_d128_C3.md"),
    "C4": (175.8e6, "profiles/fwd_pipelined_bf16_d64_C4.md"),
    "C5": (1020.3e6, "profiles/fwd_pipelined_fp8qk_d128_C5.md"),
}
HBM_PEAK_GBS = 8000.0


def time_launches(fn, steps, warmup):
    """Average and per-launch durations (ms) of `fn`, HIP events on the launch stream."""
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    starts = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
    ends = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
    t0 = time.perf_counter()
    for i in range(steps):
        starts[i].record()
        fn()
        ends[i].record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    per = sorted(s.elapsed_time(e) for s, e in zip(starts, ends))
    return wall_ms / steps, per


def load_mfma_probe():
    """bench_mfma_probe of libbench_mfma_probe.so (built by __graft_entry__.build()): loops of
    matrix instructions only, the benchmark's own measurement aid."""
    import ctypes
    path = os.path.join(ROOT, "libbench_mfma_probe.so")
    if not os.path.exists(path):
        raise ImportError(f"{path} is not built; run `python -c 'import __graft_entry__ as g; g.build()'`")
    fn = ctypes.CDLL(path).bench_mfma_probe
    fn.restype = ctypes.c_int
    fn.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]

    def probe(operands, clocks, form, iters):
        import torch
        rc = fn(operands.data_ptr(), clocks.data_ptr(), int(form), int(iters),
                ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
        if rc != 0:
            raise RuntimeError(f"bench_mfma_probe returned {rc}")
        return 256.0 * 4 * iters * 16 * 32768.0    # flop of the launch
    return probe


LDS_PATTERNS = (
    (0, "ds_read_b128", "linear: 16 bytes per lane in lane order"),
    (1, "ds_read_b128", "piece g of row n16, rows of 64 bytes (the fragment blocks' first layout)"),
    (2, "ds_read_b128", "the same with the pieces of a row permuted (forward K tiles, all-E4M3 tiles)"),
    (3, "ds_read_b128", "two blocks of 16 rows x 32 bytes (backward tiles)"),
    (10, "ds_read_b64_tr_b16", "linear: 8 bytes per lane in lane order (V tiles, backward tiles)"),
    (11, "ds_read_b64_tr_b16", "the transposed operand on rows of 64 bytes (the backward's first layout)"),
    (12, "ds_read_b64_tr_b16", "the same on rows with permuted pieces"),
)


def lds_probe(dev):
    """--lds-probe: launches of the benchmark's LDS probe, one read pattern each (one workgroup of
    four waves, 16 reads in flight per wave): shader clocks per wave instruction here; the LDS
    counters of `rocprofv3 --pmc SQ_LDS_IDX_ACTIVE SQ_LDS_BANK_CONFLICT SQ_INSTS_LDS` attach to the
    same launches and give the LDS cycles and the conflict cycles per instruction."""
    import ctypes
    import torch
    path = os.path.join(ROOT, "libbench_lds_probe.so")
    if not os.path.exists(path):
        raise ImportError(f"{path} is not built; run `python -c 'import __graft_entry__ as g; g.build()'`")
    fn = ctypes.CDLL(path).bench_lds_probe
    fn.restype = ctypes.c_int
    fn.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
    clk = torch.zeros(4, dtype=torch.int64, device=dev)
    iters = 2000

    def run(pattern):
        for _ in range(2):
            rc = fn(clk.data_ptr(), pattern, iters, ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
            if rc != 0:
                raise RuntimeError(f"bench_lds_probe({pattern}) returned {rc}")
        torch.cuda.synchronize()
        return max(clk.cpu().tolist()) / (iters * 16.0 + 8.0)

    out = {"patterns": [{"pattern": p, "instruction": ins, "layout": what, "clocks_per_wave_instruction": run(p)}
                        for p, ins, what in LDS_PATTERNS]}
    # Which lanes the LDS serves in the same pass: lane 1 of a linear pattern reads lane j's
    # address instead of its own.  Served in the same pass the two are one address (a broadcast,
    # no conflict); otherwise lane 1 collides with the lane of its own pass that owns those banks
    # (j = 1, 17, 33, 49, or 1, 33 for the 8-byte read, are lane 1's own banks: no conflict either
    # way).  One launch per j; the clocks barely move (the probe is bound by instruction issue),
    # so this part is for the counters only.
    for base in (100, 200):
        for j in range(64):
            rc = fn(clk.data_ptr(), base + j, 200, ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
            if rc != 0:
                raise RuntimeError(f"bench_lds_probe({base + j}) returned {rc}")
    torch.cuda.synchronize()
    out["dispatch_order"] = ("two launches per pattern above, in that order; then ds_read_b128 with lane 1 on the "
                             "address of lane j = 0..63, then ds_read_b64_tr_b16 likewise, one launch each")
    return out


def measure_mfma_ceiling(args, si, dev):
    """Loops of nothing but matrix instructions on Gaussian operands: TFLOP/s and shader clock
    per instruction form (the fp8 forms only with --fp8-all)."""
    import torch
    g = torch.Generator(device="cpu").manual_seed(7)
    ops16 = torch.randn(32768, generator=g, dtype=torch.float32).to(torch.bfloat16).to(dev)
    ops8 = si.to_e4m3fn(torch.randn(65536, generator=g, dtype=torch.float32)).view(torch.uint8).to(dev)
    clk = torch.zeros(3, dtype=torch.int64, device=dev)
    mfma_probe = load_mfma_probe()
    ceil = {}
    for form, name in ((0, "32x32x16_bf16"), (1, "16x16x32_bf16"), (2, "16x16x128_e4m3"),
                       (3, "16x16x128_e4m3_with_l2_stage_b_mix"), (4, "16x16x128_e4m3_with_softmax_stage_b_mix")):
        iters = 100000
        if form >= 2 and not args.fp8_all:
            continue
        ops = ops8 if form >= 2 else ops16
        for _ in range(2):
            flop = mfma_probe(ops, clk, form, iters)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        flop = mfma_probe(ops, clk, form, iters)
        e1.record()
        torch.cuda.synchronize()
        c = clk.cpu().tolist()
        ceil[name] = {"tflops": flop / (e0.elapsed_time(e1) * 1e-3) / 1e12, "shader_ghz": 0.1 * c[0] / max(c[1], 1)}
    return ceil


def cpu_baseline(w, q, k, v, budget_s=12.0):
    """The fp64 oracle, as it stands, on a bounded sample: whole heads of the workload, one
    after the other, until about `budget_s` seconds of CPU time have been spent."""
    import numpy as np
    import oracle
    import synthetic_inputs as si
    (qb, qk), (kb, kk), (vb, vk) = (si.storage_bits(t) for t in (q, k, v))
    kinds = (qk, kk, vk)
    threads = oracle.num_threads()
    rows = np.arange(w.N, dtype=np.int32)
    heads, elapsed = 0, 0.0
    while heads < w.B * w.H and elapsed < budget_s:
        t0 = time.perf_counter()
        oracle.spherical_attention_rows(qb, kb, vb, heads, rows, kinds)
        elapsed += time.perf_counter() - t0
        heads += 1
    flops = 4.0 * heads * w.N * w.N * w.d
    return {
        "value": flops / elapsed / 1e12, "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
        "sample": f"{heads} of {w.B * w.H} heads of {w.name} (all {w.N} query rows x {w.N} keys each), "
                  f"fp64, {elapsed:.1f} s; the whole workload extrapolates to "
                  f"{elapsed * w.B * w.H / heads:.0f} s",
    }


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="C3", help="C1..C5, or P1 = the paper's own point (fp16, d=128, N=3x13824), "
                         "or a shape of one's own as B,H,N,d[,dtype]; default C3: the configuration the target is quoted on")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-twin", action="store_true")
    ap.add_argument("--no-after-idle", action="store_true", help="skip the second timing taken after 1 s of idle")
    ap.add_argument("--grn", type=int, default=0, metavar="H_KV",
                    help="also time the gene-regulatory-network entry point on the same shape with "
                         "H_KV shared K/V heads and Poisson(1.5) multiplicities")
    ap.add_argument("--splitkv", type=int, default=0, metavar="HEADS",
                    help="also time the split-key forward against the unsplit call on the first HEADS "
                         "heads of batch 0 of the workload (few heads leave CUs idle; the split fills them)")
    ap.add_argument("--no-mfma-ceiling", action="store_true",
                    help="skip the loops of nothing but bf16 matrix instructions on Gaussian operands (the "
                         "rate the matrix pipes sustain at the power limit, reported next to the kernel's)")
    ap.add_argument("--fp8-all", action="store_true",
                    help="also time the all-E4M3 forward (sphattn_fp8_fwd: V and the scores in E4M3, too) on "
                         "the workload's shape")
    ap.add_argument("--bwd", action="store_true", help="also time the backward pass (sphattn_bwd) on the workload")
    ap.add_argument("--lds-probe", action="store_true",
                    help="run only the LDS read-pattern probe (libbench_lds_probe.so) and print its table as JSON")
    ap.add_argument("--cross-launches", nargs=5, type=int, metavar=("B", "H", "NQ", "NK", "D"),
                    help="run only four untimed bf16 launches of sphattn_cross_fwd on this shape and exit: the "
                         "dispatches that an HBM byte counter (rocprofv3 --pmc FETCH_SIZE) is read on when "
                         "the query and key counts have to differ")
    ap.add_argument("--copy-reference", action="store_true",
                    help="also run a plain 256 MiB device copy (untimed), as the known-size "
                         "reference that HBM byte counters are scaled by when profiling")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path "
              "(heads and query tiles shard with no communication); run with --gpus 1",
              file=sys.stderr)
        return 2

    import torch
    import paper_2505_09326_amd as pkg
    import synthetic_inputs as si

    if args.lds_probe:
        print(json.dumps(lds_probe(torch.device("cuda:0"))))
        return 0

    pkg.load_library()                       # fail loudly if the HIP library is not built
    if args.cross_launches:
        B, H, Nq, Nk, d = args.cross_launches
        dev = torch.device("cuda:0")
        g = torch.Generator(device="cpu").manual_seed(3)
        qd = (torch.randn(B, H, Nq, d, generator=g) / 8).to(torch.bfloat16).to(dev)
        kd, vd = ((torch.randn(B, H, Nk, d, generator=g) / 8).to(torch.bfloat16).to(dev) for _ in range(2))
        out = torch.empty_like(qd)
        for _ in range(4):
            pkg.sphattn_cross_fwd(qd, kd, vd, None, O=out, dtype="bf16")
        torch.cuda.synchronize()
        print(json.dumps({"cross_launches": 4, "shape": [B, H, Nq, Nk, d],
                          "min_read_bytes": 2 * B * H * d * (Nq + 2 * Nk)}))
        return 0
    w, (q, k, v) = si.make_workload(args.workload)
    dev = torch.device("cuda:0")
    qd, kd, vd = q.to(dev), k.to(dev), v.to(dev)
    out_dt = {"f32": torch.float32, "f16": torch.float16}.get(w.dtype, torch.bfloat16)
    out = torch.empty(qd.shape, dtype=out_dt, device=dev)
    torch.cuda.synchronize()

    def step():
        pkg.sphattn_fwd(qd, kd, vd, out, dtype=w.dtype)

    # What the matrix pipes sustain on Gaussian operands, matrix instructions only.  It runs
    # BEFORE the timed steps on purpose: after any idle period the part's power management goes
    # through a transient of about 30 launches (boost, overshoot down to -25 %, recovery), and a
    # short timed region right after start-up would sit in the middle of it.  With ~0.2 s of matrix
    # work in front, the warm-up and timed steps measure the settled state; `after_idle` below is
    # the same measurement taken from idle, for comparison.
    # (One call first, so that loading the library's code object and raising the kernel's LDS
    # limit, which take milliseconds of idle GPU, do not fall between the probe and the steps.)
    step()
    torch.cuda.synchronize()
    ceil = None
    if not args.no_mfma_ceiling:
        try:
            ceil = measure_mfma_ceiling(args, si, dev)
        except ImportError as e:               # the probe is a measurement aid: the benchmark runs without it
            print(f"bench.py: {e}; continuing without the matrix-only ceiling", file=sys.stderr)

    ms_wall, per = time_launches(step, args.steps, args.warmup)
    ms_kernel = sum(per) / len(per)
    tflops = w.flops / (ms_wall * 1e-3) / 1e12
    kern_tflops = w.flops / (ms_kernel * 1e-3) / 1e12
    peak = PEAK_TFLOPS[w.dtype]

    elt_qk = {"f32": 4, "bf16": 2, "f16": 2, "fp8qk_bf16v": 1}[w.dtype]
    elt_vo = 4 if w.dtype == "f32" else 2
    n_el = w.B * w.H * w.N * w.d
    algo_bytes = n_el * (2 * elt_qk + 2 * elt_vo)

    result = {
        "metric": "spherical-attention fwd TFLOP/s (4*B*H*N^2*d)",
        "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_wall, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": {"bf16": "bf16", "f16": "f16", "f32": "f32", "fp8qk_bf16v": "fp8"}[w.dtype], "data": "synthetic",
        "config": {"workload": w.describe(), "B": w.B, "H": w.H, "N": w.N, "d": w.d,
                   "flop_per_step": w.flops, "min_hbm_bytes_per_step": algo_bytes},
        "roofline": {"bound": "mfma", "achieved": kern_tflops, "peak": peak, "unit": "TFLOP/s",
                     "frac": kern_tflops / peak,
                     "traffic": MEASURED_HBM_BYTES[w.name][0] if w.name in MEASURED_HBM_BYTES else None,
                     "traffic_source": (f"stored reading of {MEASURED_HBM_BYTES[w.name][1]} (rocprofv3 FETCH_SIZE + WRITE_SIZE, "
                                        "scaled by a 256 MiB copy), not measured by this run"
                                        if w.name in MEASURED_HBM_BYTES else None),
                     "kernel_ms_avg": ms_kernel, "kernel_ms_median": per[len(per) // 2],
                     "kernel_ms_min": per[0]},
    }

    # the same K steps after W warm-up steps, taken from idle (1 s of sleep): what a short timed
    # region sees when nothing ran before it
    if w.flops >= 1e11 and not args.no_after_idle:
        torch.cuda.synchronize()
        time.sleep(1.0)
        _, per_idle = time_launches(step, args.steps, args.warmup)
        result["roofline"]["timing_state"] = ("settled: the matrix-only probe ran first" if ceil is not None
                                              else "whatever preceded the warm-up steps")
        result["roofline"]["after_idle"] = {
            "kernel_ms_avg": sum(per_idle) / len(per_idle), "frac": w.flops / (sum(per_idle) / len(per_idle) * 1e-3) / 1e12 / peak,
            "note": "same steps and warm-up after 1 s of idle: inside the power-management transient"}

    # short problems are bound by launch latency and occupancy, not by the matrix pipes: also
    # state what the launch achieves against the HBM roofline (algorithmic bytes / time)
    if w.flops < 1e11:
        # launch latency apart: 1000 launches back to back, one pair of events around them
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(1000):
            step()
        e1.record()
        torch.cuda.synchronize()
        result["roofline"]["back_to_back_ms_avg_1000"] = e0.elapsed_time(e1) / 1000.0
    result["roofline"]["hbm_gbs_algorithmic"] = algo_bytes / (ms_kernel * 1e-3) / 1e9
    result["roofline"]["hbm_peak_gbs"] = HBM_PEAK_GBS
    # the paper's own figures, another machine: context only, never the baseline
    result["paper_context"] = {
        "hardware": "1x NVIDIA A100 SXM4 80GB, FP16, d=128, N multiple of 13824",
        "tflops": 200.0, "fraction_of_fp16_tensor_peak": 0.64,
        "vs_unfused_pytorch": 3.6, "vs_flashattention2": "within 5% at N=41.5K",
    }

    if not args.no_twin and w.dtype == "bf16":
        def twin():
            pkg.sphattn_softmax_fwd(qd, kd, vd, out, dtype=w.dtype)
        _, per_t = time_launches(twin, max(30, args.steps // 2), max(10, args.warmup // 2))
        ms_t = sum(per_t) / len(per_t)
        result["softmax_twin"] = {"kernel_ms_avg": ms_t, "tflops": w.flops / (ms_t * 1e-3) / 1e12,
                                  "spherical_speedup": ms_t / ms_kernel,
                                  "form": "32x32x16 MFMA kernel of its own (the faster SoftMax form at d = 128)", "shares_the_spherical_kernels_data_path": False,
                                  "note": "own data path (register-staged, padded LDS rows): the ratio mixes that "
                                          "difference into the exponential's cost; softmax_twin_same_instructions is like for like"}

        def twin16():
            pkg.sphattn_normalized_fwd(qd, kd, vd, out, dtype=w.dtype, normalizer="softmax")
        _, per_t = time_launches(twin16, max(30, args.steps // 2), max(10, args.warmup // 2))
        ms_t = sum(per_t) / len(per_t)
        result["softmax_twin_same_instructions"] = {
            "kernel_ms_avg": ms_t, "tflops": w.flops / (ms_t * 1e-3) / 1e12, "spherical_speedup": ms_t / ms_kernel,
            "form": "16x16x32 MFMA, the spherical kernel with exp/max/rescale in stage B",
            "shares_the_spherical_kernels_data_path": True}

    if not args.no_twin and w.dtype == "fp8qk_bf16v":
        def twin8():
            pkg.sphattn_normalized_fwd(qd, kd, vd, out, dtype=w.dtype, normalizer="softmax")
        _, per_t = time_launches(twin8, max(30, args.steps // 2), max(10, args.warmup // 2))
        ms_t = sum(per_t) / len(per_t)
        result["softmax_twin_same_instructions"] = {
            "kernel_ms_avg": ms_t, "tflops": w.flops / (ms_t * 1e-3) / 1e12, "spherical_speedup": ms_t / ms_kernel,
            "form": "the spherical kernel (fp8 16x16x128 scores, bf16 16x16x32 output) with exp/max/rescale in stage B",
            "shares_the_spherical_kernels_data_path": True}

    if args.grn:
        g = torch.Generator(device="cpu").manual_seed(w.seed + 1000)
        mult = torch.poisson(torch.full((w.B, w.N), 1.5), generator=g).to(torch.float32).to(dev)
        kg, vg = kd[:, :args.grn].contiguous(), vd[:, :args.grn].contiguous()

        def grn():
            pkg.sphattn_grn_fwd(qd, kg, vg, mult, out, dtype=w.dtype)
        _, per_g = time_launches(grn, max(30, args.steps // 2), max(10, args.warmup // 2))
        ms_g = sum(per_g) / len(per_g)
        result["grn_variant"] = {"H_kv": args.grn, "multiplicities": "Poisson(1.5)", "kernel_ms_avg": ms_g,
                                 "tflops": w.flops / (ms_g * 1e-3) / 1e12}

    if args.splitkv:
        hs = min(args.splitkv, w.H)
        qs, ks, vs = (t[:1, :hs].contiguous() for t in (qd, kd, vd))
        outs = torch.empty_like(vs)
        n_splits = pkg.sphattn_splitkv_heuristic(1, hs, w.N, w.d, w.dtype)
        ws = torch.empty(pkg.sphattn_splitkv_workspace_bytes(1, hs, w.N, w.d, n_splits), dtype=torch.uint8, device=dev)
        _, per_u = time_launches(lambda: pkg.sphattn_fwd(qs, ks, vs, outs, dtype=w.dtype),
                                 max(30, args.steps // 2), max(10, args.warmup // 2))
        _, per_s = time_launches(lambda: pkg.sphattn_splitkv_fwd(qs, ks, vs, ws, O=outs, n_splits=n_splits, dtype=w.dtype),
                                 max(30, args.steps // 2), max(10, args.warmup // 2))
        ms_u, ms_s = sum(per_u) / len(per_u), sum(per_s) / len(per_s)
        fl = 4.0 * hs * w.N * w.N * w.d
        result["splitkv_variant"] = {
            "shape": f"B=1 H={hs} N={w.N} d={w.d} {w.dtype}", "n_splits": n_splits,
            "workspace_bytes": ws.numel(), "unsplit_ms_avg": ms_u, "split_ms_avg": ms_s,
            "unsplit_tflops": fl / (ms_u * 1e-3) / 1e12, "split_tflops": fl / (ms_s * 1e-3) / 1e12,
            "split_speedup": ms_u / ms_s,
        }

    if ceil is not None:
        result["mfma_only_ceiling_gaussian_operands"] = ceil
        result["roofline"]["frac_of_mfma_only_ceiling"] = kern_tflops / ceil["16x16x32_bf16"]["tflops"]

    if args.fp8_all:
        q8, k8, v8 = (si.to_e4m3fn(t.to(torch.float32)).to(dev) if t.dtype != torch.float8_e4m3fn else t.to(dev)
                      for t in (q, k, v))
        ws8 = torch.empty(pkg.sphattn_fp8_workspace_bytes(w.B, w.H, w.N, w.d), dtype=torch.uint8, device=dev)
        out8 = torch.empty((w.B, w.H, w.N, w.d), dtype=torch.bfloat16, device=dev)
        _, per_8 = time_launches(lambda: pkg.sphattn_fp8_fwd(q8, k8, v8, ws8, O=out8),
                                 max(30, args.steps // 2), max(10, args.warmup // 2))
        ms_8 = sum(per_8) / len(per_8)
        tf8 = w.flops / (ms_8 * 1e-3) / 1e12
        result["fp8_all_variant"] = {
            "storage": "Q, K, V E4M3; scores rounded to E4M3; O bf16", "launches": 3,
            "ms_avg": ms_8, "tflops": tf8, "frac_of_fp8_mfma_peak": tf8 / 5000.0,
            "workspace_bytes": ws8.numel(), "speedup_over_headline_kernel": ms_kernel / ms_8,
        }
        if not args.no_twin:
            # the SoftMax twin needs inputs of moderate size (its shift is a bound, not the running
            # maximum): N(0, 0.5) cast to E4M3, for both kernels of this comparison
            qm, km_, vm = (t.to(torch.float8_e4m3fn).to(dev) for t in si.gaussian_qkv(w.B, w.H, w.N, w.d, w.seed + 3000, 0.5))
            _, per_a = time_launches(lambda: pkg.sphattn_fp8_fwd(qm, km_, vm, ws8, O=out8),
                                     max(30, args.steps // 2), max(10, args.warmup // 2))
            _, per_b = time_launches(lambda: pkg.sphattn_fp8_softmax_fwd(qm, km_, vm, ws8, O=out8),
                                     max(30, args.steps // 2), max(10, args.warmup // 2))
            ms_a, ms_b = sum(per_a) / len(per_a), sum(per_b) / len(per_b)
            result["fp8_all_variant"]["softmax_twin"] = {
                "inputs": "N(0, 0.5) cast to E4M3", "spherical_ms_avg": ms_a, "softmax_ms_avg": ms_b,
                "spherical_speedup": ms_b / ms_a,
                "form": "same kernel; shift by the Cauchy-Schwarz bound instead of a running maximum, no rescaling",
            }
        if ceil is not None:
            result["fp8_all_variant"]["frac_of_mfma_only_ceiling"] = tf8 / ceil["16x16x128_e4m3"]["tflops"]
            # what the exponential costs at the fp8 matrix rate (paper, Section 1): the same loop
            # of matrix instructions with an L2 kernel's, or a SoftMax kernel's, other per-score
            # instructions pinned behind each of them
            result["fp8_all_variant"]["l2_over_softmax_instruction_mix"] = (
                ceil["16x16x128_e4m3_with_l2_stage_b_mix"]["tflops"]
                / ceil["16x16x128_e4m3_with_softmax_stage_b_mix"]["tflops"])

    if args.bwd:
        if w.dtype not in ("bf16", "f16"):
            print("--bwd needs a 16-bit workload", file=sys.stderr)
            return 2
        g = torch.Generator(device="cpu").manual_seed(w.seed + 2000)
        dO = torch.randn(q.shape, generator=g, dtype=torch.float32).to(q.dtype).to(dev)
        Zf = torch.empty(qd.shape[:3], dtype=torch.float32, device=dev)
        pkg.sphattn_fwd_z(qd, kd, vd, out, Zf, dtype=w.dtype)
        dQ, dK, dV = (torch.empty_like(qd) for _ in range(3))
        delta = torch.empty((2, *Zf.shape), dtype=torch.float32, device=dev)
        _, per_b = time_launches(lambda: pkg.sphattn_bwd(qd, kd, vd, out, dO, Zf, dQ, dK, dV, delta, dtype=w.dtype),
                                 max(30, args.steps // 2), max(10, args.warmup // 2))
        ms_b = sum(per_b) / len(per_b)
        result["backward"] = {
            "ms_avg": ms_b, "kernels": 2,
            "tflops_10N2d": 2.5 * w.flops / (ms_b * 1e-3) / 1e12,       # five N x N x d contractions
            "tflops_executed_14N2d": 3.5 * w.flops / (ms_b * 1e-3) / 1e12,   # scores recomputed in both kernels
            "vs_forward": ms_b / ms_kernel,
        }
        if args.grn:
            # the same with gene multiplicities and args.grn shared K/V heads (sphattn_grn_bwd);
            # O and z of that forward come from sphattn_cross_fwd
            gm = torch.Generator(device="cpu").manual_seed(w.seed + 1000)
            mult = torch.poisson(torch.full((w.B, w.N), 1.5), generator=gm).to(torch.float32).to(dev)
            kg, vg = kd[:, :args.grn].contiguous(), vd[:, :args.grn].contiguous()
            pkg.sphattn_cross_fwd(qd, kg, vg, mult, O=out, Z=Zf, dtype=w.dtype)
            dKg, dVg = torch.empty_like(kg), torch.empty_like(vg)
            _, per_g = time_launches(lambda: pkg.sphattn_grn_bwd(qd, kg, vg, mult, out, dO, Zf, dQ, dKg, dVg, delta, dtype=w.dtype),
                                     max(30, args.steps // 2), max(10, args.warmup // 2))
            ms_gb = sum(per_g) / len(per_g)
            result["backward"]["grn_variant"] = {"H_kv": args.grn, "multiplicities": "Poisson(1.5)", "ms_avg": ms_gb,
                                                 "vs_plain_backward": ms_gb / ms_b}

    if args.copy_reference:
        src = torch.zeros(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w, q, k, v)

    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
