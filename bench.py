#!/usr/bin/env python3
"""Benchmark of the MoDA attention forward pass (libmoda) on one MI355X.

A "step" is one call of moda_attn_fwd (the whole fused hot path: sequence tiles,
depth slots, normalise, store) on one batch of synthetic inputs already resident
in HBM.  The default workload is the long-context configuration the headline
metric is quoted on: B=1, H=16, d=128, T=65536, depth_count=15, bf16, causal.
The same shape is also timed with depth_count=0 (the build's own causal
flash-attention kernel) to form the efficiency ratio t(depth 0) / t(depth 15),
the way the paper forms its 97.3 % figure (Table 2, row 5).

Prints ONE JSON line.  FLOP convention: 4*d per visible (query, key) pair,
i.e. 4*d*B*H*(T(T+1)/2 + T*L) for a causal call.
"""
import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

WORKLOADS = {
    # name: (B, Hq, Hk, T, d, depth_count, dtype)
    "long_context_64k": (1, 16, 16, 65536, 128, 15, "bf16"),   # BASELINE configs[2] (the metric's workload)
    "layer_1p5b_4k": (8, 16, 16, 4096, 128, 15, "bf16"),       # BASELINE configs[1]
    "tiny_fp32": (1, 2, 2, 256, 64, 4, "f32"),                 # BASELINE configs[0]
    "bwd_layer_1p5b_4k": (8, 16, 16, 4096, 128, 15, "bf16"),   # BASELINE configs[4] (backward)
    "copy_calibration": None,  # plain device copy of known size, for scaling the HBM byte counters
    "mfma_calibration": None,  # what the matrix pipe alone sustains (zero and N(0,1) bf16 operands)
    "sweep": None,             # BASELINE configs[3]: B=4 H=16 d=128, T x depth_count grid
    "paper_table2": None,      # the paper's Table 2 shapes (d=64, grouped queries, 64..256 slots), fwd+bwd
    "decode": None,            # one new token per sequence against a 64K sequence cache
    "append": None,            # the depth stream's write step (a strided copy)
}
PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}  # MI355X dense MFMA bf16 / fp32 vector


def fwd_flops(B, H, T, d, L, causal=True):
    pairs = T * (T + 1) // 2 if causal else T * T
    return 4.0 * d * B * H * (pairs + T * L)


def bwd_flops(B, H, T, d, L, causal=True):
    """10*d per visible pair: five d-length contractions (S, dP, dV, dQ, dK)."""
    pairs = T * (T + 1) // 2 if causal else T * T
    return 10.0 * d * B * H * (pairs + T * L)


def bwd_workspace_bytes(B, Hq, Hk, T, d, L):
    from paper_2603_15619_amd import MODAShape, moda_attn_bwd_workspace_bytes

    return max(16, moda_attn_bwd_workspace_bytes(MODAShape(B, Hq, Hk, T, d, L, L, 1, 0.0, 1)))


def measured_traffic(workload, kernel):
    """HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (see
    profiles/), or None if this workload has not been measured."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    try:
        table = json.load(open(path))
    except (OSError, ValueError):
        return None
    entry = table.get("%s/%s" % (workload, kernel))
    return None if entry is None else entry["hbm_bytes"]


def run_copy_calibration(args):
    n = 1 << 30  # 4 GiB of fp32 in, 4 GiB out
    a = torch.ones(n, dtype=torch.float32, device="cuda")
    b = torch.empty_like(a)
    ms, _, _ = time_calls(lambda: b.copy_(a), args.steps, args.warmup)
    print(json.dumps({"metric": "plain device copy", "bytes_read": 4 * n, "bytes_written": 4 * n,
                      "ms_per_step": round(ms, 4), "value": round(8 * n / ms / 1e6, 1), "unit": "GB/s",
                      "steps": args.steps, "warmup": args.warmup}))


def mfma_calibration(reps=6, target_ms=40.0):
    """TFLOP/s that a loop of nothing but v_mfma_f32_32x32x16_bf16 sustains on this chip (the
    library's calibration kernel: 8 waves per workgroup, 4 workgroups per compute unit's worth of
    grid), on all-zero operands and on N(0,1) operands.  Each figure is the mean of the last
    `reps - 2` of `reps` launches of about `target_ms` each (the clock settles during the first)."""
    from paper_2603_15619_amd import lib, moda_calibrate_mfma

    n = int(lib().moda_calibrate_mfma_operand_bytes()) // 2
    wgs = 256 * 4
    sink = torch.empty(int(lib().moda_calibrate_mfma_sink_bytes(wgs)) // 4, dtype=torch.float32, device="cuda")
    gen = torch.Generator(device="cuda")
    gen.manual_seed(77)
    out = {}
    for name, ops in (("zeros", torch.zeros(n, dtype=torch.bfloat16, device="cuda")),
                      ("normal", torch.randn(n, generator=gen, device="cuda").to(torch.bfloat16))):
        iters = 20000
        for _ in range(2):  # size the launch: about target_ms at the rate just seen
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            fl = moda_calibrate_mfma(ops, wgs, iters, sink)
            b.record()
            torch.cuda.synchronize()
            iters = max(1000, int(iters * target_ms / max(a.elapsed_time(b), 1e-3)))
        rates = []
        for _ in range(reps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            fl = moda_calibrate_mfma(ops, wgs, iters, sink)
            b.record()
            torch.cuda.synchronize()
            rates.append(fl / (a.elapsed_time(b) * 1e-3) / 1e12)
        out[name] = round(float(np.mean(rates[2:])), 1)
        out[name + "_launch_ms"] = round(fl / (out[name] * 1e12) * 1e3, 2)
    return out


def run_mfma_calibration(args):
    cal = mfma_calibration(reps=max(4, args.steps))
    print(json.dumps({"metric": "bf16 MFMA-only loop (moda_calibrate_mfma_kernel), TFLOP/s", "unit": "TFLOP/s",
                      "published_peak": PEAK_TFLOPS["bf16"], "operands_zero": cal["zeros"],
                      "operands_normal": cal["normal"], "launch_ms": [cal["zeros_launch_ms"], cal["normal_launch_ms"]],
                      "steps": args.steps}))


def run_sweep(args):
    """BASELINE configs[3]: TFLOP/s and depth-segment GB/s per (T, depth_count) point."""
    from paper_2603_15619_amd import moda_attn_fwd, synth

    B, H, d = 4, 16, 128
    points = []
    for T in (1024, 4096, 16384):
        inp = synth.make_inputs(B, H, H, T, d, 31, dtype="bf16", seed=3, device="cuda")
        O = torch.empty_like(inp["Q"])
        LSE = torch.empty((B, H, T), dtype=torch.float32, device="cuda")
        t0 = None
        for L in (0, 1, 7, 15, 31):
            kd = None if L == 0 else inp["Kdepth"][:, :, :, :L].contiguous()
            vd = None if L == 0 else inp["Vdepth"][:, :, :, :L].contiguous()
            fn = lambda: moda_attn_fwd(inp["Q"], inp["Kseq"], inp["Vseq"], kd, vd, depth_count=L, out=O, lse=LSE)
            ms, _, _ = time_calls(fn, args.steps, args.warmup)
            if L == 0:
                t0 = ms
            depth_bytes = 2.0 * B * H * T * L * d * 2
            alg_bytes = 2.0 * (4 * B * H * T * d) + depth_bytes + 4.0 * B * H * T
            floor_ms = max(fwd_flops(B, H, T, d, L) / (PEAK_TFLOPS["bf16"] * 1e12), alg_bytes / 8.0e12) * 1e3
            points.append({"T": T, "depth_count": L, "ms": round(ms, 4),
                           "tflops": round(fwd_flops(B, H, T, d, L) / (ms * 1e-3) / 1e12, 1),
                           "ratio_to_depth0": round(t0 / ms, 4),
                           "extra_ms": round(ms - t0, 4),
                           "depth_gbps_over_call": round(depth_bytes / (ms * 1e-3) / 1e9, 1),
                           "hbm_frac_over_call": round(alg_bytes / (ms * 1e-3) / 8.0e12, 4),
                           "roof_ms": round(floor_ms, 4), "frac_of_roof": round(floor_ms / ms, 4)})
    print(json.dumps({"metric": "MoDA attn fwd sweep (B=4 H=16 d=128 bf16 causal)", "steps": args.steps,
                      "warmup": args.warmup, "points": points}))


# Table 2 of the paper: (row, T, G, Hq, Hk, L, its FlashAttention-2 ms, its MoDA ms) -- forward and
# backward together, one A100, bf16, B=1, d=64; quoted as context (other hardware, Triton kernels).
PAPER_TABLE2 = [
    (1, 4096, 8, 64, 8, 64, 7.970, 10.750), (2, 8192, 8, 64, 8, 64, 28.700, 35.427),
    (3, 16384, 8, 64, 8, 64, 116.700, 127.661), (4, 32768, 8, 64, 8, 64, 459.854, 480.914),
    (5, 65536, 8, 64, 8, 64, 1831.668, 1883.026), (6, 16384, 2, 16, 8, 64, 28.982, 39.741),
    (7, 16384, 4, 32, 8, 64, 58.071, 68.939), (9, 16384, 16, 128, 8, 64, 233.700, 244.900),
    (10, 16384, 32, 256, 8, 64, 467.107, 480.767), (12, 16384, 8, 64, 8, 128, 116.700, 138.224),
    (13, 16384, 8, 64, 8, 256, 116.700, 167.958),
]


def run_paper_table2(args):
    """Forward + backward time at the paper's Table 2 shapes (rows 8 and 11 repeat row 3), with and
    without the depth slots, and the paper's "extra time" figure (MoDA - FA) / MoDA formed the same
    way."""
    from paper_2603_15619_amd import moda_attn_bwd, moda_attn_fwd, synth

    rows = []
    for (no, T, G, Hq, Hk, L, p_fa, p_moda) in PAPER_TABLE2:
        if args.rows and no not in args.rows:
            continue
        inp = synth.make_inputs(1, Hq, Hk, T, 64, L, dtype="bf16", seed=5, device="cuda", with_dO=True)
        O = torch.empty_like(inp["Q"])
        LSE = torch.empty((1, Hq, T), dtype=torch.float32, device="cuda")
        ws = torch.empty(bwd_workspace_bytes(1, Hq, Hk, T, 64, L), dtype=torch.uint8, device="cuda")
        with_bwd = G <= 64
        out = {"row": no, "T": T, "G": G, "Hq": Hq, "Hk": Hk, "depth_count": L, "backward_included": with_bwd,
               "paper_a100_ms": {"fa2": p_fa, "moda": p_moda, "extra_pct": round(100 * (p_moda - p_fa) / p_moda, 2)}}
        for name, kd, vd, dc in (("fa", None, None, 0), ("moda", inp["Kdepth"], inp["Vdepth"], L)):
            def step():
                moda_attn_fwd(inp["Q"], inp["Kseq"], inp["Vseq"], kd, vd, depth_count=dc, out=O, lse=LSE)
                if with_bwd:
                    moda_attn_bwd(inp["Q"], inp["Kseq"], inp["Vseq"], kd, vd, O, LSE, inp["dO"], depth_count=dc,
                                  workspace=ws)
            steps = max(2, min(args.steps, int(2e4 / T) + 2))
            ms, _, _ = time_calls(step, steps, 1)
            out[name + "_ms"] = round(ms, 3)
        out["extra_pct"] = round(100 * (out["moda_ms"] - out["fa_ms"]) / out["moda_ms"], 2)
        out["fa_over_moda"] = round(out["fa_ms"] / out["moda_ms"], 4)
        flops = (fwd_flops(1, Hq, T, 64, L) + (bwd_flops(1, Hq, T, 64, L) if with_bwd else 0.0))
        out["moda_tflops"] = round(flops / (out["moda_ms"] * 1e-3) / 1e12, 1)
        rows.append(out)
        del inp, O, LSE, ws
        torch.cuda.empty_cache()
    print(json.dumps({"metric": "MoDA vs own causal FA at the paper's Table 2 shapes (B=1 d=64 bf16, fwd+bwd)",
                      "steps": args.steps, "rows": rows}))


def run_decode(args):
    """Decoding step (one new token per sequence): bound by reading the sequence K/V cache once."""
    from paper_2603_15619_amd import moda_attn_decode, synth

    points = []
    for (B, Hq, Hk, T, d, L) in ((8, 16, 16, 65536, 128, 15), (32, 16, 16, 4096, 128, 15), (8, 64, 8, 65536, 64, 64)):
        inp = synth.make_inputs(B, Hq, Hk, T, d, 0, dtype="bf16", seed=6, device="cuda")
        one = synth.make_inputs(B, Hq, Hk, 1, d, L, dtype="bf16", seed=7, device="cuda")
        Q = one["Q"][:, :, 0].contiguous()
        Kd, Vd = one["Kdepth"][:, :, 0].contiguous(), one["Vdepth"][:, :, 0].contiguous()
        O = torch.empty_like(Q)
        LSE = torch.empty((B, Hq), dtype=torch.float32, device="cuda")
        ws = torch.empty(64 << 20, dtype=torch.uint8, device="cuda")
        fn = lambda: moda_attn_decode(Q, inp["Kseq"], inp["Vseq"], Kd, Vd, out=O, lse=LSE, workspace=ws)
        ms, ms_k, _ = time_calls(fn, args.steps, args.warmup)
        cache_bytes = 2.0 * B * Hk * T * d * 2
        points.append({"B": B, "Hq": Hq, "Hk": Hk, "T": T, "d": d, "depth_count": L, "ms": round(ms, 4),
                       "cache_GB": round(cache_bytes / 1e9, 3),
                       "hbm_gbps": round(cache_bytes / (ms_k * 1e-3) / 1e9, 1),
                       "frac_of_8TBps": round(cache_bytes / (ms_k * 1e-3) / 1e9 / 8000.0, 4),
                       "tokens_per_s": round(B / (ms * 1e-3), 1)})
        del inp
        torch.cuda.empty_cache()
    print(json.dumps({"metric": "MoDA attn decoding step (2 kernels per call), bf16", "steps": args.steps,
                      "warmup": args.warmup, "points": points}))


def run_append(args):
    """Write step: a layer's K/V [B,Hk,T,d] into one slot of the cache; every byte read once, written once."""
    from paper_2603_15619_amd import moda_depth_append, synth

    points = []
    for (B, Hk, T, d, La) in ((8, 16, 4096, 128, 16), (1, 16, 65536, 128, 16), (1, 8, 65536, 64, 64)):
        inp = synth.make_inputs(B, Hk, Hk, T, d, 0, dtype="bf16", seed=8, device="cuda")
        Kd = torch.zeros((B, Hk, T, La, d), dtype=torch.bfloat16, device="cuda")
        Vd = torch.zeros_like(Kd)
        fn = lambda: moda_depth_append(inp["Kseq"], inp["Vseq"], Kd, Vd, La // 2)
        ms, ms_k, _ = time_calls(fn, args.steps, args.warmup)
        moved = 2 * 2.0 * B * Hk * T * d * 2  # K and V, read + written
        points.append({"B": B, "Hk": Hk, "T": T, "d": d, "depth_alloc": La, "ms": round(ms, 4),
                       "hbm_gbps": round(moved / (ms_k * 1e-3) / 1e9, 1),
                       "frac_of_8TBps": round(moved / (ms_k * 1e-3) / 1e9 / 8000.0, 4)})
        del inp, Kd, Vd
        torch.cuda.empty_cache()
    print(json.dumps({"metric": "MoDA depth-stream write step (moda_depth_append), bf16", "steps": args.steps,
                      "warmup": args.warmup, "points": points}))


def run_backward(args, B, Hq, Hk, T, d, L, dtype):
    from paper_2603_15619_amd import moda_attn_bwd, moda_attn_fwd, synth

    inp = synth.make_inputs(B, Hq, Hk, T, d, L, dtype=dtype, seed=4, device="cuda", with_dO=True)
    O, LSE = moda_attn_fwd(inp["Q"], inp["Kseq"], inp["Vseq"], inp["Kdepth"], inp["Vdepth"], depth_count=L)
    ws = torch.empty(bwd_workspace_bytes(B, Hq, Hk, T, d, L), dtype=torch.uint8, device="cuda")

    def run():
        moda_attn_bwd(inp["Q"], inp["Kseq"], inp["Vseq"], inp["Kdepth"], inp["Vdepth"], O, LSE, inp["dO"],
                      depth_count=L, workspace=ws)

    ms_step, ms_kernel, ms_min = time_calls(run, args.steps, args.warmup)
    flops = bwd_flops(B, Hq, T, d, L)
    esz = 2
    # reads Q, K, V, O, dO, depth K/V; writes dQ, dK, dV, depth grads
    alg_bytes = esz * B * T * d * (Hq * 3 + Hk * 2 + Hq + 2 * Hk) + 4.0 * esz * B * Hk * T * L * d
    print(json.dumps({
        "metric": "MoDA attn bwd TFLOP/s, 1 GPU", "value": round(flops / (ms_step * 1e-3) / 1e12, 2),
        "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": dtype, "data": "synthetic",
        "config": {"workload": "%s: B=%d H=%d T=%d d=%d depth_count=%d causal bwd (3 kernels per call)" %
                               (args.workload, B, Hq, T, d, L)},
        "roofline": {"bound": "hbm", "achieved": round(alg_bytes / (ms_kernel * 1e-3) / 1e9, 1), "peak": 8000.0,
                     "unit": "GB/s", "frac": round(alg_bytes / (ms_kernel * 1e-3) / 1e9 / 8000.0, 4),
                     "traffic": measured_traffic(args.workload, "bwd"),
                     "traffic_source": "stored: profiles/traffic.json (rocprofv3 --pmc runs), not measured by this run",
                     "call_ms_mean": round(ms_kernel, 4),
                     "bytes_per_call": alg_bytes, "flops_per_call": flops}}))


def time_calls(fn, steps, warmup):
    """Wall time of `steps` back-to-back calls (sync on both sides) and the mean
    per-launch duration from HIP events recorded on the launching stream."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
           for _ in range(steps)]
    t0 = time.perf_counter()
    for a, b in evs:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    per = [a.elapsed_time(b) for a, b in evs]
    return wall_ms / steps, float(np.mean(per)), float(np.min(per))


def cpu_baseline(inp, T, d, L, H, target_rows):
    """Time the fp64 oracle, as it stands, on a sample of query rows of this workload."""
    from oracle import moda_ref as R
    from paper_2603_15619_amd import synth

    rng = np.random.default_rng(1234)
    rows = np.sort(rng.choice(T, size=min(target_rows, T), replace=False)).astype(np.int32)
    ridx = torch.from_numpy(rows.astype(np.int64)).to(inp["Q"].device)
    pick = lambda t: None if t is None else synth.to_f64(t.index_select(2, ridx))
    args = (pick(inp["Q"]), synth.to_f64(inp["Kseq"]), synth.to_f64(inp["Vseq"]),
            pick(inp["Kdepth"]), pick(inp["Vdepth"]))
    R.lib()
    t0 = time.perf_counter()
    R.fwd_rows(*args, rows, depth_count=L)
    dt = time.perf_counter() - t0
    B = inp["Q"].shape[0]
    flops = 4.0 * d * B * H * float(np.sum(rows.astype(np.float64) + 1 + L))
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": R.num_threads(),
            "kind": "oracle", "seconds": round(dt, 2),
            "sample": "%d random query rows (seed 1234) x all %d (b,h) of the same workload, "
                      "full causal key range per row, fp64" % (len(rows), B * H)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="long_context_64k", choices=sorted(WORKLOADS))
    ap.add_argument("--depth-count", type=int, default=None, help="override the workload's depth_count")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-fa", action="store_true", help="skip the depth_count=0 comparison run")
    ap.add_argument("--no-calibration", action="store_true", help="skip the MFMA-only calibration loop")
    ap.add_argument("--cpu-rows", type=int, default=4096)
    ap.add_argument("--rows", type=int, nargs="*", default=None, help="paper_table2: only these row numbers")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is single-GPU; run with --gpus 1 (every (b,h) is independent, "
              "so more GPUs would simply split heads with no communication)", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)

    from paper_2603_15619_amd import moda_attn_fwd, synth

    if args.workload == "copy_calibration":
        return run_copy_calibration(args)
    if args.workload == "mfma_calibration":
        return run_mfma_calibration(args)
    if args.workload == "sweep":
        return run_sweep(args)
    if args.workload == "paper_table2":
        return run_paper_table2(args)
    if args.workload == "decode":
        return run_decode(args)
    if args.workload == "append":
        return run_append(args)
    B, Hq, Hk, T, d, L, dtype = WORKLOADS[args.workload]
    if args.depth_count is not None:
        L = args.depth_count
    if args.workload.startswith("bwd_"):
        return run_backward(args, B, Hq, Hk, T, d, L, dtype)
    inp = synth.make_inputs(B, Hq, Hk, T, d, L, dtype=dtype, seed=2, device="cuda")
    O = torch.empty_like(inp["Q"])
    LSE = torch.empty((B, Hq, T), dtype=torch.float32, device="cuda")

    def run_moda():
        moda_attn_fwd(inp["Q"], inp["Kseq"], inp["Vseq"], inp["Kdepth"], inp["Vdepth"],
                      depth_count=L, out=O, lse=LSE)

    def run_fa():
        moda_attn_fwd(inp["Q"], inp["Kseq"], inp["Vseq"], None, None, depth_count=0, out=O, lse=LSE)

    ms_step, ms_kernel, ms_min = time_calls(run_moda, args.steps, args.warmup)
    # The depth_count = 0 kernel next to it, as interleaved pairs (FA, MoDA, FA, MoDA, ...): each pair
    # gives one ratio t(depth 0) / t(depth L) at the same clock and cache state; the median of the
    # pairs is reported with its spread.
    pairs = None
    if not args.no_fa and L > 0:
        run_fa()
        run_moda()
        torch.cuda.synchronize()
        evs = []
        for _ in range(args.steps):
            e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
            e[0].record()
            run_fa()
            e[1].record()
            run_moda()
            e[2].record()
            evs.append(e)
        torch.cuda.synchronize()
        pairs = [(e[0].elapsed_time(e[1]), e[1].elapsed_time(e[2])) for e in evs]

    flops = fwd_flops(B, Hq, T, d, L)
    value = flops / (ms_step * 1e-3) / 1e12
    achieved = flops / (ms_kernel * 1e-3) / 1e12
    esz = 2 if dtype == "bf16" else 4
    depth_bytes = 2.0 * B * Hk * T * L * d * esz
    # Which roof bounds this workload: the time its algorithmic FLOPs need at the matrix (or, for
    # fp32, vector) peak against the time its algorithmic bytes need at the HBM peak.
    alg_bytes = esz * (B * T * d * (2 * Hq + 2 * Hk) + 2.0 * B * Hk * T * L * d) + 4.0 * B * Hq * T
    stored = measured_traffic(args.workload, "fwd")
    common = {"traffic": stored,
              "traffic_source": ("stored: profiles/traffic.json (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this "
                                 "command), not measured by this run") if stored is not None
              else "no counter run stored for this workload",
              "kernel": ("moda_fwd_bf16_kernel<%d, %d>" % (d, 4 if B * Hq * ((T + 255) // 256) < 256 else 8))
              if dtype == "bf16" else ("moda_fwd_f32_kernel<%d>" % d),
              "kernel_ms_mean": round(ms_kernel, 4), "kernel_ms_min": round(ms_min, 4),
              "flops_per_launch": flops, "bytes_per_launch": alg_bytes}
    if alg_bytes / 8.0e12 > flops / (PEAK_TFLOPS[dtype] * 1e12):
        gbps = alg_bytes / (ms_kernel * 1e-3) / 1e9
        roofline = dict({"bound": "hbm", "achieved": round(gbps, 1), "peak": 8000.0, "unit": "GB/s",
                         "frac": round(gbps / 8000.0, 4)}, **common)
    else:
        roofline = dict({"bound": "mfma" if dtype == "bf16" else "alu", "achieved": round(achieved, 2),
                         "peak": PEAK_TFLOPS[dtype], "unit": "TFLOP/s",
                         "frac": round(achieved / PEAK_TFLOPS[dtype], 4)}, **common)
    out = {
        "metric": "MoDA attn fwd TFLOP/s + ratio to own causal FA kernel at T=64K, 1 GPU",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": dtype, "data": "synthetic",
        "config": {"workload": "%s: B=%d Hq=%d Hk=%d T=%d d=%d depth_count=%d causal fwd" %
                               (args.workload, B, Hq, Hk, T, d, L)},
        "roofline": roofline,
    }
    if pairs is not None:
        fa_ms = float(np.median([a for a, _ in pairs]))
        moda_ms = float(np.median([b for _, b in pairs]))
        ratios = sorted(a / b for a, b in pairs)
        fa_flops = fwd_flops(B, Hq, T, d, 0)
        out["ratio_to_causal_fa"] = round(float(np.median(ratios)), 4)
        out["ratio_to_causal_fa_spread"] = {"min": round(ratios[0], 4), "max": round(ratios[-1], 4),
                                            "pairs": len(ratios), "formed": "median over interleaved (FA, MoDA) pairs"}
        out["causal_fa"] = {"ms_median": round(fa_ms, 4), "tflops": round(fa_flops / (fa_ms * 1e-3) / 1e12, 2)}
        # the depth slots' bytes against the whole call (part of the stream overlaps with other
        # workgroups' key loops, so bytes / extra time is not a bandwidth and is not reported)
        out["depth_segment"] = {"bytes": depth_bytes, "extra_ms_median": round(moda_ms - fa_ms, 4),
                                "gbps_over_whole_call": round(depth_bytes / (ms_step * 1e-3) / 1e9, 1)}
    if dtype == "bf16" and not args.no_calibration:
        cal = mfma_calibration()
        roofline["peak_measured"] = {"mfma_loop_zero_operands": cal["zeros"], "mfma_loop_normal_operands": cal["normal"],
                                     "unit": "TFLOP/s", "kernel": "moda_calibrate_mfma_kernel, this run"}
        if roofline["bound"] == "mfma":
            roofline["frac_of_measured"] = round(achieved / cal["normal"], 4)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(inp, T, d, L, Hq, args.cpu_rows)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
