"""Benchmark of the BigBird block-sparse attention hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

A step is one pass of the hot path over one synthetic batch of the BERT-base-shaped
workload (bf16, B=4, H=12, n=4096, d=64, b=64, g/w/r = 2/3/3 blocks): the forward call
bigbird_attn_fwd (one fused kernel; the global rows are merged inside it).  Inputs are resident
in HBM before the timed region.  Prints ONE JSON line.

metric/value: useful TFLOP/s = 4 b^2 d flop per (query block, key block) pair of the
pattern (App. D cost O(n (g+w+r) b d)) divided by the time per step.
roofline: the same flops against the dense bf16 MFMA peak (256 CUs x 2.4 GHz x 4096
flop/clk/CU); the kernel time is measured with HIP events on the launch stream.
cpu_baseline: the fp64 oracle (dense mask, NumPy) timed on the host cores over a
bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import bigbird_inputs as inp  # noqa: E402

BF16_MFMA_PEAK_TFLOPS = 256 * 2.4e9 * 4096 / 1e12     # 2516.6, dense
WORKLOAD = "cfg2_bert_base"


def useful_flops_fwd(pairs: int, b: int, d: int) -> float:
    return 4.0 * b * b * d * pairs


def device_inputs(wl, torch, dev):
    t = inp.workload_tensors(wl)
    out = {}
    for name in ("Q", "K", "V") + (("dO",) if wl.backward else ()):
        if wl.dtype == "bf16":
            out[name] = torch.from_numpy(t[name + "_bits"].view(np.int16)).to(dev).view(torch.bfloat16)
        else:
            out[name] = torch.from_numpy(t[name]).to(dev)
    km = t.get("key_mask")
    out["key_mask"] = None if km is None else torch.from_numpy(km).to(dev)
    return t, out


def time_cpu_oracle(wl, t, rand_idx, sample_heads: int, repeats: int = 2):
    """Oracle forward on every batch, the first `sample_heads` heads, `repeats` times over
    (mean time of one pass), on all host cores NumPy uses."""
    import oracle
    Q, K, V = (t[x][:, :sample_heads] for x in ("Q", "K", "V"))
    t0 = time.perf_counter()
    for _ in range(repeats):
        oracle.attn_fwd(Q, K, V, rand_idx[:sample_heads], wl.b, wl.g, wl.w, wl.scale)
    dt = (time.perf_counter() - t0) / repeats
    pairs = wl.B * oracle.count_block_pairs(rand_idx[:sample_heads], wl.n, wl.b, wl.g, wl.w)
    try:
        cores = len(os.sched_getaffinity(0))
    except AttributeError:
        cores = os.cpu_count() or 1
    env_threads = os.environ.get("OMP_NUM_THREADS")
    if env_threads and env_threads.isdigit():
        cores = min(cores, int(env_threads))
    return {
        "value": useful_flops_fwd(pairs, wl.b, wl.d) / dt / 1e12,
        "unit": "useful TFLOP/s",
        "cores": cores,
        "kind": "oracle",
        "sample": f"forward of all {wl.B} batches, heads 0..{sample_heads - 1} of {wl.name}, "
                  f"{repeats} passes (fp64 dense-mask NumPy oracle, {dt:.2f} s per pass)",
        "seconds": dt,
    }


def time_fwd_bwd(bb, torch, dev, steps: int, warmup: int):
    """Forward + backward on the cfg4 workload (B=2): ms per step and useful TFLOP/s.

    Useful flops: 4 b^2 d per block pair forward, 10 b^2 d backward (five matmuls); the two
    backward kernels recompute the scores, so 14 b^2 d are executed.
    """
    wl = inp.WORKLOADS["cfg4_fwd_bwd"]
    rand_idx = bb.bigbird_make_rand_idx(wl.H, wl.n, wl.b, wl.g, wl.w, wl.r, wl.pattern_seed)
    _, dv = device_inputs(wl, torch, dev)
    ridx = torch.from_numpy(rand_idx).to(dev)
    pairs = bb.bigbird_count_block_pairs(rand_idx, None, wl.B, wl.H, wl.n, wl.b, wl.g, wl.w, wl.r)
    O = torch.empty_like(dv["Q"])
    LSE = torch.empty((wl.B, wl.H, wl.n), dtype=torch.float32, device=dev)
    grads = [torch.empty(dv["Q"].shape, dtype=torch.float32, device=dev) for _ in range(3)]
    ws = torch.empty(bb.bigbird_attn_workspace_bytes(wl.B, wl.H, wl.n, wl.d, wl.b, wl.g, wl.w, wl.r, True),
                     dtype=torch.uint8, device=dev)
    fwd = bb.prepare_attn_fwd(dv["Q"], dv["K"], dv["V"], ridx, O, LSE, ws, g=wl.g, w=wl.w, scale=wl.scale)
    bwd = bb.prepare_attn_bwd(dv["Q"], dv["K"], dv["V"], O, LSE, dv["dO"], ridx, *grads, ws,
                              g=wl.g, w=wl.w, scale=wl.scale)
    out = {}
    for name, fns, mult in (("forward", (fwd,), 4.0), ("backward", (bwd,), 10.0),
                            ("forward_backward", (fwd, bwd), 14.0)):
        for _ in range(warmup):
            for f in fns:
                f()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            for f in fns:
                f()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / steps
        fl = mult * wl.b * wl.b * wl.d * pairs
        out[name] = {"ms_per_step": ms, "useful_tflops": fl / (ms * 1e-3) / 1e12,
                     "pct_of_bf16_mfma_peak": 100.0 * fl / (ms * 1e-3) / 1e12 / BF16_MFMA_PEAK_TFLOPS}
    out["workload"] = wl.name
    out["block_pairs"] = pairs
    return out


def measured_traffic_bytes():
    """HBM bytes per forward call from the committed rocprofv3 counter summary (None if absent)."""
    path = os.path.join(ROOT, "profiles", "fwd_kernel_bf16_cfg2_hbm_traffic.md")
    try:
        for line in open(path):
            if line.startswith("hbm_bytes_per_launch_fwd_total"):
                return int(line.split("=")[1])
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=500)
    ap.add_argument("--cpu-sample-heads", type=int, default=12)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--skip-backward", action="store_true",
                    help="leave out the forward+backward timing on the cfg4 workload (extra fields only)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain 256 MiB device copy 10 times (known HBM traffic: 256 MiB read, "
                         "256 MiB written per copy), to scale the rocprofv3 FETCH_SIZE / WRITE_SIZE counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (every (batch, head) "
              "slice is independent, so sharding is a plain split); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2007_14062_amd as bb

    if not torch.cuda.is_available():
        print("bench.py needs a GPU: the library has no CPU path", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")
    if args.copy_calibration:
        src = torch.ones(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes": 256 << 20, "copies": 10}))
        return
    wl = inp.WORKLOADS[WORKLOAD]
    rand_idx = bb.bigbird_make_rand_idx(wl.H, wl.n, wl.b, wl.g, wl.w, wl.r, wl.pattern_seed)
    t, dv = device_inputs(wl, torch, dev)
    ridx = torch.from_numpy(rand_idx).to(dev)
    pairs = bb.bigbird_count_block_pairs(rand_idx, None, wl.B, wl.H, wl.n, wl.b, wl.g, wl.w, wl.r)
    flops = useful_flops_fwd(pairs, wl.b, wl.d)

    O = torch.empty_like(dv["Q"])
    LSE = torch.empty((wl.B, wl.H, wl.n), dtype=torch.float32, device=dev)
    ws_bytes = bb.bigbird_attn_workspace_bytes(wl.B, wl.H, wl.n, wl.d, wl.b, wl.g, wl.w, wl.r)
    ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=dev)

    # arguments marshalled once: each step is exactly one bigbird_attn_fwd C call
    step = bb.prepare_attn_fwd(dv["Q"], dv["K"], dv["V"], ridx, O, LSE, ws, g=wl.g, w=wl.w,
                               scale=wl.scale, key_padding_mask=dv["key_mask"])

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # the library launches on torch's current stream, so events on that stream bracket the kernels
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for _ in range(args.steps):
        step()
    ev1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    ev_ms = ev0.elapsed_time(ev1) / args.steps
    ms = max(ev_ms, 1e-9)
    tflops = flops / (ms * 1e-3) / 1e12

    props = torch.cuda.get_device_properties(dev)
    clock_khz = getattr(props, "clock_rate", 0) or 0
    device = {"name": props.name, "compute_units": props.multi_processor_count,
              "max_clock_mhz": clock_khz / 1e3 if clock_khz else None,   # not reported by every runtime
              # the same formula as the published peak, with what the device reports
              "bf16_mfma_peak_tflops_at_reported_clock":
                  props.multi_processor_count * clock_khz * 1e3 * 4096 / 1e12 if clock_khz else None}
    result = {
        "metric": "useful TFLOP/s, BigBird block-sparse attention forward (n=4096, H=12, d=64, b=64)",
        "value": tflops,
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms,
        "wall_ms_per_step": wall_ms,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": wl.name, "B": wl.B, "H": wl.H, "n": wl.n, "d": wl.d, "b": wl.b,
                   "g": wl.g, "w": wl.w, "r": wl.r, "block_pairs": pairs,
                   "useful_gflop_per_step": flops / 1e9, "pass": "forward"},
        "pct_of_bf16_mfma_peak": 100.0 * tflops / BF16_MFMA_PEAK_TFLOPS,
        "device": device,
        "roofline": {"bound": "mfma", "achieved": tflops, "peak": BF16_MFMA_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": tflops / BF16_MFMA_PEAK_TFLOPS,
                     "traffic": measured_traffic_bytes(),
                     "kernel": "bb::fwd_kernel_bf16 (the only kernel of a forward call at this size)"},
    }
    if not args.skip_backward:
        result["fwd_bwd_cfg4"] = time_fwd_bwd(bb, torch, dev, max(1, args.steps // 4), max(1, args.warmup // 4))
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = time_cpu_oracle(wl, t, rand_idx, args.cpu_sample_heads)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
