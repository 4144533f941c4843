"""Benchmark of the BigBird block-sparse attention hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

A step is one pass of the hot path over one synthetic batch of the BERT-base-shaped
workload (bf16, B=4, H=12, n=4096, d=64, b=64, g/w/r = 2/3/3 blocks): the forward call
bigbird_attn_fwd (one fused kernel; the global rows are merged inside it).  Inputs are resident
in HBM before the timed region.  Prints ONE JSON line.

Timing: W warm-up steps, then K timed steps between two events on the launch stream give
`ms_per_step` (the contract's figure).  Because K steps of this kernel can be as short as a
millisecond, during which the clocks have not settled, the headline `value` comes from a longer
measurement made right after it: a warm-up of at least 50 ms of launches, then `--batches`
batches of at least 10 ms each, of which the median time per step is taken (minimum and the
K-step figure are reported beside it).

metric/value: useful TFLOP/s = 4 b^2 d flop per (query block, key block) pair of the
pattern (App. D cost O(n (g+w+r) b d)) divided by the time per step.
roofline: the same flops against the dense bf16 MFMA peak (256 CUs x 2.4 GHz x 4096
flop/clk/CU); the kernel time is measured with HIP events on the launch stream.
cpu_baseline: the fp64 oracle (dense mask, NumPy) timed on the host cores over a
bounded sample of the same workload.
Before anything is printed, sampled rows of the output that was just timed are compared with the
oracle; a mismatch beyond the tolerance aborts the run.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import statistics
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import bigbird_inputs as inp  # noqa: E402

BF16_MFMA_PEAK_TFLOPS = 256 * 2.4e9 * 4096 / 1e12     # 2516.6, dense
FP32_MFMA_PEAK_TFLOPS = 157.3
HBM_PEAK_GBPS = 8000.0
WORKLOAD = "cfg2_bert_base"
TOL = {"bf16": 2e-2, "f32": 1e-4}


def useful_flops_fwd(pairs: int, b: int, d: int) -> float:
    return 4.0 * b * b * d * pairs


def algorithmic_bytes_fwd(wl) -> int:
    """Compulsory HBM traffic of a forward call: Q, K, V read, O written, LSE written."""
    el = 2 if wl.dtype == "bf16" else 4
    return wl.B * wl.H * (4 * wl.n * wl.d * el + 4 * wl.n)


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


def timed(torch, fns, n):
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(n):
        for f in fns:
            f()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / n


def settled_ms(torch, fns, batches: int, min_warm_ms: float = 50.0, min_batch_ms: float = 10.0):
    """Median / minimum ms per step over `batches` batches of >= min_batch_ms each, after a warm-up
    of >= min_warm_ms of launches (the library launches on torch's current stream, so events on
    that stream bracket the kernels)."""
    est = max(timed(torch, fns, 20), 1e-4)
    timed(torch, fns, max(20, int(min_warm_ms / est) + 1))
    per_batch = max(20, int(min_batch_ms / est) + 1)
    ms = [timed(torch, fns, per_batch) for _ in range(batches)]
    return statistics.median(ms), min(ms), per_batch


def check_rows_against_oracle(wl, t, rand_idx, O, LSE, n_slices: int = 3, seed: int = 0,
                              skip_padded_query_blocks: bool = False):
    """Sampled rows (both global blocks, blocks 1 and nb-2, random interior blocks) of a few
    (batch, head) slices of the output just timed, against the oracle.  Returns the worst errors."""
    import oracle
    rng = np.random.default_rng(seed)
    Oh = O.float().cpu().numpy().astype(np.float64)
    Lh = LSE.cpu().numpy().astype(np.float64)
    picks = {(0, 0), (wl.B - 1, wl.H - 1)} | {(int(rng.integers(wl.B)), int(rng.integers(wl.H)))
                                             for _ in range(n_slices)}
    worst_o = worst_l = 0.0
    for (bi, h) in sorted(picks):
        blocks = {0, wl.nb - 1, 1, wl.nb - 2} | {int(x) for x in rng.integers(2, max(3, wl.nb - 2), size=6)}
        rows = sorted({j * wl.b + o for j in blocks if 0 <= j < wl.nb for o in (0, 31, 32, wl.b - 1)})
        Or, Lr = oracle.attn_fwd_rows(t["Q"], t["K"], t["V"], rand_idx, wl.b, wl.g, wl.w, wl.scale,
                                      bi, h, rows, key_mask=t.get("key_mask"),
                                      skip_padded_query_blocks=skip_padded_query_blocks)
        fin = np.isfinite(Lr)
        if not (Lh[bi, h, rows][~fin] == -np.inf).all():
            return float("inf"), float("inf")
        worst_o = max(worst_o, float(np.abs(Oh[bi, h, rows] - Or).max()))
        if fin.any():
            worst_l = max(worst_l, float(np.abs(Lh[bi, h, rows][fin] - Lr[fin]).max()))
    return worst_o, worst_l


def time_cpu_oracle(wl, t, rand_idx, sample_heads: int, repeats: int = 2):
    """Oracle forward on every batch, the first `sample_heads` heads, `repeats` times over
    (mean time of one pass), on the host cores NumPy uses."""
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
                  f"{repeats} passes (fp64 dense-mask NumPy oracle, {dt:.2f} s per pass; only its two "
                  f"matrix products use all {cores} threads, the masking, exponentials and sums run on one)",
        "seconds": dt,
    }


def forward_line(bb, torch, dev, name: str, batches: int, skip_padded_query_blocks: bool = False):
    """Forward timing of another workload: median ms, useful TFLOP/s, fraction of the peak of its
    arithmetic type, algorithmic GB/s.  With skip_padded_query_blocks the call carries
    BB_SKIP_PADDED_QUERY_BLOCKS (query blocks without a valid position are not computed, and their
    pairs are not counted as useful work)."""
    wl = inp.WORKLOADS[name]
    flags = bb.BB_SKIP_PADDED_QUERY_BLOCKS if skip_padded_query_blocks else 0
    rand_idx = bb.bigbird_make_rand_idx(wl.H, wl.n, wl.b, wl.g, wl.w, wl.r, wl.pattern_seed)
    t, dv = device_inputs(wl, torch, dev)
    ridx = torch.from_numpy(rand_idx).to(dev)
    pairs = bb.bigbird_count_block_pairs(rand_idx, t.get("key_mask"), wl.B, wl.H, wl.n, wl.b, wl.g, wl.w, wl.r,
                                         flags)
    O = torch.empty_like(dv["Q"])
    LSE = torch.empty((wl.B, wl.H, wl.n), dtype=torch.float32, device=dev)
    ws = torch.empty(max(bb.bigbird_attn_workspace_bytes(wl.B, wl.H, wl.n, wl.d, wl.b, wl.g, wl.w, wl.r), 256),
                     dtype=torch.uint8, device=dev)
    step = bb.prepare_attn_fwd(dv["Q"], dv["K"], dv["V"], ridx, O, LSE, ws, g=wl.g, w=wl.w,
                               scale=wl.scale, key_padding_mask=dv["key_mask"], global_mode=flags)
    med, mn, _ = settled_ms(torch, (step,), batches)
    err_o, err_l = check_rows_against_oracle(wl, t, rand_idx, O, LSE, n_slices=1,
                                             skip_padded_query_blocks=skip_padded_query_blocks)
    if err_o > TOL[wl.dtype] or err_l > TOL[wl.dtype]:
        raise SystemExit(f"bench: {name}: timed output does not match the oracle "
                         f"(max|dO|={err_o:.3e}, max|dLSE|={err_l:.3e})")
    fl = useful_flops_fwd(pairs, wl.b, wl.d)
    peak = BF16_MFMA_PEAK_TFLOPS if wl.dtype == "bf16" else FP32_MFMA_PEAK_TFLOPS
    return {"workload": wl.name + (" + BB_SKIP_PADDED_QUERY_BLOCKS" if skip_padded_query_blocks else ""),
            "dtype": wl.dtype, "block_pairs_with_valid_keys": pairs,
            "ms_per_step_median": med, "ms_per_step_min": mn,
            "useful_tflops": fl / (med * 1e-3) / 1e12,
            "frac_of_mfma_peak": fl / (med * 1e-3) / 1e12 / peak,
            "algorithmic_gb_per_s": algorithmic_bytes_fwd(wl) / (med * 1e-3) / 1e9,
            "oracle_check": {"max_abs_dO": err_o, "max_abs_dLSE": err_l}}


def etc_forward_lines(bb, torch, dev, batches: int):
    """Forward timings of the ETC construction (Sec. 2: extra global tokens in front) at b = 64, total
    length 4096, 12 heads, window of 3 blocks, no random blocks: 256 global tokens (four leading
    global blocks) and 230 (App. E's NaturalQ figure: the fourth block padded with a key mask,
    which sends every item through the per-key masking path)."""
    import oracle
    out = []
    B, H, n, b, w, scale = 4, 12, 4096, 64, 3, 0.125
    for n_global in (256, 230):
        g = (n_global + b - 1) // b
        t = inp.make_tensors(B, H, n, 64, 150 + n_global, "bf16")
        km_h = None
        if g * b != n_global:
            km_h = np.ones((B, n), dtype=np.uint8)
            km_h[:, n_global:g * b] = 0
        dv = {x: torch.from_numpy(t[x + "_bits"].view(np.int16)).to(dev).view(torch.bfloat16) for x in ("Q", "K", "V")}
        km = None if km_h is None else torch.from_numpy(km_h).to(dev)
        empty_h = np.full((H, n // b, 0), -1, dtype=np.int32)
        empty = torch.zeros((H, n // b, 0), dtype=torch.int32, device=dev)
        O = torch.empty_like(dv["Q"])
        LSE = torch.empty((B, H, n), dtype=torch.float32, device=dev)
        ws = torch.empty(max(bb.bigbird_attn_workspace_bytes(B, H, n, 64, b, g, w, 0), 256), dtype=torch.uint8, device=dev)
        step = bb.prepare_attn_fwd(dv["Q"], dv["K"], dv["V"], empty, O, LSE, ws, g=g, w=w, scale=scale,
                                   key_padding_mask=km, global_mode=bb.BB_GLOBAL_LEADING)
        med, mn, _ = settled_ms(torch, (step,), batches)
        rows = [0, 100, n_global - 1, g * b, g * b + 31, 2000, n - 1]
        Or, Lr = oracle.attn_fwd_rows(t["Q"], t["K"], t["V"], empty_h, b, g, w, scale, B - 1, H - 1, rows,
                                      key_mask=km_h, global_mode=oracle.GLOBAL_LEADING)
        err_o = float(np.abs(O.float().cpu().numpy()[B - 1, H - 1, rows] - Or).max())
        err_l = float(np.abs(LSE.cpu().numpy()[B - 1, H - 1, rows] - Lr).max())
        if err_o > TOL["bf16"] or err_l > TOL["bf16"]:
            raise SystemExit(f"bench: ETC n_global={n_global}: timed output does not match the oracle "
                             f"(max|dO|={err_o:.3e}, max|dLSE|={err_l:.3e})")
        kbv = None if km_h is None else km_h
        pairs = bb.bigbird_count_block_pairs(empty_h, kbv, B, H, n, b, g, w, 0, bb.BB_GLOBAL_LEADING)
        fl = useful_flops_fwd(pairs, b, 64)
        out.append({"workload": f"etc_{n_global}_global_tokens", "n_global": n_global, "leading_global_blocks": g,
                    "block_pairs_with_valid_keys": pairs, "ms_per_step_median": med, "ms_per_step_min": mn,
                    "useful_tflops": fl / (med * 1e-3) / 1e12,
                    "frac_of_mfma_peak": fl / (med * 1e-3) / 1e12 / BF16_MFMA_PEAK_TFLOPS,
                    "oracle_check": {"max_abs_dO": err_o, "max_abs_dLSE": err_l}})
    return out


def time_fwd_bwd(bb, torch, dev, batches: int):
    """Forward + backward on the cfg4 workload (B=2): ms per step and useful TFLOP/s.

    Useful flops: 4 b^2 d per block pair forward, 10 b^2 d backward (five matmuls); the two
    backward kernels recompute the scores, so 14 b^2 d are executed.
    """
    wl = inp.WORKLOADS["cfg4_fwd_bwd"]
    rand_idx = bb.bigbird_make_rand_idx(wl.H, wl.n, wl.b, wl.g, wl.w, wl.r, wl.pattern_seed)
    t, dv = device_inputs(wl, torch, dev)
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
        med, mn, _ = settled_ms(torch, fns, batches)
        fl = mult * wl.b * wl.b * wl.d * pairs
        out[name] = {"ms_per_step_median": med, "ms_per_step_min": mn,
                     "useful_tflops": fl / (med * 1e-3) / 1e12,
                     "pct_of_bf16_mfma_peak": 100.0 * fl / (med * 1e-3) / 1e12 / BF16_MFMA_PEAK_TFLOPS}
    # the same step with attention dropout 0.1 (App. E.1): the bf16 forward then runs its per-item
    # path; the outputs of the timed calls are checked against the dropout oracle on sampled rows
    p_drop, seed = 0.1, 20200728
    fwd_d = bb.prepare_attn_fwd(dv["Q"], dv["K"], dv["V"], ridx, O, LSE, ws, g=wl.g, w=wl.w, scale=wl.scale,
                                p_drop=p_drop, seed=seed)
    bwd_d = bb.prepare_attn_bwd(dv["Q"], dv["K"], dv["V"], O, LSE, dv["dO"], ridx, *grads, ws,
                                g=wl.g, w=wl.w, scale=wl.scale, p_drop=p_drop, seed=seed)
    drop = {"p_drop": p_drop}
    for name, fns, mult in (("forward", (fwd_d,), 4.0), ("backward", (bwd_d,), 10.0),
                            ("forward_backward", (fwd_d, bwd_d), 14.0)):
        med, mn, _ = settled_ms(torch, fns, batches)
        fl = mult * wl.b * wl.b * wl.d * pairs
        drop[name] = {"ms_per_step_median": med, "ms_per_step_min": mn,
                      "useful_tflops": fl / (med * 1e-3) / 1e12,
                      "pct_of_bf16_mfma_peak": 100.0 * fl / (med * 1e-3) / 1e12 / BF16_MFMA_PEAK_TFLOPS}
    import oracle
    torch.cuda.synchronize()
    Oh = O.float().cpu().numpy().astype(np.float64)
    worst = 0.0
    rng = np.random.default_rng(1)
    for (bi, h) in ((0, 0), (wl.B - 1, wl.H - 1)):
        rows = sorted({j * wl.b + o for j in (0, 1, wl.nb - 1, int(rng.integers(2, wl.nb - 2))) for o in (0, 33, wl.b - 1)})
        Or, _ = oracle.attn_fwd_dropout_rows(t["Q"], t["K"], t["V"], rand_idx, wl.b, wl.g, wl.w, wl.scale,
                                             p_drop, seed, bi, h, rows)
        worst = max(worst, float(np.abs(Oh[bi, h, rows] - Or).max()))
    if not worst <= 2e-2:
        raise SystemExit(f"bench.py: dropout forward disagrees with the oracle: max|dO| = {worst:.3e}")
    drop["oracle_check_max_abs_err_O"] = worst
    out["dropout"] = drop
    out["workload"] = wl.name
    out["block_pairs"] = pairs
    return out


def measured_traffic():
    """HBM bytes per forward call from the committed rocprofv3 counter summary, with the kernel
    source revision it was taken at; (None, None) if the summary is missing."""
    path = os.path.join(ROOT, "profiles", "fwd_kernel_bf16_cfg2_hbm_traffic.md")
    nbytes = rev = None
    try:
        for line in open(path):
            if line.startswith("hbm_bytes_per_launch_fwd_total"):
                nbytes = int(line.split("=")[1])
            m = re.match(r"kernel_source_sha256\s*=\s*(\w+)", line)
            if m:
                rev = m.group(1)
    except OSError:
        pass
    return nbytes, rev


def kernel_source_sha256() -> str:
    import hashlib
    h = hashlib.sha256()
    with open(os.path.join(ROOT, "paper_2007_14062_amd", "csrc", "fwd_bf16.hip"), "rb") as f:
        h.update(f.read())
    return h.hexdigest()[:16]


def device_clock_mhz():
    """Shader clock level the driver reports as current right after the timed runs (sysfs,
    pp_dpm_sclk, the starred line), or None.  Read from a file: a process that has initialised
    the GPU starts no other program."""
    import glob
    for path in sorted(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk")):
        try:
            with open(path) as f:
                for line in f:
                    if "*" in line:
                        m = re.search(r"(\d+)\s*Mhz", line, re.I)
                        if m:
                            return float(m.group(1))
        except OSError:
            continue
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=500)
    ap.add_argument("--batches", type=int, default=7, help="batches of the settled measurement (median taken)")
    ap.add_argument("--cpu-sample-heads", type=int, default=12)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--skip-backward", action="store_true",
                    help="leave out the forward+backward timing on the cfg4 workload (extra fields only)")
    ap.add_argument("--skip-other-workloads", action="store_true",
                    help="leave out the forward timings of the other workload shapes (extra fields only)")
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

    # the contract's measurement: W warm-up steps, K timed steps
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ksteps_ms = timed(torch, (step,), args.steps)
    wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    # the settled measurement the headline uses
    med_ms, min_ms, per_batch = settled_ms(torch, (step,), args.batches)
    tflops = flops / (med_ms * 1e-3) / 1e12

    err_o, err_l = check_rows_against_oracle(wl, t, rand_idx, O, LSE)
    if err_o > TOL[wl.dtype] or err_l > TOL[wl.dtype]:
        raise SystemExit(f"bench: the timed output does not match the oracle (max|dO|={err_o:.3e}, "
                         f"max|dLSE|={err_l:.3e}, tolerance {TOL[wl.dtype]}): no value printed")

    props = torch.cuda.get_device_properties(dev)
    clock_khz = getattr(props, "clock_rate", 0) or 0
    sclk = device_clock_mhz()
    device = {"name": props.name, "compute_units": props.multi_processor_count,
              "max_clock_mhz": clock_khz / 1e3 if clock_khz else "unavailable",
              "sclk_mhz_after_run": sclk if sclk is not None else "unavailable"}
    if clock_khz:
        # the same formula as the published peak, with what the device reports
        device["bf16_mfma_peak_tflops_at_reported_clock"] = props.multi_processor_count * clock_khz * 1e3 * 4096 / 1e12
    traffic, traffic_rev = measured_traffic()
    traffic_fresh = traffic is not None and traffic_rev == kernel_source_sha256()
    alg_bytes = algorithmic_bytes_fwd(wl)
    result = {
        "metric": "useful TFLOP/s, BigBird block-sparse attention forward (n=4096, H=12, d=64, b=64)",
        "value": tflops,
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": med_ms,
        "ms_per_step_min": min_ms,
        "ms_per_step_k_steps": ksteps_ms,
        "wall_ms_per_step": wall_ms,
        "timing": f"median of {args.batches} batches of {per_batch} steps after >= 50 ms of warm-up launches; "
                  f"ms_per_step_k_steps is the plain {args.steps}-step figure after {args.warmup} warm-up steps",
        "higher_is_better": True,
        "scaling": "none (one GPU; every (batch, head) slice is independent)",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": wl.name, "B": wl.B, "H": wl.H, "n": wl.n, "d": wl.d, "b": wl.b,
                   "g": wl.g, "w": wl.w, "r": wl.r, "block_pairs": pairs,
                   "useful_gflop_per_step": flops / 1e9, "pass": "forward"},
        "pct_of_bf16_mfma_peak": 100.0 * tflops / BF16_MFMA_PEAK_TFLOPS,
        "oracle_check": {"max_abs_dO": err_o, "max_abs_dLSE": err_l, "tolerance": TOL[wl.dtype],
                         "rows": "sampled rows of 3-5 (batch, head) slices of the timed output"},
        "device": device,
        "roofline": {"bound": "mfma", "achieved": tflops, "peak": BF16_MFMA_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": tflops / BF16_MFMA_PEAK_TFLOPS,
                     # HBM bytes per launch from the rocprofv3 counter runs in profiles/ -- only if that
                     # summary was taken with this very kernel source
                     "traffic": traffic if traffic_fresh else None,
                     "traffic_note": ("rocprofv3 FETCH_SIZE/WRITE_SIZE summary in profiles/ matches this kernel source"
                                      if traffic_fresh else
                                      "profiles/ traffic summary is older than the kernel source (or absent): not quoted"),
                     "algorithmic_bytes": alg_bytes,
                     "algorithmic_gb_per_s": alg_bytes / (med_ms * 1e-3) / 1e9,
                     "hbm_gb_per_s": (traffic / (med_ms * 1e-3) / 1e9) if traffic_fresh else None,
                     "hbm_peak_gb_per_s": HBM_PEAK_GBPS,
                     "kernel": "bb::fwd_kernel_bf16 (the only kernel of a forward call at this size)"},
    }
    if not args.skip_other_workloads:
        result["etc_forward"] = etc_forward_lines(bb, torch, dev, max(3, args.batches // 2))
        result["other_workloads_forward"] = [forward_line(bb, torch, dev, nm, max(3, args.batches // 2))
                                             for nm in ("cfg1_fp32_small", "cfg3_key_padding", "cfg5_long_seq")]
        result["other_workloads_forward"].append(
            forward_line(bb, torch, dev, "cfg3_key_padding", max(3, args.batches // 2), skip_padded_query_blocks=True))
    if not args.skip_backward:
        result["fwd_bwd_cfg4"] = time_fwd_bwd(bb, torch, dev, max(3, args.batches // 2))
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = time_cpu_oracle(wl, t, rand_idx, args.cpu_sample_heads)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
