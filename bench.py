#!/usr/bin/env python3
"""Benchmark of the Lightning Attention hot path on one MI355X.

One "step" = one forward + one backward call of the library on the headline workload
(7B-shaped layer: Bt=4, H=32, N=8192, D=128, bf16 tensors, fp32 accumulation), with
all tensors resident in HBM before the timed region.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--preroll SECONDS] [--workload cfg3_7b|cfg2_385m|cfg_1b]
                  [--no-cpu-baseline] [--report] [--copy-calibration]
  python bench.py --traffic-from FETCH.csv WRITE.csv      (no GPU: counter CSVs -> profiles/hbm_traffic_*.json)
  (--report adds the other workloads to stderr; --copy-calibration and --preroll 0 are for counter runs)
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

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X published dense bf16 MFMA rate
MFMA_FP32_PEAK_TFLOPS = 157.3   # MI355X published fp32 matrix rate


def flops_per_token_head(D: int, B: int, plan_fwd=(0, 1), plan_bwd=(0, 1)):
    """FLOP conventions per token-head (one multiply or one add = 1 FLOP), fwd+bwd.
    plan_* = (value columns per workgroup, segments per chain) the library takes for the call."""
    def issued(passes, plan):
        # One decayed pass per token-head: 4 D^2 for the two state products (state update, query times
        # state); per 64-token block 10 of 16 score tiles, recomputed by each of the D/dv value-column
        # slices of a chain, and 12 of 16 score-times-value tiles; a chain cut into segments also runs the
        # state-only sweep (one more state update, 2 D^2).
        dv, segs = plan
        slices = D // dv if dv else 1
        return passes * ((1.25 * slices + 1.5) * B * D + 4 * D * D + (2 * D * D if segs > 1 else 0))
    return {
        "F_min": 14 * D * D,                               # recurrent form, block independent
        "F_alg": 14 * D * D + 7 * (B + 1) * D,             # blockwise method, causal half of each tile
        "F_exec": issued(1, plan_fwd) + issued(3, plan_bwd),   # what the kernels issue under the plan taken
    }


def algorithmic_bytes_per_token_head(D: int, esize: int):
    """Ideal HBM traffic: fwd reads Q,K,V writes O; bwd reads Q,K,V,dO writes dQ,dK,dV."""
    return {"fwd": 4 * D * esize, "bwd": 7 * D * esize}


def kernel_source_hash() -> str:
    """Fingerprint of the sources of the timed kernels: a stored traffic measurement is only
    quoted while it matches."""
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2307_14995_amd", "csrc")
    for name in ("ltn_pass_bf16.hip", "ltn_pass_f32_mfma.hip", "ltn_bf16_tiles.h", "ltn_kernels.h", "ltn_api.hip"):
        with open(os.path.join(csrc, name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def traffic_profile_path(workload: str) -> str:
    return os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}.json")


def stored_traffic(workload: str, kernel: str):
    """HBM bytes per launch of `kernel` as measured by the counter runs (rocprofv3 --pmc FETCH_SIZE, then
    WRITE_SIZE, each scaled by the same counter's reading of a plain copy of known size), read from
    profiles/; None when there is no measurement of the kernels as they stand."""
    try:
        with open(traffic_profile_path(workload)) as f:
            rec = json.load(f)
    except (OSError, ValueError):
        return None
    if rec.get("kernel_source_hash") != kernel_source_hash():
        return None
    return rec.get("kernels", {}).get(kernel, {}).get("hbm_bytes_per_launch")


def write_traffic_profile(workload: str, fetch_csv: str, write_csv: str) -> int:
    """Turn the two counter-collection CSVs of
        rocprofv3 --pmc FETCH_SIZE -- python3 bench.py --steps 3 --warmup 1 --preroll 0 --no-cpu-baseline --copy-calibration
        rocprofv3 --pmc WRITE_SIZE -- (same)
    into profiles/hbm_traffic_<workload>.json: per kernel, mean counter value per launch, scaled by what the
    same counter read for the calibration copy (1 GiB read, 1 GiB written)."""
    import csv
    import re

    def per_kernel(path, counter):
        acc = {}
        with open(path, newline="") as f:
            for row in csv.DictReader(f):
                if row["Counter_Name"] != counter:
                    continue
                acc.setdefault(row["Kernel_Name"], []).append(float(row["Counter_Value"]))
        return acc

    GIB = float(1 << 30)
    out = {"workload": workload, "kernel_source_hash": kernel_source_hash(), "kernels": {},
           "how": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (KiB per dispatch), one counter per run, scaled by the "
                  "counter's reading of a 1 GiB device-to-device copy in the same run"}
    fetch, write = per_kernel(fetch_csv, "FETCH_SIZE"), per_kernel(write_csv, "WRITE_SIZE")
    cal_f = [v for k, vs in fetch.items() if "copyBuffer" in k for v in vs if v > 1e5]
    cal_w = [v for k, vs in write.items() if "copyBuffer" in k for v in vs if v > 1e5]
    if not cal_f or not cal_w:
        print("no calibration copy found in the counter runs (run bench.py with --copy-calibration)", file=sys.stderr)
        return 1
    sf, sw = GIB / (sum(cal_f) / len(cal_f) * 1024.0), GIB / (sum(cal_w) / len(cal_w) * 1024.0)
    out["scale"] = {"FETCH_SIZE": round(sf, 4), "WRITE_SIZE": round(sw, 4)}
    for name in fetch:
        m = re.search(r"pass_bf16_kernel<(\d+), (\d+), (\d+)", name)
        mf = re.search(r"pass_f32_mfma_kernel<(\d+), (\d+), (\d+)", name)
        if not (m or mf) or name not in write:
            continue
        if m:
            key = f"pass_bf16_kernel<{m.group(1)},{m.group(2)}>" + ("" if m.group(3) == "0" else f" mode {m.group(3)}")
        else:
            key = f"pass_f32_mfma_kernel<{mf.group(1)},{mf.group(2)},{mf.group(3)}>"
        rd = sum(fetch[name]) / len(fetch[name]) * 1024.0 * sf
        wr = sum(write[name]) / len(write[name]) * 1024.0 * sw
        out["kernels"][key] = {"launches": len(fetch[name]), "read_bytes_per_launch": round(rd),
                               "written_bytes_per_launch": round(wr), "hbm_bytes_per_launch": round(rd + wr)}
    with open(traffic_profile_path(workload), "w") as f:
        json.dump(out, f, indent=1)
        f.write("\n")
    print(json.dumps(out))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # defaults: 100 warm-up and 400 timed steps are about 0.4 s of GPU time; the clock ramp of an idle GPU
    # is taken out by the pre-roll below, whatever --warmup says
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--preroll", type=float, default=6.0,
                    help="upper bound, in seconds, of the untimed pre-roll that brings the GPU to sustained "
                         "clocks before the warm-up steps (0 = none; counter runs use 0)")
    ap.add_argument("--traffic-from", nargs=2, metavar=("FETCH_CSV", "WRITE_CSV"),
                    help="no GPU work: write profiles/hbm_traffic_<workload>.json from two counter-collection CSVs")
    ap.add_argument("--workload", default="cfg3_7b")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--report", action="store_true")
    ap.add_argument("--sections", default="",
                    help="with --report: comma-separated subset of machine,shapes,fp32,gated,tiled,lrpe,dims,decode")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="first run one untimed 1 GiB device-to-device copy, so that a counter run "
                         "(rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE) holds a kernel of known traffic")
    args = ap.parse_args()
    if args.traffic_from:
        return write_traffic_profile(args.workload, *args.traffic_from)
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (the attention path has no collective "
              "inside it and no multi-GPU code is part of it); run with --gpus 1", file=sys.stderr)
        return 2

    import torch
    import paper_2307_14995_amd as ltn
    from paper_2307_14995_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the library has no CPU path", file=sys.stderr)
        return 2
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    ltn.load_library()

    if args.copy_calibration:
        src = torch.ones(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    w = synth.CONFIGS[args.workload]
    esize = 2 if w.dtype == torch.bfloat16 else 4
    block = w.block or ltn.ltn_attn_pick_block(w.D, w.dtype)
    q, k, v = synth.make_qkv(w.Bt, w.H, w.N, w.D, w.dtype, w.seed)
    d_o = synth.make_do(w.Bt, w.H, w.N, w.D, w.dtype, w.seed)
    decay = synth.decay_bench_rule(w.H)
    qd, kd, vd, gd, dd = (t.to(dev) for t in (q, k, v, d_o, decay))
    o = torch.empty_like(qd)
    grads = tuple(torch.empty_like(qd) for _ in range(3))

    def step():
        ltn.ltn_attn_fwd(qd, kd, vd, dd, block=w.block, out=o)
        ltn.ltn_attn_bwd(qd, kd, vd, gd, dd, block=w.block, out=grads)

    # Pre-roll (untimed, reported): after an idle period the GPU runs its first ~100 steps 4-8 % slower
    # (clocks ramp up).  The same step is repeated in windows of 50 until two consecutive windows agree
    # within 1 %, so that the timed figure is the sustained one whatever --warmup says.
    preroll_steps, preroll_s = 0, 0.0
    if args.preroll > 0:
        t_pre = time.perf_counter()
        prev = None
        while time.perf_counter() - t_pre < args.preroll:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(50):
                step()
            e1.record()
            torch.cuda.synchronize()
            preroll_steps += 50
            cur = e0.elapsed_time(e1)
            if prev is not None and abs(cur - prev) <= 0.01 * prev:
                break
            prev = cur
        preroll_s = time.perf_counter() - t_pre

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # Timed region: exactly K steps; HIP events on the stream the kernels run on
    # (torch's current stream is the one handed to the library).
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t_wall0 = time.perf_counter()
    for i in range(args.steps):
        ev[i][0].record()
        ltn.ltn_attn_fwd(qd, kd, vd, dd, block=w.block, out=o)
        ev[i][1].record()
        ltn.ltn_attn_bwd(qd, kd, vd, gd, dd, block=w.block, out=grads)
        ev[i][2].record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t_wall0) * 1e3
    fwd_t = sorted(e[0].elapsed_time(e[1]) for e in ev)
    bwd_t = sorted(e[1].elapsed_time(e[2]) for e in ev)
    step_t = sorted(e[0].elapsed_time(e[2]) for e in ev)
    fwd_ms = sum(fwd_t) / args.steps
    bwd_ms = sum(bwd_t) / args.steps
    ms_per_step = wall_ms / args.steps

    token_heads = w.Bt * w.H * w.N
    tokens = w.Bt * w.N
    tokens_per_s = tokens / (ms_per_step * 1e-3)
    plan_f = ltn.ltn_attn_query_plan(w.Bt, w.H, w.N, w.D, w.dtype, 0)
    plan_b = ltn.ltn_attn_query_plan(w.Bt, w.H, w.N, w.D, w.dtype, 1)
    fl = flops_per_token_head(w.D, block, plan_f, plan_b)
    ab = algorithmic_bytes_per_token_head(w.D, esize)
    tflops = {n: f * token_heads / (ms_per_step * 1e-3) / 1e12 for n, f in fl.items()}

    # Dominant kernel: the backward launch (all three gradients in one kernel).
    bwd_kernel = f"pass_bf16_kernel<{w.D},{plan_b[0]}>" if w.dtype == torch.bfloat16 else f"pass_f32_mfma_kernel<{w.D},{plan_b[0]},{block}>"
    bwd_bytes = ab["bwd"] * token_heads
    achieved = bwd_bytes / (bwd_ms * 1e-3) / 1e9
    if w.dtype == torch.float32:
        # fp32 tensors: the matrix cores' fp32 rate bounds the launch, not memory.  FLOPs the backward launch
        # issues per token-head: three passes, each with causal score tiles ((B/16+1)/2 of B/16 per 16-token
        # strip, recomputed per value-column slice), the same share of P C, and 4 D^2 of state products.
        causal = (block / 16 + 1) / 2 * 16
        bwd_flops = 3 * (2 * causal * w.D * (w.D // plan_b[0]) + 2 * causal * w.D + 4 * w.D * w.D) * token_heads
        ach_t = bwd_flops / (bwd_ms * 1e-3) / 1e12
        roofline = {
            "bound": "mfma", "kernel": bwd_kernel + " (the backward launch: dV, dK and dQ passes of every chain)",
            "achieved": round(ach_t, 1), "peak": MFMA_FP32_PEAK_TFLOPS, "unit": "TFLOP/s",
            "frac": round(ach_t / MFMA_FP32_PEAK_TFLOPS, 4), "traffic": stored_traffic(args.workload, bwd_kernel),
            "issued_flops": bwd_flops, "kernel_ms": round(bwd_ms, 4), "fwd_kernel_ms": round(fwd_ms, 4),
            "hbm_achieved_GBs": round(achieved, 1),
        }
    else:
        roofline = {
            "bound": "hbm",
            "kernel": bwd_kernel + " (the backward launch: dV, dK and dQ passes of every chain"
                      + (f", {plan_b[1]} segments per chain" if plan_b[1] > 1 else "") + ")",
            "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBS, 4),
            "traffic": stored_traffic(args.workload, bwd_kernel),
            "algorithmic_bytes": bwd_bytes,
            "kernel_ms": round(bwd_ms, 4),
            "kernel_ms_median": round(bwd_t[len(bwd_t) // 2], 4), "kernel_ms_min": round(bwd_t[0], 4),
            "fwd_kernel_ms": round(fwd_ms, 4),
            "fwd_kernel_ms_median": round(fwd_t[len(fwd_t) // 2], 4), "fwd_kernel_ms_min": round(fwd_t[0], 4),
            "fwd_achieved_GBs": round(ab["fwd"] * token_heads / (fwd_ms * 1e-3) / 1e9, 1),
        }

    out = {
        "metric": "Lightning Attention fwd+bwd tokens/s (7B-shaped layer: Bt=4, H=32, N=8192, D=128)"
                  if args.workload == "cfg3_7b" else f"Lightning Attention fwd+bwd tokens/s ({w.name})",
        "value": round(tokens_per_s, 1),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "ms_per_step_events": {"mean": round(sum(step_t) / args.steps, 4), "median": round(step_t[len(step_t) // 2], 4),
                               "min": round(step_t[0], 4)},
        "preroll_s": round(preroll_s, 2), "preroll_steps": preroll_steps,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if w.dtype == torch.bfloat16 else "f32",
        "data": "synthetic",
        "config": {"workload": w.name, "Bt": w.Bt, "H": w.H, "N": w.N, "D": w.D, "block": block,
                   "pass": "fwd+bwd", "decay": "lambda_h=exp(-2^(-8(h+1)/H))"},
        "tflops": {n: round(x, 1) for n, x in tflops.items()},
        "mfma_peak_frac": {n: round(x / MFMA_BF16_PEAK_TFLOPS, 4) for n, x in tflops.items()},
        "token_heads_per_s": round(token_heads / (ms_per_step * 1e-3), 1),
        "roofline": roofline,
    }

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, q, k, v, d_o, decay)
    if args.report:
        extended_report(ltn, synth, torch, dev, args.sections)
    print(json.dumps(out), flush=True)
    return 0


def cpu_baseline(w, q, k, v, d_o, decay):
    """The fp64 oracle (recurrent form, as it stands) timed on the host cores.  It is fast
    enough that the whole workload (every chain, full N, forward + backward) is its own
    bounded sample; for larger workloads whole chains are subsampled to about 10 s."""
    from oracle import ltn_oracle as orc
    cores = orc.num_threads()
    # ~2.6e-2 s per (chain of 8192 tokens, D=128) per core for fwd+bwd: budget about 10 s
    per_chain = 2.6e-2 * (w.N / 8192.0) * (w.D / 128.0) ** 2
    n_chains = int(max(cores, min(w.Bt * w.H, 10.0 * cores / per_chain)))
    bs = max(1, min(w.Bt, n_chains // w.H))
    hs = min(w.H, n_chains) if bs == 1 else w.H
    sl = (slice(0, bs), slice(0, hs))
    qs, ks, vs, gs, ds = q[sl], k[sl], v[sl], d_o[sl], decay[:hs]
    t0 = time.perf_counter()
    orc.fwd_recurrent(qs, ks, vs, ds)
    orc.bwd_recurrent(qs, ks, vs, gs, ds)
    dt = time.perf_counter() - t0
    token_heads = bs * hs * w.N
    # one chain on one thread, scaled to the layer: the per-core figure
    orc.set_num_threads(1)
    one = (slice(0, 1), slice(0, 1))
    t1 = time.perf_counter()
    orc.fwd_recurrent(q[one], k[one], v[one], decay[:1])
    orc.bwd_recurrent(q[one], k[one], v[one], d_o[one], decay[:1])
    dt1 = time.perf_counter() - t1
    orc.set_num_threads(cores)
    return {
        "single_thread_value": round(w.N / dt1 / w.H, 1),
        "value": round(token_heads / dt / w.H, 1),
        "unit": "tokens/s",
        "cores": cores,
        "kind": "oracle",
        "sample": f"{bs * hs} of {w.Bt * w.H} (batch,head) chains at full N={w.N}, fwd+bwd recurrent fp64, "
                  f"{dt:.1f} s; token-heads/s divided by H={w.H} gives layer tokens/s",
        "seconds": round(dt, 2),
    }


def extended_report(ltn, synth, torch, dev, sections=""):
    """Other workloads (not the bench line): printed to stderr as JSON lines."""
    chosen = {x for x in sections.split(",") if x}

    def want(name):
        return not chosen or name in chosen

    def time_call(fn, n=10, warm=3):
        """Mean ms per call over n back-to-back calls (HIP events on the launch stream)."""
        for _ in range(warm):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(n):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n

    def time_stats(fn, n=20, warm=5):
        """(median, min) ms per call, one event pair per call."""
        for _ in range(warm):
            fn()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
        for i in range(n):
            ev[i].record()
            fn()
        ev[n].record()
        torch.cuda.synchronize()
        ts = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(n))
        return ts[n // 2], ts[0]

    D = 128

    def section_machine():
        # what this machine gives: a plain 1 GiB device copy and a large bf16 GEMM (library calls, only
        # to put the published peaks of 8 TB/s and 2.5 PFLOP/s into perspective)
        src = torch.ones(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        t_copy = time_call(lambda: dst.copy_(src), n=10, warm=3)
        del src, dst
        a = torch.randn(8192, 8192, device=dev, dtype=torch.float32).to(torch.bfloat16)
        b = torch.randn(8192, 8192, device=dev, dtype=torch.float32).to(torch.bfloat16)
        t_gemm = time_call(lambda: torch.matmul(a, b), n=10, warm=3)
        del a, b
        print(json.dumps({"workload": "machine", "copy_1GiB_GBs": round(2 * (1 << 30) / (t_copy * 1e-3) / 1e9, 1),
                          "bf16_gemm_8192_TFLOPs": round(2 * 8192 ** 3 / (t_gemm * 1e-3) / 1e12, 1)}),
              file=sys.stderr, flush=True)
        # the library's own streaming-read probe: the tile pipeline's load pattern with nothing behind it
        # (64 KB in flight per compute unit), out of L2 / the memory-side cache / HBM
        buf = torch.ones(256 * (16 << 20), dtype=torch.uint8, device=dev)
        for wgs in (256, 128):
            line = {"workload": "stream_read_probe", "workgroups": wgs}
            for label, per_wg in (("L2_64KB", 64 << 10), ("cache_512KB", 512 << 10), ("HBM_16MB", 16 << 20)):
                iters = (64 << 20) // per_wg
                for regs in (0, 1):
                    t = time_call(lambda: ltn.ltn_probe_stream_read(buf, per_wg, wgs, iters, regs), n=3, warm=1)
                    line[f"{label}_{'regs' if regs else 'lds'}_TBs"] = round(wgs * per_wg * iters / (t * 1e-3) / 1e12, 2)
            print(json.dumps(line), file=sys.stderr, flush=True)
        del buf


    def section_shapes():
        shapes = [("cfg2_385m", 8, 8, 2048), ("cfg_1b", 8, 16, 2048), ("cfg3_7b", 4, 32, 8192)]
        shapes += [(f"long_N{n}", 1, 32, n) for n in synth.LONG_CONTEXT_N]
        long_times = []
        for name, Bt, H, N in shapes:
            q, k, v = (torch.randn(Bt, H, N, D, device=dev, dtype=torch.float32).div_(D ** 0.5).to(torch.bfloat16)
                       for _ in range(3))
            g = torch.randn(Bt, H, N, D, device=dev, dtype=torch.float32).to(torch.bfloat16)
            dd = synth.decay_bench_rule(H).to(dev)
            o = torch.empty_like(q)
            gr = tuple(torch.empty_like(q) for _ in range(3))
            f, fmin = time_stats(lambda: ltn.ltn_attn_fwd(q, k, v, dd, out=o))
            b, bmin = time_stats(lambda: ltn.ltn_attn_bwd(q, k, v, g, dd, out=gr))
            th = Bt * H * N
            line = {"workload": name, "Bt": Bt, "H": H, "N": N, "fwd_ms": round(f, 4), "bwd_ms": round(b, 4),
                    "fwd_min_ms": round(fmin, 4), "bwd_min_ms": round(bmin, 4),
                    "tokens_per_s": round(Bt * N / ((f + b) * 1e-3), 1),
                    "fwd_GBs": round(4 * D * 2 * th / (f * 1e-3) / 1e9, 1),
                    "bwd_GBs": round(7 * D * 2 * th / (b * 1e-3) / 1e9, 1),
                    "F_alg_TFLOPs": round((14 * D * D + 7 * 65 * D) * th / ((f + b) * 1e-3) / 1e12, 1)}
            if name == "cfg2_385m":
                # its 8 tensors (268 MB) about fit the 256 MB memory-side cache: also time it cold, rotating
                # through 8 sets of buffers so that no call finds its operands cached
                sets = [tuple(torch.randn(Bt, H, N, D, device=dev, dtype=torch.float32).to(torch.bfloat16)
                              for _ in range(8)) for _ in range(8)]
                it = [0]

                def cold_fwd():
                    x = sets[it[0] % 8]; it[0] += 1
                    ltn.ltn_attn_fwd(x[0], x[1], x[2], dd, out=x[4])

                def cold_bwd():
                    x = sets[it[0] % 8]; it[0] += 1
                    ltn.ltn_attn_bwd(x[0], x[1], x[2], x[3], dd, out=(x[5], x[6], x[7]))
                line["fwd_cold_ms"] = round(time_stats(cold_fwd, n=24, warm=8)[0], 4)
                line["bwd_cold_ms"] = round(time_stats(cold_bwd, n=24, warm=8)[0], 4)
                del sets
            print(json.dumps(line), file=sys.stderr, flush=True)
            if name.startswith("long_"):
                long_times.append((N, f + b))
            del q, k, v, g, o, gr
        # time linear in N (long context): log-log slope and doubling ratios of fwd+bwd
        import math
        xs = [math.log(n) for n, _ in long_times]
        ys = [math.log(t) for _, t in long_times]
        mx, my = sum(xs) / len(xs), sum(ys) / len(ys)
        slope = sum((x - mx) * (y - my) for x, y in zip(xs, ys)) / sum((x - mx) ** 2 for x in xs)
        big = [(n, t) for n, t in long_times if n >= 8192]
        slope_big = math.log(big[-1][1] / big[0][1]) / math.log(big[-1][0] / big[0][0])
        print(json.dumps({"workload": "long_context_linearity", "loglog_slope_all_N": round(slope, 3),
                          "loglog_slope_N_ge_8192": round(slope_big, 3),
                          "doubling_ratios": {str(b_[0]): round(b_[1] / a_[1], 3)
                                              for a_, b_ in zip(long_times, long_times[1:])}}),
              file=sys.stderr, flush=True)

    def section_fp32():
        # fp32 tensors (fp32 MFMA kernel): config 1's tiny shape and the 385M-shaped layer
        for name, Bt, H, N, Dh, blk in (("cfg1_fp32_small", 1, 2, 256, 64, 64), ("cfg2_385m_shape_fp32", 8, 8, 2048, 128, 0)):
            q, k, v = (torch.randn(Bt, H, N, Dh, device=dev).div_(Dh ** 0.5) for _ in range(3))
            g = torch.randn(Bt, H, N, Dh, device=dev)
            dd = synth.decay_bench_rule(H).to(dev)
            o = torch.empty_like(q)
            gr = tuple(torch.empty_like(q) for _ in range(3))
            f, fmin = time_stats(lambda: ltn.ltn_attn_fwd(q, k, v, dd, block=blk, out=o))
            b, bmin = time_stats(lambda: ltn.ltn_attn_bwd(q, k, v, g, dd, block=blk, out=gr))
            th = Bt * H * N
            B_ = blk or ltn.ltn_attn_pick_block(Dh, torch.float32)
            pf = ltn.ltn_attn_query_plan(Bt, H, N, Dh, torch.float32, 0)
            pb_ = ltn.ltn_attn_query_plan(Bt, H, N, Dh, torch.float32, 1)
            # FLOPs the kernel issues per token-head and pass with 16-token strips: causal score tiles
            # (B/16+1)/2 of B/16 per strip, recomputed per value-column slice; the same share of P C
            def issued(passes, dv):
                causal = (B_ / 16 + 1) / 2 * 16
                return passes * (2 * causal * Dh * (Dh // dv) + 2 * causal * Dh + 4 * Dh * Dh)
            print(json.dumps({"workload": name, "Bt": Bt, "H": H, "N": N, "D": Dh, "block": B_, "dv_fwd": pf[0], "dv_bwd": pb_[0],
                              "fwd_ms": round(f, 4), "bwd_ms": round(b, 4), "fwd_min_ms": round(fmin, 4), "bwd_min_ms": round(bmin, 4),
                              "fwd_GBs": round(4 * Dh * 4 * th / (f * 1e-3) / 1e9, 1),
                              "bwd_GBs": round(7 * Dh * 4 * th / (b * 1e-3) / 1e9, 1),
                              "fwd_issued_TFLOPs": round(issued(1, pf[0]) * th / (f * 1e-3) / 1e12, 1),
                              "bwd_issued_TFLOPs": round(issued(3, pb_[0]) * th / (b * 1e-3) / 1e12, 1),
                              "fp32_mfma_peak_TFLOPs": 157.3}), file=sys.stderr, flush=True)
            del q, k, v, g, o, gr

    def section_gated():
        # token mixer epilogue (gated SimpleRMSNorm): fused into the forward vs. forward + gate kernel
        for name, Bt, H, N in (("cfg3_7b", 4, 32, 8192), ("256chains", 8, 32, 4096)):
            q, k, v = (torch.randn(Bt, H, N, D, device=dev, dtype=torch.float32).div_(D ** 0.5).to(torch.bfloat16)
                       for _ in range(3))
            u, g = (torch.randn(Bt, H, N, D, device=dev, dtype=torch.float32).to(torch.bfloat16) for _ in range(2))
            dd = synth.decay_bench_rule(H).to(dev)
            o, y, dx, du = (torch.empty_like(q) for _ in range(4))
            th = Bt * H * N
            unit = D * 2 * th                      # bytes of one tensor
            t_plain = time_call(lambda: ltn.ltn_attn_fwd(q, k, v, dd, out=o))
            t_gate = time_call(lambda: ltn.ltn_gate_fwd(o, u, 1e-6, out=y))
            t_inf = time_call(lambda: ltn.ltn_attn_fwd_gated(q, k, v, u, dd, eps=1e-6, store_o=False, y_out=y))
            t_trn = time_call(lambda: ltn.ltn_attn_fwd_gated(q, k, v, u, dd, eps=1e-6, out=o, y_out=y))
            t_gbwd = time_call(lambda: ltn.ltn_gate_bwd(o, u, g, 1e-6, out=(dx, du)))
            print(json.dumps({"workload": "gated_" + name, "Bt": Bt, "H": H, "N": N,
                              "fwd_plain_ms": round(t_plain, 4), "gate_fwd_ms": round(t_gate, 4),
                              "unfused_ms": round(t_plain + t_gate, 4),
                              "fused_inference_ms": round(t_inf, 4), "fused_training_ms": round(t_trn, 4),
                              "gate_bwd_ms": round(t_gbwd, 4),
                              "gate_fwd_GBs": round(3 * unit / (t_gate * 1e-3) / 1e9, 1),
                              "gate_bwd_GBs": round(5 * unit / (t_gbwd * 1e-3) / 1e9, 1),
                              "fused_inference_GBs": round(5 * unit / (t_inf * 1e-3) / 1e9, 1),
                              "fused_training_GBs": round(6 * unit / (t_trn * 1e-3) / 1e9, 1)}),
                  file=sys.stderr, flush=True)
            del q, k, v, u, g, o, y, dx, du

    def section_tiled():
        # the paper's quadratic tilings (App. B Algorithms 3 and 4) against the state recurrence
        Bt, H = 4, 32
        dd = synth.decay_bench_rule(H).to(dev)
        for N in (128, 256, 512, 1024, 2048, 4096, 8192):
            q, k, v = (torch.randn(Bt, H, N, D, device=dev, dtype=torch.float32).div_(D ** 0.5).to(torch.bfloat16)
                       for _ in range(3))
            g = torch.randn(Bt, H, N, D, device=dev, dtype=torch.float32).to(torch.bfloat16)
            o = torch.empty_like(q)
            gr = tuple(torch.empty_like(q) for _ in range(3))
            few = 5 if N >= 4096 else 20
            t_rec = time_call(lambda: ltn.ltn_attn_fwd(q, k, v, dd, out=o), n=20, warm=5)
            t_til = time_call(lambda: ltn.ltn_attn_fwd_tiled(q, k, v, dd, out=o), n=few, warm=2)
            b_rec = time_call(lambda: ltn.ltn_attn_bwd(q, k, v, g, dd, out=gr), n=20, warm=5)
            b_til = time_call(lambda: ltn.ltn_attn_bwd_tiled(q, k, v, g, dd, out=gr), n=few, warm=2)
            T = N // 64
            tile_pairs = Bt * H * T * (T + 1) // 2
            print(json.dumps({"workload": "tiled_vs_recurrence", "Bt": Bt, "H": H, "N": N,
                              "recurrence_ms": round(t_rec, 4), "tiled_ms": round(t_til, 4),
                              "tiled_over_recurrence": round(t_til / t_rec, 2),
                              "tiled_TFLOPs_full_tiles": round(tile_pairs * 4 * 64 * 64 * D / (t_til * 1e-3) / 1e12, 1),
                              "bwd_recurrence_ms": round(b_rec, 4), "bwd_tiled_ms": round(b_til, 4),
                              "bwd_tiled_over_recurrence": round(b_til / b_rec, 2),
                              # Algorithm 4 without atomics: six tile products per (i, j) pair
                              "bwd_tiled_TFLOPs_full_tiles": round(tile_pairs * 12 * 64 * 64 * D / (b_til * 1e-3) / 1e12, 1)}),
                  file=sys.stderr, flush=True)
            del q, k, v, g, o, gr

    def section_lrpe():
        # first layer: swish + LRPE-d expansion of queries and keys (Eq. 1, Eq. 2), then the attention with
        # 2D-wide queries and keys; `unit` = bytes of one [Bt,H,N,D] bf16 tensor
        for name, Bt, H, N in (("cfg3_7b", 4, 32, 8192), ("cfg2_385m", 8, 8, 2048)):
            xq, xk, g = (torch.randn(Bt, H, N, D, device=dev, dtype=torch.float32).to(torch.bfloat16) for _ in range(3))
            v = torch.randn(Bt, H, N, D, device=dev, dtype=torch.float32).div_(D ** 0.5).to(torch.bfloat16)
            th_ = synth.make_theta(H, D, 1).to(dev)
            dd = synth.decay_bench_rule(H).to(dev)
            qe, ke = ltn.ltn_prologue_fwd(xq, th_), ltn.ltn_prologue_fwd(xk, th_)
            z, o = torch.empty_like(xq), torch.empty_like(v)
            unit = D * 2 * Bt * H * N
            t_sw = time_call(lambda: ltn.ltn_prologue_fwd(xq, None, out=z), n=20, warm=5)
            t_pf = time_call(lambda: ltn.ltn_prologue_fwd(xq, th_, out=qe), n=20, warm=5)
            t_f = time_call(lambda: ltn.ltn_attn_fwd_dkdv(qe, ke, v, dd, out=o), n=20, warm=5)
            t_b = time_call(lambda: ltn.ltn_attn_bwd_dkdv(qe, ke, v, g, dd), n=20, warm=5)
            dqe = torch.randn_like(qe)
            t_pb = time_call(lambda: ltn.ltn_prologue_bwd(xq, dqe, th_), n=20, warm=5)
            t_plain_f = time_call(lambda: ltn.ltn_attn_fwd(xq, xk, v, dd, out=o), n=20, warm=5)
            t_plain_b = time_call(lambda: ltn.ltn_attn_bwd(xq, xk, v, g, dd), n=20, warm=5)
            print(json.dumps({"workload": "lrpe_first_layer_" + name, "Bt": Bt, "H": H, "N": N, "D": D,
                              "swish_only_ms": round(t_sw, 4), "swish_only_GBs": round(2 * unit / (t_sw * 1e-3) / 1e9, 1),
                              "prologue_fwd_ms": round(t_pf, 4), "prologue_fwd_GBs": round(3 * unit / (t_pf * 1e-3) / 1e9, 1),
                              "prologue_bwd_ms": round(t_pb, 4), "prologue_bwd_GBs": round(4 * unit / (t_pb * 1e-3) / 1e9, 1),
                              "attn_fwd_ms": round(t_f, 4), "attn_fwd_GBs": round(6 * unit / (t_f * 1e-3) / 1e9, 1),
                              "attn_bwd_ms": round(t_b, 4), "attn_bwd_GBs_each_tensor_once": round(11 * unit / (t_b * 1e-3) / 1e9, 1),
                              "layer_fwd_ms": round(2 * t_pf + t_f, 4), "layer_bwd_ms": round(2 * t_pb + t_b, 4),
                              "plain_attn_fwd_ms": round(t_plain_f, 4), "plain_attn_bwd_ms": round(t_plain_b, 4)}),
                  file=sys.stderr, flush=True)
            del xq, xk, g, v, qe, ke, z, o, dqe

    def section_dims():
        # other head dims: 256 features at the 7B model width (16 heads x 256 = 32 x 128), and 96
        for name, Bt, H, N, Dh in (("d256_7b_width", 4, 16, 8192, 256), ("d96_32_heads", 4, 32, 8192, 96)):
            q, k, v = (torch.randn(Bt, H, N, Dh, device=dev, dtype=torch.float32).div_(Dh ** 0.5).to(torch.bfloat16)
                       for _ in range(3))
            g = torch.randn(Bt, H, N, Dh, device=dev, dtype=torch.float32).to(torch.bfloat16)
            dd = synth.decay_bench_rule(H).to(dev)
            o = torch.empty_like(q)
            gr = tuple(torch.empty_like(q) for _ in range(3))
            f, fmin = time_stats(lambda: ltn.ltn_attn_fwd(q, k, v, dd, out=o))
            b, bmin = time_stats(lambda: ltn.ltn_attn_bwd(q, k, v, g, dd, out=gr))
            unit = Dh * 2 * Bt * H * N
            print(json.dumps({"workload": name, "Bt": Bt, "H": H, "N": N, "D": Dh,
                              "fwd_ms": round(f, 4), "bwd_ms": round(b, 4), "fwd_min_ms": round(fmin, 4),
                              "bwd_min_ms": round(bmin, 4), "tokens_per_s": round(Bt * N / ((f + b) * 1e-3), 1),
                              "fwd_GBs": round(4 * unit / (f * 1e-3) / 1e9, 1),
                              "bwd_GBs": round(7 * unit / (b * 1e-3) / 1e9, 1)}), file=sys.stderr, flush=True)
            del q, k, v, g, o, gr

    def section_decode():
        c = synth.DECODE
        Bt, H = c["Bt"], c["H"]
        dd = synth.decay_bench_rule(H).to(dev)
        kv2 = torch.randn(Bt, H, 2 * D, D, device=dev)                   # decode behind the expansion: 256 x 128 states
        q2, k2 = (torch.randn(Bt, H, 1, 2 * D, device=dev).div_(D ** 0.5).to(torch.bfloat16) for _ in range(2))
        v2 = torch.randn(Bt, H, 1, D, device=dev).to(torch.bfloat16)
        o2 = torch.empty_like(v2)
        t = time_call(lambda: ltn.ltn_attn_decode_steps_dkdv(q2, k2, v2, kv2, dd, out=o2), n=256, warm=20)
        print(json.dumps({"workload": "decode_cfg5_lrpe_first_layer", "Bt": Bt, "H": H, "Dk": 2 * D, "Dv": D,
                          "us_per_step": round(t * 1e3, 2),
                          "state_GBs": round(2 * Bt * H * 2 * D * D * 4 / (t * 1e-3) / 1e9, 1)}), file=sys.stderr, flush=True)
        del kv2, q2, k2, v2, o2
        qp, kp, vp = (torch.randn(Bt, H, c["prefix"], D, device=dev).div_(D ** 0.5).to(torch.bfloat16) for _ in range(3))
        _, kv = ltn.ltn_attn_fwd(qp, kp, vp, dd, return_state=True)      # state after a 1024-token prefix
        del qp, kp, vp
        q1, k1, v1 = (torch.randn(Bt, H, D, device=dev).div_(D ** 0.5).to(torch.bfloat16) for _ in range(3))
        o1 = torch.empty_like(q1)
        t = time_call(lambda: ltn.ltn_attn_decode_step(q1, k1, v1, kv, dd, out=o1), n=512, warm=20)
        print(json.dumps({"workload": "decode_cfg5", "Bt": Bt, "H": H, "us_per_step": round(t * 1e3, 2),
                          "state_GBs": round(2 * Bt * H * D * D * 4 / (t * 1e-3) / 1e9, 1),
                          "batch_tokens_per_s": round(Bt / (t * 1e-3), 1)}), file=sys.stderr, flush=True)
        for S in (16, 64):                         # a chunk of tokens through the block forward, state handed over
            qs, ks, vs = (torch.randn(Bt, H, S, D, device=dev).div_(D ** 0.5).to(torch.bfloat16) for _ in range(3))
            os_ = torch.empty_like(qs)
            t = time_call(lambda: ltn.ltn_attn_fwd(qs, ks, vs, dd, kv_in=kv, kv_out=kv, out=os_), n=256, warm=20)
            print(json.dumps({"workload": f"chunk_cfg5_{S}_tokens_block_forward", "Bt": Bt, "H": H, "S": S,
                              "us_per_call": round(t * 1e3, 2), "us_per_token": round(t * 1e3 / S, 2),
                              "state_GBs": round(2 * Bt * H * D * D * 4 / (t * 1e-3) / 1e9, 1),
                              "batch_tokens_per_s": round(Bt * S / (t * 1e-3), 1)}), file=sys.stderr, flush=True)
        for S in (4, 16):                          # several tokens per call: the state moves once per call
            qs, ks, vs = (torch.randn(Bt, H, S, D, device=dev).to(torch.bfloat16) for _ in range(3))
            os_ = torch.empty_like(qs)
            t = time_call(lambda: ltn.ltn_attn_decode_steps(qs, ks, vs, kv, dd, out=os_), n=256, warm=20)
            print(json.dumps({"workload": f"decode_cfg5_{S}_tokens_per_call", "Bt": Bt, "H": H, "S": S,
                              "us_per_call": round(t * 1e3, 2), "us_per_token": round(t * 1e3 / S, 2),
                              "state_GBs": round(2 * Bt * H * D * D * 4 / (t * 1e-3) / 1e9, 1),
                              "batch_tokens_per_s": round(Bt * S / (t * 1e-3), 1)}), file=sys.stderr, flush=True)

    for name, fn in (("machine", section_machine), ("shapes", section_shapes), ("fp32", section_fp32), ("gated", section_gated),
                     ("tiled", section_tiled), ("lrpe", section_lrpe), ("dims", section_dims),
                     ("decode", section_decode)):
        if want(name):
            fn()




if __name__ == "__main__":
    sys.exit(main())
