#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X.

A step = one pass of the whole hot path at the shape of the Wan-1.3B-class layer
(12 heads x 128, block of 4680 tokens, 28080 cached tokens, key length 32760):
  ifx_block_attention (one launch of the fused attention kernel)  then
  ifx_kv_cache_commit (the block's K/V go into the 6-block ring, evicting the
  oldest block, so every step sees the same shape).
Consecutive steps go round the layers of a 30-layer cache, so no step finds its
keys in a cache left warm by the step before.  Inputs are synthetic, seeded,
already resident in HBM.  The reported value is attention FLOPs
(4 * n * Lk * D * H) divided by the time of the whole step.
The K timed steps run without instrumentation; the same K steps are then run
again with the library's HIP events around everything each attention call and
each commit enqueues, which gives the times of the roofline object.  Further
legs: the same attention with queries that fail the norm bound (running-maximum
softmax), 30 attention calls in a row (one denoising step of 30 layers), and
one ifx_kv_cache_commit_layers call for 30 layers.

Prints ONE JSON line.  Only the cpu_baseline leg touches the CPU oracle.
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

PEAK_BF16_TFLOPS = 2500.0  # MI355X dense bf16 MFMA, published
PEAK_HBM_GBS = 8000.0


def measured_traffic(workload):
    """HBM bytes per attention launch: not measured in this run but read from the committed rocprofv3
    counter summary of the same workload (FETCH_SIZE and WRITE_SIZE, each calibrated against a
    plain copy kernel); None if there is no summary."""
    path = os.path.join(ROOT, "profiles", f"attn_bf16_kernel_{workload}_pmc.txt")
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("traffic_bytes_per_launch:"):
                    return float(line.split(":", 1)[1])
    except OSError:
        pass
    return None

WORKLOADS = {
    # name: (layers the steps go round, heads, head_dim, block_tokens, cached_blocks)
    "wan1.3b_layer_32k": (30, 12, 128, 4680, 6),
    "wan14b_720p_layer_54k": (1, 40, 128, 10800, 4),
    # not the headline: the same layer attending to the oldest resident block plus the newest three
    # of a ring of 7 (ifx_block_attention_ranges, five table entries), key length 23400
    "wan1.3b_layer_sink1_window3": (30, 12, 128, 4680, 7),
}
KEY_RANGES = {"wan1.3b_layer_sink1_window3": [(0, 1), (4, 3)]}
WORKLOADS["wan1.3b_layer_37k"] = (30, 12, 128, 4680, 7)  # steady state of the 7-block ring: key length 37440
# the generate-and-cache loop: 30 layers, 7 blocks x 4 denoising steps, commit after each block's last step
# the fp32 correctness configuration (2 heads x 64, blocks of 256, key length 1024): a latency figure, not a throughput one
WORKLOADS["fp32_2x64_1k"] = (1, 2, 64, 256, 3)
F32_WORKLOADS = {"fp32_2x64_1k"}
PEAK_F32_VECTOR_TFLOPS = 157.3  # MI355X fp32 vector, published
EXP2_PEAK_PER_S = 256 * 4 * 8 * 2.4e9  # transcendental issue: half the VALU rate (16 lanes per cycle and SIMD)
LOOP_WORKLOADS = {"wan1.3b_generate_7x4x30": (30, 12, 128, 4680, 7, 7, 4)}


def power_and_clock_under_load(enqueue_calls, sync):
    """Socket power and shader clocks as `amd-smi` reports them while the attention call runs back
    to back (the launch is power-limited: this is the context of every time on the line).  The tool
    runs as a child process; `enqueue_calls(k)` keeps the GPU busy in batches until it has answered,
    10 s at most.  None if the tool is missing or says nothing usable."""
    import re
    import shutil
    import subprocess

    exe = shutil.which("amd-smi") or "/opt/rocm/bin/amd-smi"
    if not os.path.exists(exe):
        return None
    # two batches always in flight: the next one is enqueued before the host waits for the one before
    import torch
    pending = []

    def keep_busy():
        enqueue_calls(40)
        ev = torch.cuda.Event()
        ev.record()
        pending.append(ev)
        if len(pending) > 2:
            pending.pop(0).synchronize()

    t_warm = time.perf_counter() + 1.5  # the reported power is an average over about a second
    while time.perf_counter() < t_warm:
        keep_busy()
    try:
        child = subprocess.Popen([exe, "metric", "-g", "0", "--power", "--clock"], stdout=subprocess.PIPE,
                                 stderr=subprocess.DEVNULL, text=True)
    except OSError:
        sync()
        return None
    t_end = time.perf_counter() + 10.0
    while child.poll() is None and time.perf_counter() < t_end:
        keep_busy()
    sync()
    if child.poll() is None:
        child.kill()
        child.wait()
        return None
    text = child.stdout.read()
    power = re.search(r"SOCKET_POWER:\s*(\d+(?:\.\d+)?)\s*W", text)
    clocks = [int(c) for c in re.findall(r"GFX_\d+:\s*\n\s*CLK:\s*(\d+)\s*MHz", text)]
    top = re.search(r"GFX_0:\s*\n\s*CLK:.*\n\s*MIN_CLK:.*\n\s*MAX_CLK:\s*(\d+)\s*MHz", text)
    if not clocks:
        return None
    cap = None
    smi = shutil.which("rocm-smi") or "/opt/rocm/bin/rocm-smi"
    if os.path.exists(smi):
        try:
            out = subprocess.run([smi, "--showmaxpower"], capture_output=True, text=True, timeout=10).stdout
            m = re.search(r"Max Graphics Package Power \(W\):\s*(\d+(?:\.\d+)?)", out)
            cap = float(m.group(1)) if m else None
        except (OSError, subprocess.TimeoutExpired):
            pass
    return {
        "socket_power_w": float(power.group(1)) if power else None,
        "power_cap_w": cap,
        "gfx_clock_mhz": clocks,
        "gfx_clock_mhz_mean": sum(clocks) / len(clocks),
        "gfx_clock_mhz_max": int(top.group(1)) if top else None,
        "source": "amd-smi metric -g 0 --power --clock, one reading while ifx_block_attention ran back to back; the cap from rocm-smi --showmaxpower",
    }


def run_generate_loop(args):
    """7 blocks x 4 steps x 30 layers: per-step and per-block times (HIP events on the caller's stream)."""
    import torch
    from paper_2511_20714_amd import binding as ifx
    from paper_2511_20714_amd import synth

    dev = torch.device("cuda:0")
    L, H, D, n, cap, blocks, steps = LOOP_WORKLOADS[args.workload]
    cache = ifx.KVCache(L, H, D, cap * n, n, ifx.IFX_BF16)
    sets = [synth.draw_qkv(args.seed, i, 0, 0, n, H, D, torch.bfloat16, dev, rms_norm=True) for i in range(4)]
    out = torch.empty((n, H, D), dtype=torch.bfloat16, device=dev)
    stream = torch.cuda.current_stream().cuda_stream
    side = torch.cuda.Stream()  # capture needs a stream of its own (default priority)
    ev = lambda: torch.cuda.Event(enable_timing=True)

    # --graph: the 4 x 30 attention calls of a block only enqueue kernels and the cache does not
    # change while a block is denoised, so they are recorded once per block position into a HIP
    # graph (in the untimed run) and replayed; the commits depend on host metadata and stay eager
    graphs = {}

    def denoise_block(b, marks):
        for s in range(steps):
            q, k, v = sets[(b + s) % 4]
            cur = torch.cuda.current_stream().cuda_stream
            for l in range(L):
                cache.attention(l, q, k, v, out, cur)
            if marks is not None:
                marks[s + 1].record()

    def one_run(record):
        cache.reset()
        per_block = []
        for b in range(blocks):
            marks = [ev() for _ in range(steps + 2)]
            if args.graph and b not in graphs:
                torch.cuda.synchronize()
                graphs[b] = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graphs[b], stream=side):
                    denoise_block(b, None)
            marks[0].record()
            if args.graph:
                graphs[b].replay()
                marks[steps].record()
            else:
                denoise_block(b, marks)
            k, v = sets[(b + steps - 1) % 4][1:]
            if args.commit == "layers":
                cache.commit_layers(0, [k] * L, [v] * L, stream)
            else:
                for l in range(L):
                    cache.commit(l, k, v, stream)
            marks[steps + 1].record()
            per_block.append(marks)
        torch.cuda.synchronize()
        if not record:
            return None
        rows = []
        for b, marks in enumerate(per_block):
            if args.graph:
                step_ms = [marks[0].elapsed_time(marks[steps]) / steps] * steps
            else:
                step_ms = [marks[i].elapsed_time(marks[i + 1]) for i in range(steps)]
            commit_ms = marks[steps].elapsed_time(marks[steps + 1])
            Lk = (b + 1) * n
            rows.append({"block": b + 1, "key_len": Lk, "ms_per_denoise_step": sum(step_ms) / steps,
                         "ms_per_block": sum(step_ms) + commit_ms, "ms_30_commits": commit_ms,
                         "attention_tflops": 4.0 * n * Lk * D * H * L / (sum(step_ms) / steps * 1e-3) / 1e12,
                         "commit_gbs": L * 2 * (2 * n * H * D * 2) / (commit_ms * 1e-3) / 1e9})
        return rows

    one_run(False)
    t0 = time.perf_counter()
    rows = one_run(True)
    t1 = time.perf_counter()
    total_flops = sum(4.0 * n * r["key_len"] * D * H * L * steps for r in rows)
    total_ms = sum(r["ms_per_block"] for r in rows)
    cache.close()
    print(json.dumps({
        "metric": "block-causal attention TFLOP/s (whole generate-and-cache loop: attention + cache commits)",
        "value": total_flops / (total_ms * 1e-3) / 1e12, "unit": "TFLOP/s", "n_gpus": 1, "steps": 1, "warmup": 1,
        "ms_per_step": total_ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"{args.workload}: {L} layers, {H} heads x {D}, {blocks} blocks of {n} tokens x {steps} "
                               f"denoising steps, ring of {cap} blocks; a step here = the whole loop; commit ({args.commit})"
                               f"{'; attention calls of each block replayed from a HIP graph' if args.graph else ''}",
                   "wall_ms_including_host": (t1 - t0) * 1e3},
        "per_block": rows, "roofline": None, "cpu_baseline": None}))



def cpu_baseline(q, k, v, cached, n, H, D, rows_wanted=16384, through_e4m3=False):
    """The fp64 oracle timed on a bounded sample of (row, head) pairs with the full key length."""
    import numpy as np
    import oracle
    import torch
    from paper_2511_20714_amd import synth

    rng = np.random.default_rng(0)
    rows = rng.integers(0, n, rows_wanted).astype(np.int64)
    heads = rng.integers(0, H, rows_wanted).astype(np.int64)

    def cached_f64(t):  # what the cache holds of a committed block
        if not through_e4m3:
            return synth.to_f64_numpy(t)
        bits = t.detach().to("cpu").contiguous().view(torch.int16).numpy().view(np.uint16)
        return oracle.bf16_bits_to_f64(oracle.bf16_bits_through_e4m3(bits))

    kc = np.concatenate([cached_f64(kk) for kk, _ in cached])
    vc = np.concatenate([cached_f64(vv) for _, vv in cached])
    qn, kn, vn = synth.to_f64_numpy(q), synth.to_f64_numpy(k), synth.to_f64_numpy(v)
    t0 = time.perf_counter()
    out, _ = oracle.attention_rows(qn, kc, vc, kn, vn, rows, heads)
    dt = time.perf_counter() - t0
    Lk = kc.shape[0] + n
    flops = 4.0 * rows_wanted * Lk * D
    return {
        "value": flops / dt / 1e12,
        "unit": "TFLOP/s",
        "cores": oracle.threads(),
        "kind": "oracle",
        "sample": f"{rows_wanted} random (query row, head) pairs of the same workload with the full key length {Lk}, "
                  f"{dt:.2f} s of fp64 three-pass softmax attention; rows are independent, so the rate carries over",
        "seconds": dt,
    }, (rows, heads, out)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--workload", default="wan1.3b_layer_32k", choices=sorted(WORKLOADS) + sorted(LOOP_WORKLOADS))
    ap.add_argument("--commit", default="copy", choices=["copy", "layers"],
                    help="copy: one ifx_kv_cache_commit per layer; layers (loop workload): one "
                         "ifx_kv_cache_commit_layers call for the 30 layers of a block")
    ap.add_argument("--graph", action="store_true",
                    help="loop workload only: replay each block's attention calls from a HIP graph recorded in the untimed run")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra-legs", action="store_true",
                    help="only the timed steps and their instrumented repeat (for profiler runs: every attention launch "
                         "is then a headline launch)")
    ap.add_argument("--cache-dtype", default="bf16", choices=["bf16", "fp8"],
                    help="fp8: the cache keeps committed blocks as E4M3 codes (IFX_FP8_E4M3); the tensors stay bf16")
    ap.add_argument("--reserve", action="store_true",
                    help="create the cache with ifx_kv_cache_reserve (twice the capacity): memory mapped piecewise into a "
                         "reserved address range instead of one allocation")
    ap.add_argument("--running-max", action="store_true",
                    help="run the timed steps themselves with queries x 4, i.e. on the running-maximum softmax "
                         "(for profiler runs of that variant)")
    ap.add_argument("--seed", type=int, default=2)
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on exactly one GPU (one process, no collectives); use --gpus 1")

    import torch
    from paper_2511_20714_amd import binding as ifx
    from paper_2511_20714_amd import synth

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the HIP path has no CPU fallback")
    if args.graph and args.workload not in LOOP_WORKLOADS:
        sys.exit("bench.py: --graph applies to the loop workload only")
    if args.workload in LOOP_WORKLOADS:
        return run_generate_loop(args)
    dev = torch.device("cuda:0")
    L, H, D, n, cap = WORKLOADS[args.workload]
    ranges = KEY_RANGES.get(args.workload)
    f32 = args.workload in F32_WORKLOADS
    tdtype, idtype = (torch.float32, ifx.IFX_F32) if f32 else (torch.bfloat16, ifx.IFX_BF16)
    fp8 = args.cache_dtype == "fp8" and not f32
    if fp8:
        idtype = ifx.IFX_FP8_E4M3
    peak = PEAK_F32_VECTOR_TFLOPS if f32 else PEAK_BF16_TFLOPS
    C = (cap if ranges is None else sum(c for _, c in ranges)) * n
    Lk = C + n
    cache = ifx.KVCache(L, H, D, cap * n, n, idtype, reserve_tokens=2 * cap * n if args.reserve else None)
    cached = []
    for b in range(cap):
        _, k, v = synth.draw_qkv(args.seed, b, 0, 0, n, H, D, tdtype, dev, rms_norm=not f32)
        for l in range(L):
            cache.commit(l, k, v)
        cached.append((k, v))
    # a few distinct input sets so consecutive steps do not reuse one buffer
    sets = [synth.draw_qkv(args.seed, cap + i, 0, 0, n, H, D, tdtype, dev, rms_norm=not f32) for i in range(4)]
    outs = [torch.empty((n, H, D), dtype=tdtype, device=dev) for _ in range(4)]
    stream = torch.cuda.current_stream().cuda_stream

    if args.running_max and not f32:
        sets = [((s[0].float() * 4.0).to(tdtype), s[1], s[2]) for s in sets]

    def attend(i, q=None):
        qq, k, v = sets[i % 4]
        if ranges is None:
            cache.attention(i % L, qq if q is None else q, k, v, outs[i % 4], stream)
        else:
            cache.attention_ranges(i % L, qq if q is None else q, k, v, ranges, outs[i % 4], None, stream)

    def step(i):
        attend(i)
        cache.commit(i % L, sets[i % 4][1], sets[i % 4][2], stream)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.warmup, args.warmup + args.steps):
        step(i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    # The same K steps once more with the library's HIP events around what every attention call and
    # every commit enqueues (on the caller's stream): the times of the roofline.  Kept out of the
    # timed pass above because the four event records per step cost about 15 us of a 0.8 ms step.
    cache.profile(True)
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    for i in range(args.warmup + args.steps, args.warmup + 2 * args.steps):
        step(i)
    torch.cuda.synchronize()
    t3 = time.perf_counter()
    attn_ms, attn_launches, commit_ms, commit_launches = cache.profile_read()
    last_step = args.warmup + 2 * args.steps - 1
    got_last = outs[last_step % 4].to("cpu")  # checked against the oracle at the end

    # The running-maximum softmax: the same calls with queries four times as long, which puts the
    # Cauchy-Schwarz bound on the scores (65 in log2 units) over the limit of the fixed-maximum
    # variant, so every wavefront takes the online softmax with its running maximum.
    rm = None
    if not f32 and not args.no_extra_legs:
        q_long = [(s[0].float() * 4.0).to(tdtype) for s in sets]
        for i in range(10):
            attend(i, q_long[i % 4])
        torch.cuda.synchronize()
        cache.profile_read()
        for i in range(args.steps):
            attend(i, q_long[i % 4])
        torch.cuda.synchronize()
        rm_ms, rm_launches, _, _ = cache.profile_read()
        rm = rm_ms / max(rm_launches, 1)
    cache.profile(False)

    # One denoising step of a 30-layer model: 30 attention calls in a row, no commits.
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    denoise_step_ms = None
    if not args.no_extra_legs:
        reps = max(1, min(10, args.steps // 30))
        for i in range(30):
            attend(i)
        e0.record()
        for i in range(30 * reps):
            attend(i)
        e1.record()
        torch.cuda.synchronize()
        denoise_step_ms = e0.elapsed_time(e1) / reps

    # One ifx_kv_cache_commit_layers call for the blocks of 30 layers (the end of a block's last step).
    commit30_ms = None
    if L >= 30 and not args.no_extra_legs:
        ks = [sets[l % 4][1] for l in range(30)]
        vs = [sets[l % 4][2] for l in range(30)]
        for _ in range(3):
            cache.commit_layers(0, ks, vs, stream)
        e0.record()
        for _ in range(20):
            cache.commit_layers(0, ks, vs, stream)
        e1.record()
        torch.cuda.synchronize()
        commit30_ms = e0.elapsed_time(e1) / 20
        # (the ring of every layer has advanced by 23 blocks of the same four input sets; the oracle
        # leg below uses the output of the last instrumented step, taken before this)

    # a device-to-device copy of the same bytes, for the commit's bandwidth figure; over enough
    # different buffers (about 0.5 GB) that the 256 MB memory-side cache cannot hold them, as the
    # commits' own sources and slots do not fit it either
    pairs = max(2, int(0.5e9 // (4 * n * H * D * (4 if f32 else 2))) + 1)
    srcs = [torch.empty(2 * n * H * D, dtype=tdtype, device=dev) for _ in range(pairs)]
    dsts = [torch.empty_like(srcs[0]) for _ in range(pairs)]
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for i in range(pairs):
        dsts[i].copy_(srcs[i])
    e0.record()
    for i in range(4 * pairs):
        dsts[i % pairs].copy_(srcs[i % pairs])
    e1.record()
    torch.cuda.synchronize()
    copy_ms = e0.elapsed_time(e1) / (4 * pairs)
    del srcs, dsts

    # What the chip does meanwhile: power and clocks while the headline call runs back to back.
    power_clock = None
    if not f32 and not args.no_extra_legs:
        power_clock = power_and_clock_under_load(lambda k: [attend(i) for i in range(k)], torch.cuda.synchronize)

    # The running-maximum variant once more, on the headline's own score distribution: layer 0 gets
    # a block in which one key per head is four times as long (one key in 32 760), which alone puts
    # every wavefront's bound over the limit; queries as in the timed steps.  What this leg costs
    # over the headline is the variant's bookkeeping; what the leg above costs over this one is the
    # rescaling that its sharper softmax rows (queries x 4) really ask for.  Last: it changes layer 0.
    rm_same = None
    if rm is not None and ranges is None:
        k_long = sets[0][1].clone()
        k_long[0] *= 4.0
        cache.commit(0, k_long, sets[0][2], stream)
        cache.profile(True)
        for i in range(10):
            cache.attention(0, *sets[i % 4], outs[i % 4], stream)
        torch.cuda.synchronize()
        cache.profile_read()
        for i in range(args.steps):
            cache.attention(0, *sets[i % 4], outs[i % 4], stream)
        torch.cuda.synchronize()
        same_ms, same_launches, _, _ = cache.profile_read()
        rm_same = same_ms / max(same_launches, 1)
        cache.profile(False)

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    flops = 4.0 * n * Lk * D * H
    tflops = flops / (ms_per_step * 1e-3) / 1e12
    kern_ms = attn_ms / max(attn_launches, 1)
    kern_tflops = flops / (kern_ms * 1e-3) / 1e12
    esize = 4 if f32 else 2
    commit_bytes = 2 * n * H * D * esize + 2 * n * H * D * (1 if fp8 else esize)  # K and V, read + write
    commit_kern_ms = commit_ms / max(commit_launches, 1)

    result = {
        "metric": "block-causal attention TFLOP/s (whole step: attention + cache commit)",
        "value": tflops,
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32" if f32 else "bf16",
        "data": "synthetic",
        "config": {
            "workload": f"{args.workload}: 1 layer per step (steps go round {L} layers' caches), {H} heads x {D}, block {n} tokens, {C} cached tokens "
                        f"(ring of {cap} blocks{'' if ranges is None else ', resident block ranges ' + str(ranges)}), "
                        f"key length {Lk}; step = attention + commit ({args.commit})"
                        f"{'; cache memory mapped piecewise into a reserved address range' if args.reserve else ''}"
                        f"{'; cache kept as fp8 (E4M3) codes' if fp8 else ''}",
            "heads": H, "head_dim": D, "block_tokens": n, "cached_tokens": C, "key_len": Lk,
        },
        ("pct_fp32_vector_peak" if f32 else "pct_bf16_mfma_peak"): 100.0 * tflops / peak,
        "attention_call_ms": kern_ms,
        "ms_per_denoise_step_30_layers": denoise_step_ms,
        "ms_per_step_with_kernel_events": (t3 - t2) * 1e3 / args.steps,
        "timing": "value and ms_per_step: K steps between two synchronisations, no instrumentation; attention_call_ms, roofline "
                  "and commit: a second pass over the same K steps with HIP events around everything each "
                  "ifx_block_attention call (one kernel launch) and each commit enqueues; ms_per_denoise_step_30_layers: "
                  "30 attention calls in a row between two events, measured",
        "roofline": {
            "bound": "alu" if f32 else "mfma",
            "kernel": "attn_f32_kernel" if f32 else "attn_bf16_kernel",
            "achieved": kern_tflops,
            "peak": peak,
            "unit": "TFLOP/s",
            "frac": kern_tflops / peak,
            "traffic": measured_traffic(args.workload),
            "traffic_unit": "bytes per launch (HBM read + write); from the committed rocprofv3 counter summary of this "
                            "workload under profiles/, not measured in this run",
            "algorithmic_bytes_per_launch": 2.0 * n * H * D * esize + 2.0 * n * H * D * esize + 2.0 * C * H * D * (1 if fp8 else esize),
            "avg_kernel_ms": kern_ms,
            "launches": attn_launches,
            "flops_per_launch": flops,
            # second ceiling of the same launch: one exp2 per (query, key, head); a 64-wide v_exp_f32 holds
            # a SIMD's VALU port for 8 cycles: 256 CUs x 4 SIMDs x 8 lanes per cycle x 2.4 GHz
            "exp2": {"per_launch": float(n) * Lk * H, "achieved_per_s": float(n) * Lk * H / (kern_ms * 1e-3),
                     "peak_per_s": EXP2_PEAK_PER_S, "frac": float(n) * Lk * H / (kern_ms * 1e-3) / EXP2_PEAK_PER_S},
        },
        "commit": {
            "bound": "hbm",
            "avg_ms": commit_kern_ms,
            "achieved": commit_bytes / (commit_kern_ms * 1e-3) / 1e9 if commit_kern_ms > 0 else None,
            "peak": PEAK_HBM_GBS,
            "unit": "GB/s",
            "bytes_per_call": commit_bytes,
            "device_copy_of_the_same_bytes_gbs": commit_bytes / (copy_ms * 1e-3) / 1e9,
        },
    }
    if rm is not None:
        result["roofline_running_max"] = {
            "bound": "mfma", "kernel": "attn_bf16_kernel, every wavefront on the running-maximum softmax (queries x 4)",
            "achieved": flops / (rm * 1e-3) / 1e12, "peak": peak, "unit": "TFLOP/s", "frac": flops / (rm * 1e-3) / 1e12 / peak,
            "avg_kernel_ms": rm, "launches": rm_launches,
        }
        if rm_same is not None:
            result["roofline_running_max"]["on_the_headline_scores"] = {
                "inputs": "the timed steps' queries; one cached key per head x 4 puts every wavefront on the running maximum",
                "achieved": flops / (rm_same * 1e-3) / 1e12, "frac": flops / (rm_same * 1e-3) / 1e12 / peak,
                "avg_kernel_ms": rm_same, "launches": same_launches,
            }
    if power_clock is not None:
        result["power_clock_under_load"] = power_clock
    if commit30_ms is not None:
        result["commit_layers_30"] = {
            "bound": "hbm", "avg_ms": commit30_ms, "achieved": 30 * commit_bytes / (commit30_ms * 1e-3) / 1e9,
            "peak": PEAK_HBM_GBS, "unit": "GB/s", "bytes_per_call": 30 * commit_bytes,
            "frac": 30 * commit_bytes / (commit30_ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
            "device_copy_of_the_same_bytes_gbs": commit_bytes / (copy_ms * 1e-3) / 1e9,
        }

    if not args.no_cpu_baseline:
        q, k, v = sets[last_step % 4]
        # what layer last_step % L held when that step's attention ran: the pre-filled blocks, then
        # the block of every earlier step on that layer; the ring keeps the last `cap` of them
        layer = last_step % L
        history = cached + [(sets[i % 4][1], sets[i % 4][2]) for i in range(last_step) if i % L == layer]
        before_last = history[-cap:]
        if ranges is not None:
            before_last = [blk for first, count in ranges for blk in before_last[first:first + count]]
        base, (rows, heads, want) = cpu_baseline(q, k, v, before_last, n, H, D, through_e4m3=fp8)
        got = got_last.to(torch.float64).numpy()[rows, heads]
        err = abs(got - want)
        base["gpu_vs_oracle_max_abs_err"] = float(err.max())
        base["gpu_vs_oracle_mean_abs_err"] = float(err.mean())
        result["cpu_baseline"] = base
    else:
        result["cpu_baseline"] = None

    cache.close()
    print(json.dumps(result))


if __name__ == "__main__":
    main()
