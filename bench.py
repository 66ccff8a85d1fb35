#!/usr/bin/env python3
"""Benchmark of the streaming denoiser hot path on one MI355X.

A "step" is one sdv2_denoise_step call: timestep conditioning plus every block of the model on one
chunk of synthetic input, with all inputs, weights and caches already resident in HBM.  The default
workload is the 1.3B-shaped model (30 blocks) at steady state (sink full, window full, so every
step evicts), one denoising step per chunk.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-cpu-baseline] [--no-also]

Besides the headline workload the line carries, under "also", the per-chunk latency of the 14B-shaped
model (40 blocks) measured the same way on a few steps, so that both model sizes are on record.

Timing: W warm-up steps, then K steps between two torch.cuda.synchronize() calls and a pair of
events on the stream the library launches on (value = the slower of wall clock and events is not
taken: value is the event time; the wall time is reported beside it).  A second pass over K more
steps runs with the library's per-launch event timing switched on and yields the per-kernel
durations used for the roofline object.  The oracle is then timed on the host cores on one step.
"""

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=6)
    ap.add_argument("--workload", default="wan1.3b-step")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-also", action="store_true", help="skip the secondary 14B-shaped measurement")
    ap.add_argument("--dist-chunks", type=int, default=60,
                    help="steady-state chunks in the latency-distribution pass (skipped with --no-also)")
    ap.add_argument("--batch-sweep", default="",
                    help="comma-separated batch sizes (1..8): instead of the usual line, measure the step latency "
                         "L(T, B) of the workload with B streams per call and print the table with the batch size "
                         "the SLO-aware scheduler picks for a few target frame rates")
    ap.add_argument("--cpu-layers", type=int, default=0, help="blocks the oracle times (0: all, bounded to ~30 s)")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MiB",
                    help="also run a plain device copy of this many MiB (read + write) three times before the timed "
                         "region, as the known-size reference for rocprofv3 FETCH_SIZE / WRITE_SIZE counters")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); --gpus %d is not supported"
              % args.gpus, file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2511_07399_amd import binding, cost_model as cm, workloads as wk

    from paper_2511_07399_amd.runner import DeviceModel

    binding.load_library()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    wl = wk.WORKLOADS[args.workload]
    if args.batch_sweep:
        print(json.dumps(batch_sweep(args.workload, [int(b) for b in args.batch_sweep.split(",")], args.steps, args.warmup)))
        return
    m = measure(args.workload, args.steps, args.warmup, args.copy_calibration, 0 if args.no_also else args.dist_chunks)
    ms_per_step, wall_ms, kernels, roofline = m["ms_per_step"], m["wall_ms"], m["kernels"], m["roofline"]
    step_flops, gemm_tflops, attn_tflops, l_kv = m["step_flops"], m["gemm_tflops"], m["attn_tflops"], m["l_kv"]
    B, L, Cw = wl.B, wl.L, wl.C
    peaks = measure_peaks()
    add_measured_fractions(roofline, peaks)
    also = None
    if not args.no_also:
        also = {}
        for name, k_steps, k_warm in (("wan14b-step", 8, 2), ("wan14b-480p-b4", 2, 1)):
            if name == args.workload:
                continue
            m2 = measure(name, k_steps, k_warm, 0)
            w2 = wk.WORKLOADS[name]
            add_measured_fractions(m2["roofline"], peaks)
            frac = m2["step_flops"] / (m2["ms_per_step"] * 1e-3) / cm.MI355X_BF16_FLOPS
            also[name] = {
                "workload": "%d blocks, C %d, %d heads x 128, FFN %d, %d stream(s) x %d query tokens per chunk, L_kv %d, "
                            "%d text tokens, 1 denoising step per chunk" % (w2.N, w2.C, w2.H, w2.F, w2.B, w2.L, m2["l_kv"], w2.L_t),
                "value": round(m2["ms_per_step"], 4), "unit": "ms", "steps": k_steps, "warmup": k_warm,
                "wall_ms_per_step": round(m2["wall_ms"], 4),
                "step_tflops": round(m2["step_flops"] / (m2["ms_per_step"] * 1e-3) / 1e12, 1),
                "step_frac_mfma_peak": round(frac, 4),
                "step_frac_measured_mfma_peak": round(frac * cm.MI355X_BF16_FLOPS / (peaks["mfma_bf16"]["measured"] * 1e12), 4),
                "gemm_tflops": round(m2["gemm_tflops"], 1), "attn_tflops": round(m2["attn_tflops"], 1),
                "roofline": m2["roofline"], "kernels": m2["kernels"]}
        also["graph_replay"] = measure_graph_replay(args.workload, args.steps, args.warmup)
        also["stream_batch"] = measure_stream_batch(args.workload) if args.workload == "wan1.3b-step" else None
        also["latents"] = measure_latents(args.workload) if args.workload == "wan1.3b-step" else None
        also["refresh"] = measure_refresh(args.workload)
        also["motion"] = measure_motion()

    # ---- oracle on the host cores (a reported baseline, not the target)
    cpu_baseline = None
    if not args.no_cpu_baseline:
        cpu_baseline = time_oracle(wl, args.cpu_layers)

    out = {
        "metric": "per-chunk denoise-step latency", "value": round(ms_per_step, 4), "unit": "ms",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {
            "workload": "%s: %d blocks, C %d, %d heads x 128, FFN %d, %d stream(s) x %d query tokens per chunk, "
                        "sink %d + window %d tokens (steady state, L_kv %d), %d text tokens, 1 denoising step per "
                        "chunk, fp32 residual stream" % (wl.name, wl.N, Cw, wl.H, wl.F, B, L, wl.S, wl.W, l_kv, wl.L_t),
            "global_batch": B, "seq_len": L,
        },
        "wall_ms_per_step": round(wall_ms, 4),
        "step_tflops": round(step_flops / (ms_per_step * 1e-3) / 1e12, 1),
        "step_frac_mfma_peak": round(step_flops / (ms_per_step * 1e-3) / cm.MI355X_BF16_FLOPS, 4),
        "gemm_tflops": round(gemm_tflops, 1), "attn_tflops": round(attn_tflops, 1),
        "step_frac_measured_mfma_peak": round(step_flops / (ms_per_step * 1e-3) / (peaks["mfma_bf16"]["measured"] * 1e12), 4),
        "roofline": roofline, "peaks": peaks, "cpu_baseline": cpu_baseline, "kernels": kernels, "latency": m["latency"],
        "also": also,
    }
    print(json.dumps(out))


def measure_peaks():
    """What the chip sustains, beside the published peaks: a register-resident loop of bf16 matrix instructions on
    every compute unit (no memory traffic) and a streaming copy of 1 GiB (read + write), each the best of five
    launches between events on the launch stream."""
    import torch
    from paper_2511_07399_amd import binding, cost_model as cm
    dev = "cuda:0"
    stream = torch.cuda.current_stream()
    wgs, iters = 256 * 4, 4096
    sink = torch.empty(wgs * 512, dtype=torch.float32, device=dev)
    src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
    dst = torch.empty_like(src)

    def best(fn, reps=5):
        fn()
        out = []
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            work = fn()
            e1.record(stream)
            torch.cuda.synchronize()
            out.append(work / (e0.elapsed_time(e1) * 1e-3))
        return max(out)

    mfma = best(lambda: binding.prof_peak_mfma(iters, wgs, sink))
    copy = best(lambda: 2 * binding.prof_peak_copy(src, dst))
    assert torch.equal(src[:4096], dst[:4096]) and torch.equal(src[-4096:], dst[-4096:])
    del src, dst, sink
    # the LDS pipeline of one compute unit: shader clocks per wave instruction that moves 1 KB
    lds_iters = 2000
    scratch = torch.zeros(40960 // 8, dtype=torch.int64, device=dev)
    binding.prof_lds_rates(lds_iters, scratch)
    binding.prof_lds_rates(lds_iters, scratch)
    torch.cuda.synchronize()
    ticks = [int(t) for t in scratch[:3].cpu()]
    lds = {n: round(t / (lds_iters * 8 * 8.0), 2) for n, t in zip(("ds_read_b128", "ds_write_b128", "direct global->LDS load x4"), ticks)}
    del scratch
    torch.cuda.empty_cache()
    return {
        "lds_clocks_per_wave_instruction_of_1KB": dict(lds, how="one workgroup of eight waves issuing the same instruction "
                                                       "back to back, s_memtime from first issue to last result"),
        "mfma_bf16": {"published": cm.MI355X_BF16_FLOPS / 1e12, "measured": round(mfma / 1e12, 1), "unit": "TFLOP/s",
                      "how": "v_mfma_f32_32x32x16_bf16 on register operands, 8 independent accumulators per wave, "
                             "8 waves per workgroup, %d workgroups x %d iterations" % (wgs, iters)},
        "hbm_copy": {"published": cm.MI355X_HBM_BW / 1e9, "measured": round(copy / 1e9, 1), "unit": "GB/s",
                     "how": "1 GiB device copy, 16-byte accesses, read + write bytes counted"},
    }


def add_measured_fractions(roofline, peaks):
    roofline["peak_measured"] = peaks["mfma_bf16"]["measured"]
    roofline["frac_of_measured_peak"] = round(roofline["achieved"] / peaks["mfma_bf16"]["measured"], 4)


def measure(workload, steps, warmup, copy_calibration, n_dist=0):
    """Steady-state timing of sdv2_denoise_step on one workload: the headline pass and the per-launch pass."""
    import numpy as np
    import torch
    from paper_2511_07399_amd import binding, cost_model as cm, workloads as wk
    from paper_2511_07399_amd.runner import DeviceModel

    wl = wk.WORKLOADS[workload]
    dev = "cuda:0"
    B, L, Cw = wl.B, wl.L, wl.C
    gpu = DeviceModel(wl, base_seed=0, device=dev, weight_device=dev)
    frames = wl.frames_per_chunk
    n_inputs = 8
    xs = [torch.stack([wk.chunk_input(wl, c, s, device=dev) for s in range(B)]).contiguous() for c in range(n_inputs)]
    stream = torch.cuda.current_stream()

    if copy_calibration:
        src = torch.empty(copy_calibration * (1 << 20) // 4, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # fill the caches so that the timed steps run at steady state (every chunk evicts)
    fill_chunks = (wl.sink_frames + wl.window_frames + frames - 1) // frames + 1
    chunk = 0

    def one_step(c):
        x = xs[c % n_inputs].clone()
        descs = [(s, c * frames, frames, 1) for s in range(B)]
        ts = [wk.timestep(wl, c, 0, s) for s in range(B)]
        return x, descs, ts

    for _ in range(fill_chunks + warmup):
        x, descs, ts = one_step(chunk)
        gpu.denoise(x, descs, timesteps=ts)
        chunk += 1
    torch.cuda.synchronize()
    st = gpu.state(0, 0)
    assert st["win_fill"] == wl.W and st["evicted"] > 0, "not at steady state"
    l_kv = st["sink_fill"] + st["win_fill"]

    # ---- pass 1: the headline number
    prepared = [one_step(chunk + i) for i in range(steps)]
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev0.record(stream)
    for x, descs, ts in prepared:
        gpu.denoise(x, descs, timesteps=ts)
    ev1.record(stream)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps
    ms_per_step = ev0.elapsed_time(ev1) / steps
    chunk += steps
    assert all(torch.isfinite(x).all().item() for x, _, _ in prepared[-2:])

    # ---- pass 2: same steps again with per-launch events
    n_launch = steps * wl.N * len(binding.LAUNCH_TAGS)
    prepared = [one_step(chunk + i) for i in range(steps)]
    torch.cuda.synchronize()
    binding.prof_begin(n_launch)
    for x, descs, ts in prepared:
        gpu.denoise(x, descs, timesteps=ts)
    samples = binding.prof_end(n_launch)
    chunk += steps
    per_tag = {}
    for tag, ms in samples:
        per_tag.setdefault(tag, []).append(ms)
    rows = B * L
    flops = {
        1: cm.gemm_flops(rows, 3 * Cw, Cw), 4: cm.gemm_flops(rows, Cw, Cw), 6: cm.gemm_flops(rows, Cw, Cw),
        9: cm.gemm_flops(rows, Cw, Cw), 11: cm.gemm_flops(rows, wl.F, Cw), 12: cm.gemm_flops(rows, Cw, wl.F),
        3: cm.attention_flops(rows, l_kv, Cw), 8: cm.attention_flops(rows, wl.L_t, Cw),
    }
    hbm_bytes = {
        0: rows * Cw * (4 + 2), 5: rows * Cw * (4 + 2), 10: rows * Cw * (4 + 2),      # fp32 x in, bf16 h out
        2: rows * Cw * 2 * (3 + 3), 7: rows * Cw * 2 * 2,                              # qkv in; q, k, v out
    }
    kernels = {}
    for tag, vals in sorted(per_tag.items()):
        avg_us = float(np.mean(vals)) * 1e3
        entry = {"avg_us": round(avg_us, 2), "launches": len(vals)}
        if tag in flops:
            entry["tflops"] = round(flops[tag] / (avg_us * 1e-6) / 1e12, 1)
            entry["frac_mfma_peak"] = round(flops[tag] / (avg_us * 1e-6) / cm.MI355X_BF16_FLOPS, 4)
        if tag in hbm_bytes:
            entry["gbps"] = round(hbm_bytes[tag] / (avg_us * 1e-6) / 1e9, 1)
            entry["frac_hbm_peak"] = round(hbm_bytes[tag] / (avg_us * 1e-6) / cm.MI355X_HBM_BW, 4)
        kernels[binding.LAUNCH_TAGS[tag]] = entry
    gemm_tags = (1, 4, 6, 9, 11, 12)
    attn_tags = (3, 8)
    sum_us = lambda tags: sum(float(np.mean(per_tag[t])) * 1e3 for t in tags if t in per_tag)
    gemm_tflops = sum(flops[t] for t in gemm_tags) / (sum_us(gemm_tags) * 1e-6) / 1e12
    attn_tflops = sum(flops[t] for t in attn_tags) / (sum_us(attn_tags) * 1e-6) / 1e12
    # Dominant kernel = the kernel instantiation (as a profiler names it) whose launch sites together take the largest
    # share of the step: the library tells which instantiation its planner picks for each site's shape.
    cap = (wl.S + wl.W + 63) // 64 * 64
    cap_t = (wl.L_t + 63) // 64 * 64
    site_kernel = {
        1: binding.prof_kernel_name("gemm", B, L, 3 * Cw, Cw, 0), 4: binding.prof_kernel_name("gemm", B, L, Cw, Cw, 2),
        6: binding.prof_kernel_name("gemm", B, L, Cw, Cw, 0), 9: binding.prof_kernel_name("gemm", B, L, Cw, Cw, 3),
        11: binding.prof_kernel_name("gemm", B, L, wl.F, Cw, 1), 12: binding.prof_kernel_name("gemm", B, L, Cw, wl.F, 2),
        3: binding.prof_kernel_name("attention", B, L, wl.H, l_kv, cap),
        8: binding.prof_kernel_name("attention", B, L, wl.H, wl.L_t, cap_t),
    }
    groups = {}
    for tag, name in site_kernel.items():
        if tag in per_tag:
            groups.setdefault(name, []).append(tag)
    all_us = sum_us(per_tag.keys())
    dom_name, dom_tags = max(groups.items(), key=lambda kv: sum_us(kv[1]))
    dom_tags = sorted(dom_tags)
    dom_us = sum_us(dom_tags) / len(dom_tags)                       # average duration of one launch site of the kernel
    dom_flops = sum(flops[t] for t in dom_tags) / len(dom_tags)     # average algorithmic flops of one such launch site
    achieved = dom_flops / (dom_us * 1e-6) / 1e12
    for tag, name in site_kernel.items():
        if binding.LAUNCH_TAGS[tag] in kernels:
            kernels[binding.LAUNCH_TAGS[tag]]["kernel"] = name
    roofline = {
        "bound": "mfma", "kernel": dom_name, "launch_sites": [binding.LAUNCH_TAGS[t] for t in dom_tags],
        "share_of_step_time": round(sum_us(dom_tags) / all_us, 4),
        "achieved": round(achieved, 1), "peak": cm.MI355X_BF16_FLOPS / 1e12, "unit": "TFLOP/s",
        "frac": round(achieved * 1e12 / cm.MI355X_BF16_FLOPS, 4), "avg_launch_us": round(dom_us, 2),
        "flops_per_launch": dom_flops,
        "note": "durations are HIP-event brackets around each launch (the reduce pass of a k-split GEMM and the merge "
                "pass of a split-KV attention are launches of their own); they read 2-3 us above rocprofv3's kernel durations",
        "traffic": load_traffic(wl.name, dom_name),
    }
    step_flops = wl.N * cm.block_flops(rows, Cw, wl.F, l_kv, wl.L_t)
    latency = None
    if n_dist:
        # bound the pass to about ten seconds of GPU time
        per_chunk_ms = ms_per_step * sum(set((1,) + tuple(wl.steps)))
        latency = latency_distribution(gpu, wl, xs, min(n_dist, max(8, int(10000.0 / per_chunk_ms))))
    gpu.close()
    del gpu, xs, prepared
    torch.cuda.empty_cache()
    return {"ms_per_step": ms_per_step, "wall_ms": wall_ms, "kernels": kernels, "roofline": roofline,
            "step_flops": step_flops, "gemm_tflops": gemm_tflops, "attn_tflops": attn_tflops, "l_kv": l_kv,
            "latency": latency}



def latency_distribution(gpu, wl, xs, n_chunks):
    """Per-chunk latency of a stream started from an empty cache: every denoise step is bracketed by events on the
    launch stream (no synchronisation until the end).  Reports the warm-up chunks (the cache is filling, fewer keys)
    one by one and the distribution over the steady-state chunks, for 1 denoising step per chunk and for the other
    step counts the workload names (all steps of a chunk summed; steps after the first rewrite the chunk's K/V)."""
    import numpy as np
    import torch
    from paper_2511_07399_amd import binding, workloads as wk
    stream = torch.cuda.current_stream()
    B, frames = wl.B, wl.frames_per_chunk
    fill = (wl.sink_frames + wl.window_frames + frames - 1) // frames
    out = {}
    for n_steps in sorted(set((1,) + tuple(wl.steps))):
        for s_id in range(B):
            binding.kv_cache_reset(gpu.cache, s_id)
        total = fill + n_chunks
        inputs = [xs[c % len(xs)].clone() for c in range(min(total, 16))]
        evs = [[torch.cuda.Event(enable_timing=True) for _ in range(n_steps + 1)] for _ in range(total)]
        torch.cuda.synchronize()
        for c in range(total):
            x = inputs[c % len(inputs)]
            evs[c][0].record(stream)
            for st in range(n_steps):
                descs = [(s_id, c * frames, frames, 1 if st == 0 else 0) for s_id in range(B)]
                ts = [wk.timestep(wl, c, st, s_id) for s_id in range(B)]
                gpu.denoise(x, descs, timesteps=ts)
                evs[c][st + 1].record(stream)
        torch.cuda.synchronize()
        per_chunk = np.array([evs[c][0].elapsed_time(evs[c][n_steps]) for c in range(total)])
        steady = per_chunk[fill:]
        q = lambda p: round(float(np.percentile(steady, p)), 4)
        out["%d step(s) per chunk" % n_steps] = {
            "warmup_chunk_ms": [round(float(v), 4) for v in per_chunk[:fill]],
            "steady_chunk_ms": {"n": int(steady.size), "median": q(50), "p10": q(10), "p90": q(90), "p99": q(99),
                                "mean": round(float(steady.mean()), 4)},
        }
    return out


def batch_sweep(workload, sizes, steps, warmup):
    """L(T, B): the denoise-step latency of the workload with B independent streams in one call, and what
    sdv2_slo_pick_batch makes of the table (Section 4.1, SLO-aware batching scheduler)."""
    import dataclasses
    from paper_2511_07399_amd import binding, workloads as wk
    base = wk.WORKLOADS[workload]
    table = {}
    for b in sizes:
        name = "%s/B%d" % (base.name, b)
        wk.WORKLOADS[name] = dataclasses.replace(base, name=name, B=b)
        m = measure(name, steps, warmup, 0)
        table[b] = m["ms_per_step"]
        print("B=%d: %.3f ms per step" % (b, table[b]), file=sys.stderr, flush=True)
    T = base.frames_per_chunk
    lat = {b: ms * 1e-3 for b, ms in table.items()}
    freq = {b: b * T / lat[b] for b in lat}
    b1 = min(lat)
    picks = {}
    for f_slo in (16.0, 0.9 * max(freq.values()), 2.0 * max(freq.values())):
        for tol in (0.0, 0.05):
            r = binding.slo_pick_batch(lat, T, f_slo, 10 ** 6, tol)
            picks["f_slo %.1f, knee_tol %.2f" % (f_slo, tol)] = None if r is None else {"B": r[0], "f": round(r[1], 1), "meets_slo": r[2]}
    return {"workload": base.name, "frames_per_chunk": T, "ms_per_step": {str(b): round(v, 4) for b, v in table.items()},
            "frames_per_s": {str(b): round(freq[b], 1) for b in freq},
            "f_over_f1": {str(b): round(freq[b] / freq[b1], 3) for b in freq},
            "memory_bound_model_B_over_1_plus_B": {str(b): round((b / (1.0 + b)) / (b1 / (1.0 + b1)), 3) for b in freq},
            "picks": picks}


def measure_graph_replay(workload, steps, warmup):
    """The same steady-state steps through sdv2_denoise_graph_launch (the step recorded once as a HIP graph, the ring
    positions in a device-side descriptor), each step's input copied into the recorded buffer inside the timed region:
    GPU time per step between events, and the host's time to enqueue a step (no synchronisation inside the loop),
    beside the same two numbers for the eager sdv2_denoise_step."""
    import torch
    from paper_2511_07399_amd import binding, workloads as wk
    from paper_2511_07399_amd.runner import DeviceModel
    wl = wk.WORKLOADS[workload]
    dev = "cuda:0"
    stream = torch.cuda.current_stream()
    B, L, frames = wl.B, wl.L, wl.frames_per_chunk
    gpu = DeviceModel(wl, base_seed=0, device=dev, weight_device=dev)
    xs = [torch.stack([wk.chunk_input(wl, c, s, device=dev) for s in range(B)]).contiguous() for c in range(4)]
    x = torch.zeros(B, L, wl.C, dtype=torch.float32, device=dev)
    handle = gpu.graph(x, list(range(B)), frames)
    fill = (wl.sink_frames + wl.window_frames + frames - 1) // frames + 1
    out = {}
    chunk = 0

    def run(n, mode):
        nonlocal chunk
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ev0.record(stream)
        for _ in range(n):
            descs = [(s, chunk * frames, frames, 1) for s in range(B)]
            ts = [wk.timestep(wl, chunk, 0, s) for s in range(B)]
            x.copy_(xs[chunk % 4])
            if mode == "graph":
                binding.denoise_graph_launch(handle, ts, binding.chunk_descs(descs))
            else:
                gpu.denoise(x, descs, timesteps=ts)
            chunk += 1
        ev1.record(stream)
        host_ms = (time.perf_counter() - t0) * 1e3 / n
        torch.cuda.synchronize()
        return ev0.elapsed_time(ev1) / n, host_ms

    run(fill + warmup, "graph")
    st = gpu.state(0, 0)
    assert st["win_fill"] == wl.W and st["evicted"] > 0
    for mode in ("graph", "eager", "graph"):
        ms, host_ms = run(steps, mode)
        out[mode] = {"ms_per_step": round(ms, 4), "host_enqueue_ms_per_step": round(host_ms, 4)}
    assert bool(torch.isfinite(x).all())
    binding.denoise_graph_destroy(handle)
    gpu.close()
    del gpu
    torch.cuda.empty_cache()
    return {"workload": "%s at steady state, %d steps per pass, input copy included" % (wl.name, steps), **out}


def measure_stream_batch(workload, depths=(2, 4), steps=12):
    """Stream batch over denoising steps (Section 4.2): one stream denoised in n steps per chunk runs as n batch rows
    at n noise depths, each depth with its own rolling cache, one batched denoise step per micro-step and one
    finished chunk per micro-step.  Steady state (pipeline full, every depth cache full and evicting): latency of a
    micro-step, which is also the time between finished chunks, and the same per batch row."""
    import dataclasses
    import torch
    from paper_2511_07399_amd import binding, cost_model as cm, workloads as wk
    from paper_2511_07399_amd.runner import DeviceModel
    base = wk.WORKLOADS[workload]
    dev = "cuda:0"
    stream = torch.cuda.current_stream()
    out = {}
    for n in depths:
        wl = dataclasses.replace(base, name="%s/n%d" % (base.name, n), B=n)
        gpu = DeviceModel(wl, base_seed=0, device=dev, weight_device=dev)
        kt = binding.ptr_array([gpu.kt[layer][0] for layer in range(wl.N)])
        vtt = binding.ptr_array([gpu.vtt[layer][0] for layer in range(wl.N)])
        rows = torch.empty(binding.stream_batch_rows_bytes(gpu.cfg, n, wl.frames_per_chunk), dtype=torch.uint8, device=dev)
        sb = binding.stream_batch_create(gpu.cfg, n, list(range(n)), wl.frames_per_chunk, rows)
        ws = gpu.workspace(n, wl.L)
        xs = [wk.chunk_input(wl, c, 0, device=dev) for c in range(4)]
        x_out = torch.empty(wl.L, wl.C, dtype=torch.float32, device=dev)
        ts = [1000.0 * (n - d) / (n + 1) for d in range(n)]             # a fixed schedule, noisiest first
        fill = (wl.sink_frames + wl.window_frames) // wl.frames_per_chunk + n + 2
        m = 0
        for _ in range(fill):
            binding.stream_batch_step(sb, gpu.cfg, gpu.mw, gpu.cache, xs[m % 4], m * wl.frames_per_chunk, ts, kt, vtt, x_out, ws)
            m += 1
        torch.cuda.synchronize()
        st = gpu.state(wl.N - 1, n - 1)
        assert st["win_fill"] == wl.W and st["evicted"] > 0, "deepest cache not at steady state"
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        ev0.record(stream)
        emitted = 0
        for _ in range(steps):
            e, r = binding.stream_batch_step(sb, gpu.cfg, gpu.mw, gpu.cache, xs[m % 4], m * wl.frames_per_chunk, ts, kt, vtt, x_out, ws)
            assert r == n
            emitted += int(e)
            m += 1
        ev1.record(stream)
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) * 1e3 / steps
        ms = ev0.elapsed_time(ev1) / steps
        assert emitted == steps and bool(torch.isfinite(x_out).all())
        l_kv = st["sink_fill"] + st["win_fill"]
        flops = wl.N * cm.block_flops(n * wl.L, wl.C, wl.F, l_kv, wl.L_t)
        out["%d steps per chunk" % n] = {
            "batch_rows": n, "ms_per_micro_step": round(ms, 4), "wall_ms_per_micro_step": round(wall, 4),
            "ms_per_row": round(ms / n, 4), "finished_chunks_per_s": round(1e3 / ms, 1),
            "step_tflops": round(flops / (ms * 1e-3) / 1e12, 1),
            "step_frac_mfma_peak": round(flops / (ms * 1e-3) / cm.MI355X_BF16_FLOPS, 4)}
        # the same rotation with rows of latents (patch embedding, head and sampler update inside every micro-step)
        binding.stream_batch_reset(sb)
        for layer_stream in range(n):
            binding.kv_cache_reset(gpu.cache, layer_stream)
        io = gpu.io()
        ws_l = torch.empty(binding.stream_batch_latents_workspace_bytes(gpu.cfg, n, wl.frames_per_chunk), dtype=torch.uint8, device=dev)
        zs = [wk.latent_chunk(wl, c, 0, device=dev).contiguous() for c in range(4)]
        eps = torch.stack([wk.latent_chunk(wl, 0, 0, device=dev, kind=2 + d) for d in range(n)]).contiguous()
        z_out = torch.empty_like(zs[0])
        sig = [1.0 - d / n for d in range(n + 1)]
        m = 0
        for _ in range(fill):
            binding.stream_batch_latents_step(sb, gpu.cfg, gpu.mw, io, gpu.cache, zs[m % 4], m * wl.frames_per_chunk, sig, eps, kt, vtt, z_out, ws_l)
            m += 1
        torch.cuda.synchronize()
        ev0.record(stream)
        for _ in range(steps):
            binding.stream_batch_latents_step(sb, gpu.cfg, gpu.mw, io, gpu.cache, zs[m % 4], m * wl.frames_per_chunk, sig, eps, kt, vtt, z_out, ws_l)
            m += 1
        ev1.record(stream)
        torch.cuda.synchronize()
        assert bool(torch.isfinite(z_out).all())
        out["%d steps per chunk" % n]["ms_per_micro_step_rows_of_latents"] = round(ev0.elapsed_time(ev1) / steps, 4)
        binding.stream_batch_destroy(sb)
        gpu.close()
        del gpu, rows, ws, xs, ws_l
        torch.cuda.empty_cache()
    return {"workload": "%s, one stream, n denoising steps per chunk as n batch rows at n noise depths (own cache per "
                        "depth), steady state, %d timed micro-steps" % (base.name, steps), "depths": out}


def measure_latents(workload, steps=10):
    """The same step with latents in and latents out (sdv2_denoise_latents_step: timestep vector, patch embedding, the
    blocks, output head, sampler update) beside the hidden-state step the headline times: what the steps around the
    blocks add.  Cache at steady state, one stream, one denoising step per chunk."""
    import torch
    from paper_2511_07399_amd import workloads as wk
    from paper_2511_07399_amd.runner import DeviceModel
    wl = wk.WORKLOADS[workload]
    dev = "cuda:0"
    stream = torch.cuda.current_stream()
    gpu = DeviceModel(wl, base_seed=0, device=dev, weight_device=dev, n_streams=1)
    gpu.io()
    zs = [wk.latent_chunk(wl, c, 0, device=dev).unsqueeze(0).contiguous() for c in range(4)]
    eps = wk.latent_chunk(wl, 0, 0, device=dev, kind=1).unsqueeze(0).contiguous()
    z = torch.empty_like(zs[0])
    fill = (wl.sink_frames + wl.window_frames) // wl.frames_per_chunk + 3
    c = 0
    for _ in range(fill):
        z.copy_(zs[c % 4])
        gpu.denoise_latents(z, [(0, c * wl.frames_per_chunk, wl.frames_per_chunk, 1)], [0.75], [0.5], eps_next=eps)
        c += 1
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record(stream)
    for _ in range(steps):
        gpu.denoise_latents(z, [(0, c * wl.frames_per_chunk, wl.frames_per_chunk, 1)], [0.75], [0.5], eps_next=eps)
        c += 1
    ev1.record(stream)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(z).all())
    ms = ev0.elapsed_time(ev1) / steps
    gpu.close()
    return {"ms_per_step_latents_in_latents_out": round(ms, 4),
            "latent_shape": list(zs[0].shape[1:]), "entry_point": "sdv2_denoise_latents_step"}


def measure_refresh(workload, reps=20):
    """The three cache-refresh operations (sink similarity, sink copy, key move) on ONE (layer, stream) cache of the
    workload's geometry at steady state: average launch time over `reps` launches and the rate on their
    algorithmic bytes (similarity: the value rows of two frames per sink; copy: keys and values of a frame read and
    written; move: the 44 rotated elements of every head of every resident key read and written)."""
    import torch
    from paper_2511_07399_amd import binding, workloads as wk
    wl = wk.WORKLOADS[workload]
    dev = "cuda:0"
    ccfg = binding.cache_cfg(1, 1, wl.H, wl.P, wl.S, wl.W)
    storage = torch.zeros(binding.kv_cache_bytes(ccfg), dtype=torch.uint8, device=dev)
    h = binding.kv_cache_init(ccfg, storage)
    gen = torch.Generator().manual_seed(5)
    n = wl.frames_per_chunk * wl.P
    binding.kv_cache_append_evict(h, 0, 0, torch.randn(wl.S, wl.C, generator=gen).to(dev, torch.bfloat16),
                                  torch.randn(wl.S, wl.C, generator=gen).to(dev, torch.bfloat16), True)
    for _ in range(wl.W // n + 1):
        binding.kv_cache_append_evict(h, 0, 0, torch.randn(n, wl.C, generator=gen).to(dev, torch.bfloat16),
                                      torch.randn(n, wl.C, generator=gen).to(dev, torch.bfloat16), True)
    m = wl.S // wl.P
    alpha = torch.empty(m, dtype=torch.float32, device=dev)
    ws = torch.empty(binding.sink_similarity_workspace_bytes(h), dtype=torch.uint8, device=dev)

    def timed(fn):
        for i in range(3):
            fn(i)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for i in range(reps):
            fn(i)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps * 1e3

    frame = wl.P * wl.C * 2
    ops = {
        "sink similarity": (timed(lambda i: binding.sink_similarity(h, 0, 0, alpha, ws, 0)), 2 * frame * m),
        "sink copy": (timed(lambda i: binding.kv_cache_refresh_sink(h, 0, 0, 0, 0)), 4 * frame),
        "key move": (timed(lambda i: binding.kv_cache_rotate_keys(h, 0, 0, 3 if i % 2 == 0 else -3)),
                     2 * (wl.S + wl.W) * wl.H * 44 * 2),
    }
    binding.kv_cache_destroy(h)
    return {"cache": "%s: one layer, one stream, %d-token frames, sink %d + window %d tokens, C %d"
                     % (wl.name, wl.P, wl.S, wl.W, wl.C),
            "ops": {k: {"us": round(us, 2), "bytes": b, "GB/s": round(b / (us * 1e-6) / 1e9, 1)} for k, (us, b) in ops.items()}}


def measure_motion(reps=20):
    """The motion-aware noise scheduler update (frame differences + the rate recurrence) on 512 x 512 latents
    (16 x 64 x 64 fp32 per frame) for one and for four frames per call; algorithmic bytes: each frame and its
    predecessor read once."""
    import torch
    from paper_2511_07399_amd import binding
    dev = "cuda:0"
    n = 16 * 64 * 64
    cfg = binding.motion_cfg(3, 1.0, 0.3, 0.1, 0.9, 0.5)
    state = torch.empty(binding.motion_state_bytes(cfg), dtype=torch.uint8, device=dev)
    binding.motion_init(cfg, state)
    out = {}
    for T in (1, 4):
        frames = torch.randn(T, n, device=dev)
        prev = torch.randn(n, device=dev)
        o = [torch.empty(T, dtype=torch.float32, device=dev) for _ in range(3)]
        for _ in range(3):
            binding.motion_update(cfg, state, frames, prev, *o)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            binding.motion_update(cfg, state, frames, prev, *o)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) / reps * 1e3
        b = 2 * T * n * 4
        out["%d frame(s) of 16x64x64 fp32" % T] = {"us": round(us, 2), "bytes": b, "GB/s": round(b / (us * 1e-6) / 1e9, 1)}
    return out


def load_traffic(workload, kernel):
    """HBM bytes per launch of the dominant kernel, as derived from the rocprofv3 --pmc runs whose summary
    is committed under profiles/ (null when no such measurement is recorded for this kernel of this workload:
    counters cannot be read from inside the timed run)."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    try:
        with open(path) as f:
            return json.load(f).get(workload, {}).get(kernel)
    except (OSError, ValueError):
        return None


def time_oracle(wl, n_layers_req):
    """Wall clock of the oracle's denoise step at steady state on the host cores.

    Layers are timed one after the other so that only one layer's float64 weights are alive; the
    caches are pre-filled with random history (untimed) so that the step attends over a full
    window.  If the model has more layers than fit ~30 s, the first layers are timed and scaled.
    """
    import numpy as np
    import oracle
    from paper_2511_07399_amd import workloads as wk
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count()
    flops_block = wl.block_flops() / wl.B
    budget_flops = 25.0 * 250e9          # ~25 s at the ~250 GFLOP/s float64 BLAS rate of a 16-core share
    n_layers = n_layers_req or max(1, min(wl.N, int(budget_flops / flops_block)))
    mw = wk.to_numpy(wk.model_weights(wl))
    t = wk.timestep(wl, 0)
    x = wk.chunk_input(wl, 0).double().numpy()
    t_start = time.perf_counter()
    e0 = oracle.conditioning(mw, t=t)
    timed = time.perf_counter() - t_start
    rng = np.random.default_rng(0)
    for layer in range(n_layers):
        w = wk.to_numpy(wk.block_weights(wl, layer))
        ctx = wk.text_context(wl).double().numpy()
        tk, tv = oracle.text_kv_prepare(ctx, w)
        cache = oracle.RollingKVCache(wl.S, wl.W, wl.P, wl.C)
        done = 0
        while done < wl.S + wl.W:          # random history, untimed
            n = min(wl.L, wl.W)
            cache.append_evict(rng.standard_normal((n, wl.C)), rng.standard_normal((n, wl.C)))
            done += n
        t_start = time.perf_counter()
        x = oracle.dit_block_forward(x, e0, w, cache, tk, tv, wl.H, wl.P, wl.grid_w, frame_pos0=100)
        timed += time.perf_counter() - t_start
    scale = wl.N / n_layers
    ms = timed * 1e3 * scale * wl.B
    return {
        "value": round(ms, 1), "unit": "ms", "cores": cores, "kind": "oracle",
        "sample": "oracle (numpy float64) denoise step at steady state, %d of %d blocks timed on one stream%s"
                  % (n_layers, wl.N, "" if n_layers == wl.N and wl.B == 1 else
                     ", scaled x%.2f to %d blocks x %d stream(s)" % (scale * wl.B, wl.N, wl.B)),
    }


if __name__ == "__main__":
    main()
