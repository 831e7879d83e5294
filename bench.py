#!/usr/bin/env python3
"""Benchmark of hybrid-batch attention on one MI355X.

One "step" is one pod_attn_forward call (every stage of the hot path: role binding, prefill
items, decode units, split-KV combine) on one synthetic hybrid batch whose inputs already sit
in HBM.  Prints ONE JSON line on stdout; details of the comparison modes go to stderr.

The headline workload is configuration 4 (the long-context, grouped-query batch: the only one
bound by the matrix units, and the one furthest from its roofline).  The same line carries a
`configs` array with every other benchmark batch (configurations 2 and 3 and the twelve batches
of the ratio sweep), each timed the same way and checked against the oracle on sampled rows.

    python bench.py [--gpus 1] [--steps 30] [--warmup 5] [--config 4] [--batch-index 0]
                    [--no-cpu-baseline] [--mode fused] [--no-configs] [--sweep FILE]
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

PEAK_MFMA_16BIT = 2.5e15        # dense fp16/bf16 MFMA flop/s, MI355X
PEAK_HBM = 8.0e12               # bytes/s, MI355X HBM3E
# HBM bytes per fused launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this same
# command (`--config N --no-configs`), scaled by what the same counters read for a plain device copy
# of known size; None = not measured.  These come from the files under profiles/, not from this run.
MEASURED_TRAFFIC_BYTES = {
    # (config, batch_index): {kernel: FETCH_SIZE KiB x 2.0 (copy calibration: the counter reads half of a
    # plain copy's bytes) + WRITE_SIZE KiB x 1.0, per launch}  (files under profiles/)
    (2, 0): {"fused_kernel": 4416896205, "fused_cta_kernel": 4623039283},
    #   fused_kernel: 2145859.8 KiB fetched, 21655.6 KiB written
    #   fused_cta_kernel: 2246222.3 KiB fetched, 22242.2 KiB written
    (3, 0): {"fused_kernel": 4994009498, "fused_cta_kernel": 5153556582},
    #   fused_kernel: 2417927.3 KiB fetched, 41107.8 KiB written
    #   fused_cta_kernel: 2495912.2 KiB fetched, 40945.7 KiB written
    (4, 0): {"fused_kernel": 2582235443, "fused_cta_kernel": 2749092147},
    #   fused_kernel: 1240935.5 KiB fetched, 39843.3 KiB written
    #   fused_cta_kernel: 1322148.0 KiB fetched, 40364.3 KiB written
}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def event_times_us(fn, steps, torch):
    """Per-call durations from HIP events recorded on torch's current stream (the launch stream)."""
    starts = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
    stops = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
    for i in range(steps):
        starts[i].record()
        fn()
        stops[i].record()
    torch.cuda.synchronize()
    return np.array([s.elapsed_time(e) * 1e3 for s, e in zip(starts, stops)])


def sample_rows(batch, n_prefill_rows_wanted, n_decode_wanted, seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    npr = batch.n_prefill_rows
    pr = np.sort(rng.choice(npr, size=min(npr, n_prefill_rows_wanted), replace=False)) if npr else np.array([], int)
    dr = np.sort(rng.choice(batch.n_decode, size=min(batch.n_decode, n_decode_wanted), replace=False)) \
        if batch.n_decode else np.array([], int)
    return np.concatenate([pr, npr + dr]).astype(np.int32)


def pairs_of_rows(batch, rows):
    """Visible (row, key) pairs of the given output rows (per query head)."""
    npr = batch.n_prefill_rows
    total = 0
    starts = batch.seq_meta[:batch.n_prefill, 0]
    for g in rows:
        if g < npr:
            r = int(np.searchsorted(starts, g, side="right") - 1)
            q_start, q_len, kv_len, _ = (int(x) for x in batch.seq_meta[r])
            total += kv_len - q_len + (g - q_start) + 1
        else:
            r = batch.n_prefill + int(np.nonzero(batch.seq_meta[batch.n_prefill:, 0] == g - npr)[0][0])
            total += int(batch.seq_meta[r, 2])
    return total


def all_pairs(batch):
    return batch.visible_pairs() + int(batch.seq_meta[batch.n_prefill:, 2].sum())


def measure_peaks(torch, pod):
    """What this GPU sustains: a coalesced 4 GiB read stream and a dense fp16 MFMA issue loop."""
    buf = torch.empty(4 << 30, dtype=torch.uint8, device="cuda:0")
    buf.zero_()
    sink = torch.zeros(16, dtype=torch.uint8, device="cuda:0")
    rd = lambda: pod.pod_attn_probe_hbm_read(buf.data_ptr(), buf.numel(), sink.data_ptr(),
                                             torch.cuda.current_stream().cuda_stream)
    for _ in range(3):
        rd()
    t_rd = float(np.median(event_times_us(rd, 10, torch)))
    flops = [0.0]

    def mf():
        flops[0] = pod.pod_attn_probe_mfma(20000, sink.data_ptr(), torch.cuda.current_stream().cuda_stream)
    for _ in range(2):
        mf()
    t_mf = float(np.median(event_times_us(mf, 5, torch)))
    del buf
    torch.cuda.empty_cache()
    return {"hbm_read_GBps": (4 << 30) / t_rd / 1e3, "mfma_f16_TFLOPs": flops[0] / t_mf / 1e6}


def plan_times_us(attn, torch, pod, reps=5):
    """Host time of the two calls made once per batch (every layer's forward reuses their result):
    building the plan, and copying its tables into a workspace (ends with a stream synchronisation)."""
    scratch = torch.empty(attn.ws_bytes + 256, dtype=torch.uint8, device=attn.workspace.device)
    ws = (scratch.data_ptr() + 255) & ~255
    stream = torch.cuda.current_stream().cuda_stream
    torch.cuda.synchronize()
    create, upload = [], []
    for _ in range(reps):
        t0 = time.perf_counter()
        plan = pod.pod_attn_plan_create(attn.params, attn.batch_meta)
        t1 = time.perf_counter()
        pod.pod_attn_plan_upload(plan, ws, attn.ws_bytes, stream)
        t2 = time.perf_counter()
        plan.close()
        create.append((t1 - t0) * 1e6)
        upload.append((t2 - t1) * 1e6)
    return {"create_us": float(np.median(create)), "upload_us": float(np.median(upload))}


CLOCK_RAMP_S = 0.08


def ramp_clocks(fn, torch):
    """Untimed calls for CLOCK_RAMP_S of wall time.  After the GPU has idled (here: while the host
    runs the oracle, copies inputs or builds a plan) its clocks take 20-40 ms of work to come back
    up; calls timed in that window measure 5-15 % slow (configuration 4: 1328 us for iterations 5-24
    after two idle seconds, 1257 us from iteration 50 on).  This is not one of the `--warmup` steps."""
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < CLOCK_RAMP_S:
        for _ in range(4):
            fn()
        torch.cuda.synchronize()


def wall_us_per_step(fn, steps, warmup, torch):
    """Mean time of exactly `steps` back-to-back calls, bracketed by synchronisation, after
    `warmup` untimed calls (and, before those, the clock ramp above)."""
    ramp_clocks(fn, torch)
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t1) / steps * 1e6


def run_clock_by_mode(config, batch_index, torch, pod, wl):
    """Graphics clock under each schedule in a sustained loop, and each schedule's time per launch
    sustained, with a synchronisation after every launch, and with 20 ms of idle time before it."""
    import re
    import subprocess
    import threading
    batch = wl.config_batch(config, batch_index, device="cuda:0")
    out = torch.empty((batch.n_rows, batch.n_q_heads, batch.head_dim), dtype=batch.torch_dtype, device="cuda:0")
    attn = pod.HybridAttention(batch)
    attn_base = pod.HybridAttention(batch, max_prefill_waves=2)
    bs = batch.block_size
    heavy_built = batch.head_dim == 128 and (bs == 0 or (bs >= 16 and bs & (bs - 1) == 0))
    modes = ["decode_only", "prefill_only", "serial", "fused"] + (["fused_heavy"] if heavy_built else [])

    def sample(stop, acc):
        while not stop.is_set():
            try:
                r = subprocess.run(["rocm-smi", "--showclocks"], capture_output=True, text=True, timeout=5)
                m = re.search(r"sclk clock level: *\d+: *\((\d+)Mhz\)", r.stdout)
                if m:
                    acc.append(int(m.group(1)))
            except (OSError, subprocess.SubprocessError):
                pass
            time.sleep(0.25)

    print(f"graphics clock and time per launch by schedule: {batch.name} (one MI355X; sclk from rocm-smi while the "
          f"schedule loops for 3 s; us per launch: in that loop / with a synchronisation after every launch / "
          f"with 20 ms of idle time before every launch)")
    for name in modes:
        which = attn if name in ("fused", "decode_only") else attn_base
        f = lambda: which.forward(batch, out=out, mode=pod.MODES[name])
        stop, acc = threading.Event(), []
        th = threading.Thread(target=sample, args=(stop, acc))
        th.start()
        t0 = time.perf_counter()
        n = 0
        while time.perf_counter() - t0 < 3.0:
            for _ in range(50):
                f()
            torch.cuda.synchronize()
            n += 50
        sustained = (time.perf_counter() - t0) / n * 1e6
        stop.set()
        th.join()
        one, spaced = [], []
        for gap, dst in ((0.0, one), (0.02, spaced)):
            for _ in range(12):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                torch.cuda.synchronize()
                time.sleep(gap)
                e0.record()
                f()
                e1.record()
                torch.cuda.synchronize()
                dst.append(e0.elapsed_time(e1) * 1e3)
        clk = f"{int(np.median(acc[2:] or acc or [0]))} MHz (min {min(acc or [0])}, max {max(acc or [0])}, {len(acc)} readings)"
        print(f"  {name:14s} sclk {clk:48s} {sustained:7.0f} / {np.median(one):7.0f} / {np.median(spaced):7.0f} us")
    attn.close()
    attn_base.close()


KERNEL_OF_MODE = {"serial": "prefill_kernel + decode_kernel",
                  "streams": "prefill_kernel + decode_kernel",
                  "fused_heavy": "prefill_heavy_kernel + decode_lite_kernel"}


def oracle_check(batch, out, wl, torch):
    """A function rows -> (max-abs error of `out` on those rows against the fp64 oracle, oracle seconds)."""
    from oracle import reference
    host = dict(pq=wl.bits(batch.prefill_q), dq=wl.bits(batch.decode_q), k=wl.bits(batch.k_cache),
                v=wl.bits(batch.v_cache), bt=None if batch.block_table is None else batch.block_table.cpu().numpy())
    kw = dict(n_prefill=batch.n_prefill, n_decode=batch.n_decode, n_q_heads=batch.n_q_heads,
              n_kv_heads=batch.n_kv_heads, head_dim=batch.head_dim, dtype=batch.dtype,
              softmax_scale=batch.softmax_scale, block_size=batch.block_size,
              max_blocks_per_seq=batch.max_blocks_per_seq, kv_seq_stride=batch.kv_seq_stride)

    def run(r):
        t1 = time.time()
        ref = reference.attention(host["pq"], host["dq"], host["k"], host["v"], batch.seq_meta, host["bt"], rows=r, **kw)
        dt = time.time() - t1
        got = out[torch.from_numpy(r.astype(np.int64)).to(out.device)].to(torch.float64).cpu().numpy()
        return float(np.abs(got - ref).max()), dt
    return run


def run_config(config, batch_index, steps, warmup, want_cpu, main_mode, torch, pod, wl, peaks=None,
               headline=True):
    """Time one benchmark batch in every mode, check it against the oracle on sampled rows and
    return its record.  `headline` adds what only the headline carries: the oracle timed as the CPU
    baseline on a larger sample, the dominant kernel alone, and the plan's host time."""
    dev = "cuda:0"
    t0 = time.time()
    batch = wl.config_batch(config, batch_index, device=dev)
    torch.cuda.synchronize()
    log(f"[bench] {batch.name}: inputs generated on the GPU in {time.time() - t0:.1f}s "
        f"(KV cache {2 * batch.k_cache.numel() * 2 / 2**30:.2f} GiB)")
    attn = pod.HybridAttention(batch)
    info = attn.info
    # The baselines get the plan that suits them: their stand-alone prefill kernel has both slots
    # of every compute unit to itself, so its items may fill two rounds (the fused launch plans one
    # round when a decode worker holds the other slot of every unit).
    attn_base = pod.HybridAttention(batch, max_prefill_waves=2)
    out = torch.empty((batch.n_rows, batch.n_q_heads, batch.head_dim), dtype=batch.torch_dtype, device=dev)
    baseline_modes = (pod.MODE_SERIAL, pod.MODE_STREAMS, pod.MODE_PREFILL_ONLY)

    def fwd(mode):
        # the prefill-heavy configuration also runs a stand-alone prefill kernel with both slots
        stand_alone = (mode & 0xff) in baseline_modes or (mode & pod.MODE_FLAG_PREFILL_HEAVY)
        which = attn_base if stand_alone else attn
        return lambda: which.forward(batch, out=out, mode=mode)

    bs = batch.block_size
    heavy_built = batch.head_dim == 128 and (bs == 0 or (bs >= 16 and bs & (bs - 1) == 0))

    flops = batch.prefill_flops()
    kv_bytes = batch.kv_bytes()
    t_f, t_b = flops / PEAK_MFMA_16BIT, kv_bytes / PEAK_HBM
    t_roof_us = max(t_f, t_b) * 1e6

    # --- correctness on sampled rows against the CPU oracle (on the headline also the cpu_baseline) ----
    cpu = None
    out.fill_(float("nan"))
    fwd(pod.MODES[main_mode])()
    torch.cuda.synchronize()
    check = oracle_check(batch, out, wl, torch)
    rows = sample_rows(batch, 96, 96, seed=config * 100 + batch_index) if headline else \
        sample_rows(batch, 12, 12, seed=config * 100 + batch_index)
    max_err, t_cpu = check(rows)
    n_pairs = pairs_of_rows(batch, rows)
    if headline and want_cpu:
        # the small sample has set the oracle's rate; one more sample sized for about 12 s of CPU work
        scale = 12.0 / max(t_cpu, 1e-3)
        if scale >= 2.0 and len(rows) < batch.n_rows:
            frac_p = batch.n_prefill_rows / max(batch.n_rows, 1)
            n_want = int(min(batch.n_rows, len(rows) * scale))
            rows = sample_rows(batch, int(n_want * frac_p) + 1, int(n_want * (1 - frac_p)) + 1,
                               seed=config * 100 + batch_index + 7)
            err2, t_cpu = check(rows)
            max_err = max(max_err, err2)
            n_pairs = pairs_of_rows(batch, rows)
        from oracle import reference
        est_us = t_cpu / n_pairs * all_pairs(batch) * 1e6
        cpu = {"value": est_us, "unit": "us/batch", "cores": reference.num_threads(), "kind": "oracle",
               "sample": f"{len(rows)} of {batch.n_rows} output rows (all {batch.n_q_heads} heads), "
                         f"{t_cpu:.1f}s of oracle time, scaled by visible (row,key) pairs"}
        log(f"[bench] oracle sample: {len(rows)} rows in {t_cpu:.1f}s -> est. {est_us / 1e6:.1f}s per batch")
    log(f"[bench] {batch.name}: max-abs error of the GPU output on sampled rows {max_err:.2e}")
    del check

    # --- timing: every mode the same way (exactly `steps` calls bracketed by synchronisation), ----
    # --- plus per-call HIP-event times on the launch stream for the spread ------------------------
    results = {}
    for name in ("fused", "serial", "streams", "prefill_only", "decode_only", "fused_cta", "fused_heavy"):
        if name == "fused_heavy" and not heavy_built:
            continue
        f = fwd(pod.MODES[name])
        wall = wall_us_per_step(f, steps, warmup, torch)
        ev = event_times_us(f, steps, torch)
        results[name] = {"wall_us": wall, "median_us": float(np.median(ev)), "min_us": float(ev.min()),
                         "p90_us": float(np.percentile(ev, 90))}
    value_us = results[main_mode]["wall_us"]
    bound = "hbm" if t_b >= t_f else "mfma"
    rec = {
        "workload": batch.name, "config": config, "batch_index": batch_index,
        "fused_us": results["fused"]["wall_us"], "serial_us": results["serial"]["wall_us"],
        "streams_us": results["streams"]["wall_us"], "fused_cta_parallel_us": results["fused_cta"]["wall_us"],
        "prefill_heavy_us": results["fused_heavy"]["wall_us"] if heavy_built else None,
        "prefill_heavy_advised": bool(info.prefill_heavy_advised),   # the planner's reading of Section 4.2.2's choice
        "overlap_roofline_us": t_roof_us, "bound": bound,
        "pct_of_overlap_roofline": 100.0 * t_roof_us / value_us,
        "frac": t_roof_us / value_us,
        "speedup_vs_serial": results["serial"]["wall_us"] / results["fused"]["wall_us"],
        "speedup_vs_streams": results["streams"]["wall_us"] / results["fused"]["wall_us"],
        "max_abs_err_vs_oracle": max_err, "rows_checked": int(len(rows)),
        "modes": results,
    }
    if not headline:
        attn.close()
        attn_base.close()
        return rec

    # the dominant kernel alone (no combine pass), for the roofline object
    f_kernel = fwd(pod.MODES[main_mode] | pod.MODE_FLAG_NO_COMBINE)
    for _ in range(warmup):
        f_kernel()
    kernel_us = float(np.mean(event_times_us(f_kernel, steps, torch)))
    attn.forward(batch, out=out, mode=pod.MODES[main_mode])       # leave `out` complete again
    torch.cuda.synchronize()
    plan_us = plan_times_us(attn, torch, pod)

    if bound == "hbm":
        achieved, peak, unit = kv_bytes / (kernel_us * 1e-6) / 1e9, PEAK_HBM / 1e9, "GB/s"
    else:
        achieved, peak, unit = flops / (kernel_us * 1e-6) / 1e12, PEAK_MFMA_16BIT / 1e12, "TFLOP/s"
    launched = {"fused": "fused_kernel", "fused_cta": "fused_cta_kernel"}.get(main_mode)
    traffic = MEASURED_TRAFFIC_BYTES.get((config, batch_index), {}).get(launched)
    head = {
        "metric": "hybrid-batch attention us per batch (fused prefill+decode)",
        "value": value_us, "unit": "us", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": value_us / 1e3, "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16" if batch.dtype == wl.F16 else "bf16", "data": "synthetic",
        "config": {"workload": batch.name, "config": config, "batch_index": batch_index, "mode": main_mode,
                   "n_q_heads": batch.n_q_heads, "n_kv_heads": batch.n_kv_heads, "head_dim": batch.head_dim,
                   "prefill": [[int(m[1]), int(m[2])] for m in batch.seq_meta[:batch.n_prefill]],
                   "n_decode": batch.n_decode,
                   "decode_ctx_mean": float(batch.seq_meta[batch.n_prefill:, 2].mean()) if batch.n_decode else 0.0,
                   "kv_layout": f"paged{batch.block_size}" if batch.block_size else "contiguous",
                   "prefill_items": info.n_prefill_items, "decode_units": info.n_decode_units,
                   "role_ratio": [info.prefill_ratio, info.decode_ratio],
                   "prefill_heavy_advised": bool(info.prefill_heavy_advised)},
        "roofline": {"bound": bound, "achieved": achieved, "peak": peak, "unit": unit, "frac": achieved / peak,
                     "traffic": traffic,
                     "traffic_source": "rocprofv3 --pmc summaries under profiles/ (separate runs of this command), not this run",
                     "kernel": launched or KERNEL_OF_MODE[main_mode], "kernel_us": kernel_us,
                     "algorithmic_bytes": kv_bytes, "algorithmic_flops": flops},
        # value, the roofline percentage and the speed-ups all use the same clock: exactly `steps`
        # back-to-back forward calls (combine pass included) bracketed by synchronisation
        "overlap_roofline_us": t_roof_us, "pct_of_overlap_roofline": rec["pct_of_overlap_roofline"],
        "prefill_flops_time_us": t_f * 1e6, "kv_bytes_time_us": t_b * 1e6,
        "speedup_vs_serial": rec["speedup_vs_serial"], "speedup_vs_streams": rec["speedup_vs_streams"],
        "modes": results, "max_abs_err_vs_oracle": max_err, "cpu_baseline": cpu,
        "plan_host_us": plan_us,       # once per batch, reused by every layer; not part of `value`
    }
    if peaks:
        t_roof_meas = max(flops / (peaks["mfma_f16_TFLOPs"] * 1e12), kv_bytes / (peaks["hbm_read_GBps"] * 1e9)) * 1e6
        head["measured_peaks"] = peaks
        head["overlap_roofline_measured_peaks_us"] = t_roof_meas
        head["pct_of_overlap_roofline_measured_peaks"] = 100.0 * t_roof_meas / value_us
    attn.close()
    attn_base.close()
    return head


def run_colocation(steps, warmup, torch, pod):
    """Section 3.3's experiment on this GPU: 8192 compute items and 8192 memory items (c = a + b over
    1 GiB per array), the compute loop sized to take as long as the memory operation alone."""
    dev = "cuda:0"
    n_items, item_bytes = 8192, 128 << 10
    a = torch.ones(n_items * item_bytes // 4, dtype=torch.float32, device=dev)
    b = torch.full_like(a, 2.0)
    c = torch.zeros_like(a)
    ctr = torch.zeros(1026, dtype=torch.int32, device=dev)
    sink = torch.zeros(4, dtype=torch.float32, device=dev)
    side = torch.cuda.Stream(device=dev)

    def launch(variant, iters, n_mem=n_items, n_cmp=n_items, stream=None):
        st = (stream or torch.cuda.current_stream(dev)).cuda_stream
        pod.pod_attn_probe_colocation(variant, a.data_ptr(), b.data_ptr(), c.data_ptr(), item_bytes, n_mem, n_cmp,
                                      iters, ctr.data_ptr(), sink.data_ptr(), st)

    def timed(fn):
        for _ in range(warmup):
            fn()
        return float(np.median(event_times_us(fn, steps, torch)))

    t_mem = timed(lambda: launch(1, 0))
    iters = 2048
    t_cmp = timed(lambda: launch(0, iters))
    iters = max(64, int(iters * t_mem / t_cmp))
    t_cmp = timed(lambda: launch(0, iters))

    def two_streams():
        main = torch.cuda.current_stream(dev)
        side.wait_stream(main)
        launch(0, iters)
        launch(1, 0, stream=side)
        main.wait_stream(side)

    res = {"compute_alone": t_cmp, "memory_alone": t_mem,
           "serial": timed(lambda: (launch(0, iters), launch(1, 0))),
           "streams": timed(two_streams),
           "fused_by_index": timed(lambda: launch(2, iters)),
           "fused_bound_per_unit": timed(lambda: launch(3, iters))}
    torch.cuda.synchronize()
    ok = bool((c == 3.0).all())
    moved = 3 * n_items * item_bytes
    log("[colocation] " + ", ".join(f"{k} {v:.1f} us" for k, v in res.items()) + f"; c == a + b: {ok}")
    return {"metric": "co-location experiment (Section 3.3), us per run", "unit": "us", "n_gpus": 1, "steps": steps,
            "warmup": warmup, "data": "synthetic", "dtype": "f32",
            "config": {"workload": "colocation", "compute_items": n_items, "memory_items": n_items,
                       "bytes_moved": moved, "compute_iters": iters},
            "times_us": res, "memory_alone_GBps": moved / t_mem / 1e3, "result_ok": ok,
            "speedup_bound_vs_serial": res["serial"] / res["fused_bound_per_unit"],
            "speedup_by_index_vs_serial": res["serial"] / res["fused_by_index"]}


def run_chunk_series(model, n_decode, steps, warmup, torch, pod, wl):
    """Every chunk of a 16K prompt with the same decodes (the paper's Figure 6 / Table 8 workload):
    per chunk the median time of the fused launch, of the serial and two-stream baselines, and of
    two ablations of the fused launch (Section 5.4.2: the proportional policy as the paper states it,
    i.e. without this library's cap of one decode-first workgroup per unit, whose ratio is recorded;
    the 50:50 policy plans exactly what the automatic one plans whenever that one arrives at 1:1, which
    it does on every chunk here, so it is not timed a second time; Section 5.4: no cap on prefill splits)."""
    dev = "cuda:0"
    base = wl.series_base(model, n_decode, device=dev)
    n_chunks = wl.SERIES_PROMPT // wl.SERIES_CHUNK
    out = torch.empty((base.n_rows, base.n_q_heads, base.head_dim), dtype=base.torch_dtype, device=dev)
    rows = []
    for k in range(n_chunks):
        batch = wl.series_chunk(base, k)
        rec = {"chunk": k, "kv_len": int(batch.seq_meta[0, 2])}
        variants = {"fused": {}, "serial": {"max_prefill_waves": 2}, "streams": {"max_prefill_waves": 2},
                    "fused_proportional": {"policy": pod.POLICY_PROPORTIONAL},
                    "fused_uncapped": {"max_prefill_waves": 64}}
        plans = {}
        for name, kw in variants.items():
            key = tuple(sorted(kw.items()))
            if key not in plans:
                plans[key] = pod.HybridAttention(batch, **kw)
            attn = plans[key]
            mode = pod.MODES[name] if name in pod.MODES else pod.MODE_FUSED
            fn = lambda: attn.forward(batch, out=out, mode=mode)
            for _ in range(warmup):
                fn()
            t = event_times_us(fn, steps, torch)
            rec[name] = float(np.median(t))
            if name == "fused":
                rec["prefill_items"], rec["decode_units"] = attn.info.n_prefill_items, attn.info.n_decode_units
                rec["ratio"] = [attn.info.prefill_ratio, attn.info.decode_ratio]
            if name == "fused_proportional":
                rec["ratio_proportional"] = [attn.info.prefill_ratio, attn.info.decode_ratio]
        for attn in plans.values():
            attn.close()
        flops, kv_bytes = batch.prefill_flops(), batch.kv_bytes()
        rec["roofline_us"] = max(flops / PEAK_MFMA_16BIT, kv_bytes / PEAK_HBM) * 1e6
        rows.append(rec)
        log(f"[series] {model} d{n_decode} chunk {k:2d} kv {rec['kv_len']:5d}: fused {rec['fused']:7.1f} serial {rec['serial']:7.1f} "
            f"streams {rec['streams']:7.1f} | proportional {rec['ratio_proportional'][0]}:{rec['ratio_proportional'][1]} "
            f"{rec['fused_proportional']:7.1f} uncapped {rec['fused_uncapped']:7.1f} | "
            f"roofline {rec['roofline_us']:6.1f} us")
    tot = {k: float(sum(r[k] for r in rows)) for k in ("fused", "serial", "streams", "fused_proportional", "fused_uncapped", "roofline_us")}
    return {"metric": "hybrid-batch attention us per batch, summed over the 32 chunks of a 16K prompt",
            "unit": "us", "n_gpus": 1, "steps": steps, "warmup": warmup, "data": "synthetic", "dtype": "bf16",
            "config": {"workload": f"chunk-series-{model}", "chunk": wl.SERIES_CHUNK, "prompt": wl.SERIES_PROMPT,
                       "n_decode": n_decode, "decode_ctx": wl.SERIES_DECODE_CTX, "kv_layout": "paged16"},
            "totals_us": tot, "speedup_vs_serial": tot["serial"] / tot["fused"],
            "pct_of_overlap_roofline": 100.0 * tot["roofline_us"] / tot["fused"], "chunks": rows}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=4,
                    help="headline configuration 1..5 (default 4); 6 = the extra 256-channel shape")
    ap.add_argument("--no-configs", action="store_true",
                    help="time the headline batch only (no `configs` array with the other benchmark batches)")
    ap.add_argument("--batch-index", type=int, default=0, help="batch of the config-5 ratio sweep (0..11)")
    ap.add_argument("--mode", default="fused", choices=["fused", "serial", "streams", "fused_heavy"],
                    help="which schedule the headline value times (fused_heavy: the prefill-heavy configuration)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-peaks", action="store_true", help="skip the HBM-read and MFMA peak probes")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a 1 GiB device copy and the 4 GiB read probe (known sizes, for scaling "
                         "the FETCH_SIZE / WRITE_SIZE counters of a profiler run) and exit")
    ap.add_argument("--sweep", default=None, help="also write the whole record, indented, to this file")
    ap.add_argument("--chunk-series", default=None, choices=["yi-6b", "llama-3-8b"],
                    help="instead of a configuration, time every 512-token chunk of a 16K prompt, each with "
                         "--series-decodes decode requests at 16K context (fused, serial, two streams, and the "
                         "fused launch with the uncapped proportional policy and without the prefill split cap)")
    ap.add_argument("--colocation", action="store_true",
                    help="instead of a configuration, run the co-location experiment of the paper's Section 3.3: "
                         "a compute-bound and a memory-bound operation serially, on two streams, fused by "
                         "workgroup index and fused with per-compute-unit binding")
    ap.add_argument("--issue-probe", action="store_true",
                    help="instead of a configuration, time the instruction-mix probes (matrix instructions alone "
                         "and beside softmax-like vector work, one and two wavefronts per SIMD) and print a table")
    ap.add_argument("--trace-summary", action="store_true",
                    help="instead of timing, run one fused launch of --config with the library's workgroup trace "
                         "and event log switched on and print where and when the two operations ran (text)")
    ap.add_argument("--clock-by-mode", action="store_true",
                    help="instead of one timing, loop every schedule of --config for three seconds each while "
                         "reading the graphics clock with rocm-smi, then time each schedule again with idle gaps "
                         "between the launches (text): what the chip's clock management does to each schedule")
    ap.add_argument("--series-decodes", type=int, default=64)
    ap.add_argument("--series-out", default=None, help="write the chunk-series records to this file")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (one MI355X per box); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2410_18038_amd import pod
    from paper_2410_18038_amd import workloads as wl
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the attention path has no CPU fallback", file=sys.stderr)
        sys.exit(2)
    pod.lib()
    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0")
        src.zero_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        peaks = measure_peaks(torch, pod)
        print(json.dumps({"copy_bytes": 1 << 30, "copies": 3, "read_probe_bytes": 4 << 30, "peaks": peaks}))
        return

    if args.colocation:
        print(json.dumps(run_colocation(args.steps, args.warmup, torch, pod)), flush=True)
        return
    if args.issue_probe:
        sink = torch.zeros(4, dtype=torch.float32, device="cuda:0")
        print("instruction-mix probe: ns per matrix instruction (last two lines: per vector instruction), per wavefront "
              "and per SIMD (32x32x16 bf16; 32 cycles at full rate)")
        for variant, name in enumerate(pod.ISSUE_PROBE_VARIANTS):
            for w in (1, 2):
                n = [0.0]

                def go():
                    n[0] = pod.pod_attn_probe_issue(variant, 20000, w, sink.data_ptr(),
                                                    torch.cuda.current_stream().cuda_stream)
                go()
                t = float(np.min(event_times_us(go, 5, torch)))
                print(f"  {variant} {name:82s} {w} wavefront(s)/SIMD: {t * 1e3 / n[0]:6.2f} per wavefront, "
                      f"{t * 1e3 / n[0] / w:6.2f} per SIMD")
        return
    if args.trace_summary:
        from paper_2410_18038_amd import trace_report
        batch = wl.config_batch(args.config, args.batch_index, device="cuda:0")
        attn = pod.HybridAttention(batch)
        for _ in range(args.warmup):
            attn.forward(batch)
        attn.enable_trace()
        attn.enable_event_log()
        attn.forward(batch)
        rep = trace_report.colocation(attn.read_trace(), attn.read_event_log(), attn.info.n_prefill_items,
                                      attn.info.n_decode_units)
        print(trace_report.as_text(f"{batch.name} ({attn.info.n_prefill_items} prefill items, "
                                   f"{attn.info.n_decode_units} decode units, {attn.info.fused_grid} workgroups)", rep))
        attn.close()
        return
    if args.clock_by_mode:
        run_clock_by_mode(args.config, args.batch_index, torch, pod, wl)
        return
    if args.chunk_series:
        rec = run_chunk_series(args.chunk_series, args.series_decodes, args.steps, args.warmup, torch, pod, wl)
        if args.series_out:
            with open(args.series_out, "w") as fh:
                json.dump(rec, fh, indent=1)
        print(json.dumps(rec), flush=True)
        return

    peaks = None if args.no_peaks else measure_peaks(torch, pod)
    if peaks:
        log(f"[bench] measured peaks: HBM read {peaks['hbm_read_GBps']:.0f} GB/s, "
            f"fp16 MFMA {peaks['mfma_f16_TFLOPs']:.0f} TFLOP/s")
    rec = run_config(args.config, args.batch_index, args.steps, args.warmup, not args.no_cpu_baseline,
                     args.mode, torch, pod, wl, peaks)
    log("[bench] modes (us): " + json.dumps(rec["modes"]))
    if not args.no_configs:
        # every other benchmark batch, same clock, same checks (no CPU-baseline sample, no probes)
        todo = [(c, 0) for c in (2, 3, 4)] + [(5, i) for i in range(len(wl.RATIO_SWEEP))] + [(6, 0)]
        others = []
        for c, i in todo:
            if (c, i) == (args.config, args.batch_index):
                r = {k: rec[k] for k in ("overlap_roofline_us", "pct_of_overlap_roofline", "speedup_vs_serial",
                                         "speedup_vs_streams", "max_abs_err_vs_oracle")}
                r.update(workload=rec["config"]["workload"], config=c, batch_index=i,
                         fused_us=rec["modes"]["fused"]["wall_us"], serial_us=rec["modes"]["serial"]["wall_us"],
                         streams_us=rec["modes"]["streams"]["wall_us"],
                         fused_cta_parallel_us=rec["modes"]["fused_cta"]["wall_us"],
                         prefill_heavy_us=rec["modes"].get("fused_heavy", {}).get("wall_us"),
                         prefill_heavy_advised=rec["config"]["prefill_heavy_advised"],
                         frac=rec["pct_of_overlap_roofline"] / 100.0,
                         bound=rec["roofline"]["bound"], headline=True)
            else:
                torch.cuda.empty_cache()
                r = run_config(c, i, args.steps, args.warmup, False, "fused", torch, pod, wl, None, headline=False)
                r.pop("modes")
            heavy_txt = f"prefill-heavy {r['prefill_heavy_us']:.1f} us, " if r.get("prefill_heavy_us") else ""
            log(f"[bench] {r['workload']}: fused {r['fused_us']:.1f} us, serial {r['serial_us']:.1f} us, "
                f"streams {r['streams_us']:.1f} us, {heavy_txt}{r['pct_of_overlap_roofline']:.1f}% of overlap roofline, "
                f"x{r['speedup_vs_serial']:.3f} vs serial, max-abs err {r['max_abs_err_vs_oracle']:.1e}")
            others.append(r)
        rec["configs"] = others
        # the summary is over the benchmark configurations; the extra 256-channel shape is listed, not counted
        others = [r for r in others if r["config"] <= 5]
        pct = [r["pct_of_overlap_roofline"] for r in others]
        rec["configs_summary"] = {"n": len(others), "min_pct_of_overlap_roofline": min(pct),
                                  "mean_pct_of_overlap_roofline": float(np.mean(pct)),
                                  "n_at_or_above_70pct": int(sum(p >= 70.0 for p in pct)),
                                  "n_ahead_of_serial": int(sum(r["speedup_vs_serial"] > 1.0 for r in others)),
                                  "max_abs_err_vs_oracle": max(r["max_abs_err_vs_oracle"] for r in others)}
    if args.sweep:
        with open(args.sweep, "w") as fh:
            json.dump(rec, fh, indent=1)
    print(json.dumps(rec), flush=True)


if __name__ == "__main__":
    main()
