#!/usr/bin/env python3
"""Benchmark of the ADORE decode step on one MI355X.

A "step" is one pass of the whole hot path (insert + sparse attention, controller, release select,
rebuild select, re-projection GEMM + scatter) for one batch of B sequences of one decoder layer, in
steady state (cache full, R tokens rebuilt per sequence and step).  All inputs are generated from a
seed, uploaded, and resident in HBM before the timed region; the library is told so
(adore_set_input_order(0): its side stream need not wait for the caller's stream before it reads a
step's inputs).  The step with that wait in place (the library's default, for inputs produced by work
still queued on the stream) is timed as well and reported as "ordered_inputs".

Prints ONE JSON line: tokens/s per layer for the whole job, per-kernel times measured live with HIP
events on the library's stream, the roofline fraction of the dominant kernel, and the CPU oracle
timed on this host on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0           # MI355X HBM3E
MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}


INPUTS_ORDERED = False          # --input-order; see the module docstring


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def algorithmic_work(w):
    """Bytes / flops one step must move / compute, per kernel (not the dense work the method avoids)."""
    es = 2 if w.dtype == "bf16" else 4
    BH = w.B * w.H
    att_bytes = 2 * BH * w.K * w.d * es + BH * (w.K * 4 + 3 * w.d * es + w.d * 4)
    gemm_flops = 2.0 * (w.B * w.R) * w.D * (2 * w.H * w.d)
    ctrl_flops = 2.0 * w.B * w.D * 3 * w.dprime + 2.0 * w.B * w.dprime * 4 * w.dprime
    sel_bytes = BH * w.K * 8 + w.B * w.N_max * 4
    return dict(attend_bytes=att_bytes, gemm_flops=gemm_flops, ctrl_flops=ctrl_flops, select_bytes=sel_bytes)


def recorded_traffic(w, path_name="decode_step"):
    """HBM bytes per launch measured with rocprofv3 counters (FETCH_SIZE / WRITE_SIZE scaled by a copy
    kernel of known size); recorded in profiles/ because bench.py cannot run the profiler on itself."""
    path = os.path.join(ROOT, "profiles", f"{path_name}_{w.name}_hbm_traffic.txt")
    out = {}
    if os.path.exists(path):
        for line in open(path):
            parts = line.split()
            if len(parts) == 3 and parts[0] == "traffic_bytes":
                out[parts[1]] = int(parts[2])
    return out


def run_gpu(w, steps, warmup, prof_steps, ordered_steps=0):
    import torch
    from gen import SyntheticInputs
    from gen.gpu_job import GpuJob, to_dev
    t0 = time.time()
    inp = SyntheticInputs(w)
    job = GpuJob(w, inp, ordered=INPUTS_ORDERED)
    log(f"inputs generated and uploaded in {time.time() - t0:.1f}s")
    job.init()
    room = w.N_max - w.S - warmup - steps          # positions left for the untimed extras
    assert room >= 0, "not enough positions for this many steps"
    prof_steps = min(prof_steps, room)
    if ordered_steps > room - prof_steps:
        ordered_steps = 0
    total = warmup + steps + prof_steps + ordered_steps
    assert w.S + total <= w.N_max, "not enough positions for this many steps"
    qkv = []
    for t in range(total):
        q, k, v = inp.step_qkv(w.S + t)
        qkv.append(tuple(to_dev(a[0], job.st) for a in (q, k, v)))
    xs = [job.hidden[0][:, w.S + t].contiguous() for t in range(total)]
    hidden0 = job.hidden[0]
    out = job.out[0]
    torch.cuda.synchronize()

    def step(t):
        q, k, v = qkv[t]
        job.adore.decode_step(q, k, v, hidden0, xs[t], None, out, job.slot_map)

    for t in range(warmup):
        step(t)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for t in range(warmup, warmup + steps):
        step(t)
    host = time.perf_counter() - t1             # the host's share: all launches enqueued
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t1
    log(f"host enqueue {1e6 * host / steps:.1f} us per step, step {1e6 * elapsed / steps:.1f} us")

    # per-kernel durations, HIP events on the library's stream around every launch
    job.adore.set_timing(True)
    for t in range(warmup + steps, warmup + steps + prof_steps):
        step(t)
    timing = job.adore.read_timing()
    job.adore.set_timing(False)
    per_kernel_us = {k: (1e3 * ms / cnt if cnt else 0.0) for k, (ms, cnt) in timing.items()}

    # the same step in the other input order
    other = None
    if ordered_steps > warmup:
        job.adore.set_input_order(not INPUTS_ORDERED)
        t0 = warmup + steps + prof_steps
        for t in range(t0, t0 + warmup):
            step(t)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for t in range(t0 + warmup, total):
            step(t)
        torch.cuda.synchronize()
        other = (time.perf_counter() - t1) / (ordered_steps - warmup)
        log(f"step with input order {'off' if INPUTS_ORDERED else 'on'}: {1e6 * other:.1f} us")
    assert bool(torch.isfinite(out).all())
    job.adore.close()
    return elapsed, per_kernel_us, other


def run_gpu_device_inputs(w, steps, warmup, prof_steps):
    """A single-layer workload through adore_decode_step with its large tensors drawn on the device (seeded torch
    generator; the host generator of the parity tests takes minutes at these sizes).  Inputs complete in memory
    before every call.  Returns (seconds for `steps` steps, microseconds per launch and kernel)."""
    import torch
    from gen import DeviceNormals, SyntheticInputs
    from gen.gpu_job import DEV, storage_dtype, to_dev
    from paper_2407_02328_amd import Adore, make_config
    st = storage_dtype(w)
    total = warmup + steps + prof_steps
    w = w.scaled(T=max(w.T, total))
    drawer = DeviceNormals(w.seed, DEV)
    small = SyntheticInputs(w.scaled(L=1, H=1, d=64, B=1)).weights()    # controller tensors do not depend on L, H, d, B
    wts = {k: to_dev(v, st if k in ("gru_w_ih", "gru_w_hh") else torch.float32) for k, v in small.items() if k != "w_kv"}
    wts["w_kv"] = drawer.normal((1, 2 * w.H * w.d, w.D), w.w_std, st)
    hidden = drawer.normal((1, w.B, w.N_max, w.D), w.act_std, st)
    prompt_k = drawer.normal((1, w.B, w.H, w.S, w.d), w.act_std, st)
    prompt_v = drawer.normal((1, w.B, w.H, w.S, w.d), w.act_std, st)
    q, k, v = (drawer.normal((w.B, w.H, w.d), w.act_std, st) for _ in range(3))
    out = torch.empty((w.B, w.H, w.d), dtype=torch.float32, device=DEV)
    slot_map = torch.empty((w.B, w.H, w.K), dtype=torch.int32, device=DEV)
    cfg = make_config(layers=1, batch=w.B, heads=w.H, head_dim=w.d, hidden=w.D, cache_slots=w.K, rebuild_budget=w.R,
                      max_positions=w.N_max, ctrl_hidden=w.dprime, dtype=w.dtype, pos_scale=w.pos_scale,
                      score_mode=2 if w.h2o else 1 if w.rescore else 0, rope_base=w.rope_base)
    a = Adore(cfg, wts, DEV)
    a.set_input_order(INPUTS_ORDERED)
    a.init_cache(prompt_k, prompt_v, hidden, hidden[0][:, :w.S].contiguous(), None, w.S)
    xs = [hidden[0][:, w.S + t].contiguous() for t in range(total)]
    torch.cuda.synchronize()

    def step(t):
        a.decode_step(q, k, v, hidden[0], xs[t], None, out, slot_map)

    for t in range(warmup):
        step(t)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for t in range(warmup, warmup + steps):
        step(t)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t1
    a.set_timing(True)
    for t in range(warmup + steps, total):
        step(t)
    timing = a.read_timing()
    a.set_timing(False)
    assert bool(torch.isfinite(out).all())
    a.close()
    return elapsed, {kk: (1e3 * ms / cnt if cnt else 0.0) for kk, (ms, cnt) in timing.items()}


def other_workload_entry(name, steps=150, warmup=30, prof_steps=30):
    """Compact record of another single-layer workload for the default line: step time, the attention launch against
    the HBM peak and the GEMM against the MFMA peak (or, where M is too small for that, against what streaming W costs)."""
    from gen import workload
    w = workload(name)
    elapsed, us = run_gpu_device_inputs(w, steps, warmup, prof_steps)
    work = algorithmic_work(w)
    att = us["attend"] + us["attend_combine"]
    gemm = us["rebuild_gemm"]
    entry = {"workload": name, "batch": w.B, "cache_slots_K": w.K, "rebuild_budget_R": w.R, "prompt": w.S,
             "ms_per_step": round(1e3 * elapsed / steps, 4), "tokens_per_s_per_layer": round(w.B * steps / elapsed, 1),
             "attend_us": round(att, 2), "attend_algorithmic_bytes": work["attend_bytes"],
             "attend_GBs": round(work["attend_bytes"] / (att * 1e-6) / 1e9, 1),
             "attend_frac_of_hbm_peak": round(work["attend_bytes"] / (att * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
             "rebuild_gemm_us": round(gemm, 2), "rebuild_gemm_TFLOPs": round(work["gemm_flops"] / (gemm * 1e-6) / 1e12, 1),
             "rebuild_gemm_frac_of_mfma_peak": round(work["gemm_flops"] / (gemm * 1e-6) / 1e12 / MFMA_PEAK_TFLOPS["bf16"], 4),
             "inputs": "drawn on the device (seeded)"}
    if w.B * w.R < 400:     # below the ridge the GEMM streams W: priced against HBM as well
        wbytes = 2.0 * w.H * w.d * w.D * 2
        entry["rebuild_gemm_weight_stream_frac_of_hbm_peak"] = round(wbytes / (gemm * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)
    return entry


def stack_workload_entry(steps=24, warmup=6, prof_steps=6):
    """Compact record of the 32-layer stack for the default line: per-layer step time through the fine-grained calls
    and the throughput ratio against the full-attention comparator of Eq. 1 on the same shapes (see run_stack)."""
    from gen import workload
    w = workload("stack32")
    w = w.scaled(T=warmup + steps + prof_steps)
    el_s, us_s, el_f, us_f = run_stack(w, steps, warmup, prof_steps)
    work = algorithmic_work(w)
    att = us_s["attend"] + us_s["attend_combine"]
    n_mid = w.S + warmup + steps // 2
    return {"workload": "stack32", "layers": w.L, "batch": w.B, "cache_slots_K": w.K, "rebuild_budget_R": w.R, "prompt": w.S,
            "ms_per_step_all_layers": round(1e3 * el_s / steps, 4), "ms_per_step": round(1e3 * el_s / steps / w.L, 4),
            "tokens_per_s_per_layer": round(w.B * w.L * steps / el_s, 1),
            "attend_us": round(att, 2), "attend_GBs": round(work["attend_bytes"] / (att * 1e-6) / 1e9, 1),
            "attend_frac_of_hbm_peak": round(work["attend_bytes"] / (att * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
            "rebuild_gemm_us": round(us_s["rebuild_gemm"], 2),
            "rebuild_gemm_TFLOPs": round(work["gemm_flops"] / (us_s["rebuild_gemm"] * 1e-6) / 1e12, 1),
            "rebuild_gemm_frac_of_mfma_peak": round(work["gemm_flops"] / (us_s["rebuild_gemm"] * 1e-6) / 1e12 / MFMA_PEAK_TFLOPS["bf16"], 4),
            "full_attention_ms_per_step_all_layers": round(1e3 * el_f / steps, 4),
            "full_attention_rows_per_head": n_mid + 1,
            "sparse_vs_full_throughput": round(el_f / el_s, 3),
            "inputs": "drawn on the device (seeded)"}


def run_stack(w, steps, warmup, prof_steps):
    """Layer-stack workload: every step runs attend x L, one schedule, rebuild x L through the fine-grained
    calls, layers launched one after the other.  Next to it the full-attention comparator of Eq. 1: the
    same attention kernel over a cache with room for every token (K_full - 1 >= N_max, nothing released,
    nothing rebuilt), which reads n+1 rows per (sequence, head) instead of K.

    The large tensors (W_kv, hidden states, prompt K/V) are drawn on the device from a seeded torch
    generator: tens of GB, which the host generator of the parity tests would take minutes to produce;
    the small controller weights come from that generator as everywhere else."""
    import torch
    from gen import SyntheticInputs
    from paper_2407_02328_amd import Adore, make_config
    from gen.gpu_job import DEV, storage_dtype, to_dev
    st = storage_dtype(w)
    total = warmup + steps + prof_steps
    assert w.S + total <= w.N_max, "not enough positions for this many steps"
    from gen import DeviceNormals
    drawer = DeviceNormals(w.seed, DEV)

    def randn(shape, std=1.0):
        return drawer.normal(shape, std, st)

    t0 = time.time()
    dp = w.dprime
    small = SyntheticInputs(w.scaled(L=1, H=1, d=64, B=1)).weights()    # controller tensors do not depend on L, H, d, B
    wts = {k: to_dev(v, st if k in ("gru_w_ih", "gru_w_hh") else torch.float32) for k, v in small.items() if k != "w_kv"}
    wts["w_kv"] = randn((w.L, 2 * w.H * w.d, w.D), w.w_std)
    hidden = randn((w.L, w.B, w.N_max, w.D))
    q = randn((w.L, w.B, w.H, w.d)); k = randn((w.L, w.B, w.H, w.d)); v = randn((w.L, w.B, w.H, w.d))
    out = torch.empty((w.L, w.B, w.H, w.d), dtype=torch.float32, device=DEV)
    prompt_k = randn((w.L, w.B, w.H, w.S, w.d)); prompt_v = randn((w.L, w.B, w.H, w.S, w.d))
    ctrl_in = hidden[0][:, :w.S].contiguous()
    xs = [hidden[0][:, w.S + t].contiguous() for t in range(total)]
    torch.cuda.synchronize()
    log(f"stack inputs drawn on the device in {time.time() - t0:.1f}s")

    def make(K, R):
        cfg = make_config(layers=w.L, batch=w.B, heads=w.H, head_dim=w.d, hidden=w.D, cache_slots=K,
                          rebuild_budget=R, max_positions=w.N_max, ctrl_hidden=dp, dtype=w.dtype,
                          pos_scale=w.pos_scale, rope_base=w.rope_base)
        a = Adore(cfg, wts, DEV)
        a.set_input_order(INPUTS_ORDERED)
        a.init_cache(prompt_k, prompt_v, hidden, ctrl_in, None, w.S)
        torch.cuda.synchronize()
        return a

    def timed(a, with_rebuild):
        def step(t):
            for l in range(w.L):
                a.attend(l, q[l], k[l], v[l], out[l])
            a.schedule(xs[t], None, None, None, None)
            for l in range(w.L):
                a.rebuild(l, hidden[l])
        for t in range(warmup):
            step(t)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for t in range(warmup, warmup + steps):
            step(t)
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t1
        a.set_timing(True)
        for t in range(warmup + steps, total):
            step(t)
        timing = a.read_timing()
        a.set_timing(False)
        assert bool(torch.isfinite(out).all())
        # per launch: a step launches attend and the GEMM once per layer
        return elapsed, {kk: (1e3 * ms / cnt if cnt else 0.0) for kk, (ms, cnt) in timing.items()}

    sparse = make(w.K, w.R)
    el_s, us_s = timed(sparse, True)
    sparse.close()
    del sparse
    torch.cuda.empty_cache()
    full = make(w.N_max + 1, 0)            # m = K - 0 - 1 = N_max: every token stays
    el_f, us_f = timed(full, False)
    full.close()
    return el_s, us_s, el_f, us_f


def run_forward(w, steps, warmup, prof_steps):
    """Rebuild forward through the layer stack: every step is one adore_forward_step (per layer: q/k/v
    projection of the R+1 rows of every sequence with scatter into the cache, attention of the R+1 rows,
    output projection with residual; once per step: controller and the two selections).  Large tensors
    are drawn on the device from a seeded torch generator, as in run_stack."""
    import torch
    from gen import SyntheticInputs
    from paper_2407_02328_amd import Adore, make_config
    from gen.gpu_job import DEV, storage_dtype, to_dev
    st = storage_dtype(w)
    total = warmup + steps + prof_steps
    assert w.S + total <= w.N_max, "not enough positions for this many steps"
    g = torch.Generator(device=DEV)
    g.manual_seed(w.seed)

    def randn(shape, std=1.0):
        return (torch.randn(shape, generator=g, device=DEV, dtype=torch.float32) * std).to(st)

    Hd = w.H * w.d
    small = SyntheticInputs(w.scaled(L=1, H=1, d=64, B=1)).weights()
    wts = {k: to_dev(v, st if k in ("gru_w_ih", "gru_w_hh") else torch.float32) for k, v in small.items() if k != "w_kv"}
    wts["w_kv"] = randn((w.L, 2 * Hd, w.D), w.w_std)
    w_q, w_o = randn((w.L, Hd, w.D), w.w_std), randn((w.L, w.D, Hd), w.w_std)
    embed = randn((w.B, w.N_max, w.D))
    prompt_k = randn((w.L, w.B, w.H, w.S, w.d)); prompt_v = randn((w.L, w.B, w.H, w.S, w.d))
    cfg = make_config(layers=w.L, batch=w.B, heads=w.H, head_dim=w.d, hidden=w.D, cache_slots=w.K,
                      rebuild_budget=w.R, max_positions=w.N_max, ctrl_hidden=w.dprime, dtype=w.dtype,
                      pos_scale=w.pos_scale, rope_base=w.rope_base)
    a = Adore(cfg, wts, DEV)
    a.set_input_order(INPUTS_ORDERED)
    a.init_cache(prompt_k, prompt_v, None, embed[:, :w.S].contiguous(), None, w.S)
    rows = torch.zeros((w.B, w.R + 1, w.D), dtype=st, device=DEV)
    torch.cuda.synchronize()
    for t in range(warmup):
        a.forward_step(w_q, w_o, embed, None, rows)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for t in range(steps):
        a.forward_step(w_q, w_o, embed, None, rows)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t1
    a.set_timing(True)
    for t in range(prof_steps):
        a.forward_step(w_q, w_o, embed, None, rows)
    timing = a.read_timing()
    a.set_timing(False)
    assert bool(torch.isfinite(rows.float()).all())
    a.close()
    return elapsed, {k: (1e3 * ms / cnt if cnt else 0.0) for k, (ms, cnt) in timing.items()}


def forward_line(w, args):
    """JSON line of the rebuild-forward workload (tokens/s per layer = B * L * steps / elapsed)."""
    elapsed, us = run_forward(w, args.steps, args.warmup, args.profile_steps)
    es, BH, Hd, M = 2, w.B * w.H, w.H * w.d, w.B * (w.R + 1)
    att_bytes = 2 * BH * w.K * w.d * es + BH * w.K * 4 + 2 * M * Hd * es
    qkv_flops, o_flops = 2.0 * M * w.D * 3 * Hd, 2.0 * M * Hd * w.D
    traffic = recorded_traffic(w, "forward_step")      # per projection: tile kernel + skinny kernel together
    roof = lambda name, work, t, peak, unit, scale, bound: dict(
        kernel=name, bound=bound, achieved=round(work / (t * 1e-6) / scale, 1) if t else 0.0, peak=peak, unit=unit,
        frac=round(work / (t * 1e-6) / scale / peak, 4) if t else 0.0, traffic=traffic.get(name.split("+")[0]),
        us_per_launch=round(t, 2))
    roofs = {"roofline_fwd_attend": roof("fwd_attend", att_bytes, us["fwd_attend"], HBM_PEAK_GBS, "GB/s", 1e9, "hbm"),
             # each projection = the tile kernel (rebuilt tokens' rows) + the skinny kernel (current tokens' rows)
             "roofline_fwd_qkv": roof("fwd_qkv+fwd_qkv_cur", qkv_flops, us["fwd_qkv"] + us["fwd_qkv_cur"],
                                      MFMA_PEAK_TFLOPS["bf16"], "TFLOP/s", 1e12, "mfma"),
             "roofline_fwd_oproj": roof("fwd_oproj+fwd_oproj_cur", o_flops, us["fwd_oproj"] + us["fwd_oproj_cur"],
                                        MFMA_PEAK_TFLOPS["bf16"], "TFLOP/s", 1e12, "mfma")}
    dominant = max(roofs.values(), key=lambda r: r["us_per_launch"])
    return {
        "metric": "decoded tokens/sec per decode layer at cache K", "value": round(w.B * w.L * args.steps / elapsed, 1),
        "unit": "tokens/s/layer", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(1e3 * elapsed / args.steps / w.L, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name + "_forward", "batch": w.B, "heads": w.H, "head_dim": w.d, "hidden": w.D,
                   "cache_slots_K": w.K, "rebuild_budget_R": w.R, "prompt": w.S, "layers": w.L,
                   "path": "rebuild forward: R+1 query rows through every layer"},
        "roofline": dominant, **roofs,
        "kernel_us": {k: round(v, 2) for k, v in us.items()},
        "ms_per_step_all_layers": round(1e3 * elapsed / args.steps, 4),
    }


def prefill_line(w, args):
    """JSON line of the prompt side: adore_init_cache over the workload's S-token prompt (controller over every
    prompt token: input projection, recurrence, scoring; choice and fill of the residents; first rebuild)."""
    import torch
    from gen import SyntheticInputs
    from gen.gpu_job import GpuJob, to_dev
    inp = SyntheticInputs(w)
    job = GpuJob(w, inp)
    pk, pv = (to_dev(a, job.st) for a in job.prompt_np)
    ctrl_in = job.hidden[0][:, :w.S].contiguous()
    reps, warm = max(3, min(args.steps, 20)), 2
    torch.cuda.synchronize()
    for _ in range(warm):
        job.adore.init_cache(pk, pv, job.hidden, ctrl_in, None, w.S)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(reps):
        job.adore.init_cache(pk, pv, job.hidden, ctrl_in, None, w.S)
    torch.cuda.synchronize()
    elapsed = (time.perf_counter() - t1) / reps
    job.adore.set_timing(True)
    job.adore.init_cache(pk, pv, job.hidden, ctrl_in, None, w.S)
    timing = job.adore.read_timing()
    job.adore.set_timing(False)
    us = {k: 1e3 * ms for k, (ms, cnt) in timing.items() if cnt}      # per init: all launches of a kernel together
    scores = job.snapshot()["scores"][:, :w.S]
    assert np.isfinite(scores).all()
    job.adore.close()
    # the recurrence: 2 * 3d' * d' flops per token, one sequence per workgroup, tokens one after the other
    cell_flops = 2.0 * w.B * w.S * (3 * w.dprime * w.dprime + w.dprime * w.dprime)
    in_flops = 2.0 * w.B * w.S * w.D * 3 * w.dprime
    roof_cell = dict(kernel="ctrl_cell", bound="alu", achieved=round(cell_flops / (us["ctrl_cell"] * 1e-6) / 1e12, 3),
                     peak=MFMA_PEAK_TFLOPS["f32"], unit="TFLOP/s",
                     frac=round(cell_flops / (us["ctrl_cell"] * 1e-6) / 1e12 / MFMA_PEAK_TFLOPS["f32"], 5),
                     traffic=None, us_per_launch=round(us["ctrl_cell"], 1),
                     note="a recurrence: one workgroup per sequence, so at most B of the 256 compute units work on it")
    roof_in = dict(kernel="ctrl_input", bound="mfma", achieved=round(in_flops / (us["ctrl_input"] * 1e-6) / 1e12, 1),
                   peak=MFMA_PEAK_TFLOPS.get(w.dtype, 157.3), unit="TFLOP/s",
                   frac=round(in_flops / (us["ctrl_input"] * 1e-6) / 1e12 / MFMA_PEAK_TFLOPS.get(w.dtype, 157.3), 4),
                   traffic=None, us_per_launch=round(us["ctrl_input"], 1))
    return {
        "metric": "prompt tokens/sec through cache initialisation", "value": round(w.B * w.S / elapsed, 1),
        "unit": "tokens/s", "n_gpus": 1, "steps": reps, "warmup": warm, "ms_per_step": round(1e3 * elapsed, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name + "_prefill", "batch": w.B, "heads": w.H, "head_dim": w.d, "hidden": w.D,
                   "cache_slots_K": w.K, "rebuild_budget_R": w.R, "prompt": w.S, "layers": w.L,
                   "path": "adore_init_cache: controller over the prompt, residents chosen and filled, first rebuild"},
        "roofline": roof_cell if us["ctrl_cell"] >= us["ctrl_input"] else roof_in,
        "roofline_ctrl_cell": roof_cell, "roofline_ctrl_input": roof_in,
        "kernel_us": {k: round(v, 1) for k, v in us.items()},
    }


def topk_line(w, args):
    """JSON line of the top-K attention over the workload's prompts (adore_topk_attention: B * H rows of S tokens,
    K = args.topk): one call per step; the duration comes from HIP events on the stream the call enqueues on."""
    import torch
    from gen import DeviceNormals
    from paper_2407_02328_amd import topk_attention, load_library
    dev = "cuda:0"
    rows, S, d, K = w.B * w.H, w.S, w.d, args.topk
    if S > 32768 or d not in (64, 128):
        sys.exit(f"adore_topk_attention takes sequences up to 32768 tokens and head_dim 64 or 128 (asked: {S}, {d})")
    drawer = DeviceNormals(w.seed, dev)
    q, k, v = (drawer.normal((rows, S, d), 1.0, torch.bfloat16) for _ in range(3))
    out = torch.empty_like(q)
    ws = torch.empty(load_library().adore_topk_attention_workspace_bytes(rows, S, d), dtype=torch.uint8, device=dev)
    reps, warm = max(3, min(args.steps, 50)), 3
    for _ in range(warm):
        topk_attention(q, k, v, K, out=out, workspace=ws)
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]      # the call enqueues on torch's current stream
    t1 = time.perf_counter()
    ev[0].record()
    for _ in range(reps):
        topk_attention(q, k, v, K, out=out, workspace=ws)
    ev[1].record()
    torch.cuda.synchronize()
    elapsed = (time.perf_counter() - t1) / reps
    us = 1e3 * ev[0].elapsed_time(ev[1]) / reps
    assert bool(torch.isfinite(out.float()).all())
    # what the method has to compute: every weight of the causal triangle, and the kept probabilities times V
    kept = sum(min(i + 1, K) for i in range(S))
    flops = 2.0 * rows * d * (S * (S + 1) / 2 + kept)
    roof = dict(kernel="topk_attention (transpose of V + attention)", bound="mfma",
                achieved=round(flops / (us * 1e-6) / 1e12, 1), peak=MFMA_PEAK_TFLOPS["bf16"], unit="TFLOP/s",
                frac=round(flops / (us * 1e-6) / 1e12 / MFMA_PEAK_TFLOPS["bf16"], 4),
                traffic=(recorded_traffic(w, "topk_attention").get("topk_attention") if K == 96 else None),
                us_per_launch=round(us, 1), algorithmic_flops=flops,
                note="the selection (a four-pass radix select per query: LDS histograms, wave scans) runs beside the matrix work")
    line = {
        "metric": "prompt tokens/sec through top-K attention (one layer)", "value": round(w.B * S / elapsed, 1),
        "unit": "tokens/s", "n_gpus": 1, "steps": reps, "warmup": warm, "ms_per_step": round(1e3 * elapsed, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name + "_topk_attention", "batch": w.B, "heads": w.H, "head_dim": d, "prompt": S,
                   "top_k": K, "path": "adore_topk_attention: causal attention, every query keeps its K largest weights"},
        "roofline": roof,
    }
    if not args.no_cpu_baseline:
        from oracle import adore_oracle as O
        from threadpoolctl import threadpool_info
        sample = min(rows, 256)
        qs, ks, vs = (t[:sample].float().cpu().numpy().astype(np.float64) for t in (q, k, v))
        t0 = time.perf_counter()
        O.topk_attention(qs, ks, vs, K)
        dt = time.perf_counter() - t0
        cores = max([int(i.get("num_threads", 1)) for i in threadpool_info()] + [1])
        line["cpu_baseline"] = {"value": round(sample * S / w.H / dt, 2), "unit": "tokens/s", "cores": cores,
                                "kind": "oracle", "seconds": round(dt, 2),
                                "sample": f"{sample} of the {rows} rows (one head of one sequence each), all {S} queries "
                                          f"(numpy fp64, a Python loop over the queries); scaled to whole sequences of {w.H} heads"}
    return line


def other_path_entries(w):
    """The library's other paths at the same workload, compactly, for the default line: the rebuild forward through
    four layers, the cache initialisation over the prompts, the top-K attention over the prompts, the decode step in
    the H2O score mode.  Each is the measurement of its own flag (--forward, --prefill, --topk-attention, --h2o) with
    fewer steps and no oracle sample."""
    import argparse
    quick = argparse.Namespace(steps=60, warmup=10, profile_steps=20, topk=96, no_cpu_baseline=True)
    fw = forward_line(w.scaled(L=4), quick)
    pf = prefill_line(w, quick)
    tk = topk_line(w, quick)
    wh = w.scaled(h2o=True)
    el, us, _ = run_gpu(wh, 100, 20, 30)
    pick = lambda d, keys: {k: d[k] for k in keys if k in d}
    return [
        {"path": "rebuild forward (adore_forward_step), 4 layers", "ms_per_step_per_layer": fw["ms_per_step"],
         "tokens_per_s_per_layer": fw["value"],
         "kernel_us": pick(fw["kernel_us"], ("fwd_qkv", "fwd_attend", "fwd_oproj")),
         "fwd_attend_frac_of_hbm_peak": fw["roofline_fwd_attend"]["frac"],
         "fwd_qkv_frac_of_mfma_peak": fw["roofline_fwd_qkv"]["frac"],
         "fwd_oproj_frac_of_mfma_peak": fw["roofline_fwd_oproj"]["frac"]},
        {"path": "cache initialisation over the prompts (adore_init_cache)", "ms_per_init": pf["ms_per_step"],
         "prompt_tokens_per_s": pf["value"], "kernel_us": pf["kernel_us"]},
        {"path": "top-K attention over the prompts (adore_topk_attention, K = 96)", "ms_per_call": tk["ms_per_step"],
         "prompt_tokens_per_s": tk["value"], "frac_of_mfma_peak": tk["roofline"]["frac"]},
        {"path": "decode step with H2O scores (score_mode = h2o)", "ms_per_step": round(1e3 * el / 100, 4),
         "tokens_per_s_per_layer": round(wh.B * 100 / el, 1),
         "kernel_us": {k: round(v, 2) for k, v in us.items() if v and k in
                       ("attend", "h2o_release", "h2o_choice", "h2o_place", "rebuild_gemm")}},
    ]


def run_cpu_baseline(w, seqs=16, steps=40, single_thread_steps=8):
    """The oracle as it stands, on `seqs` sequences of the same workload, steady-state steps: once with the
    threads numpy's BLAS takes by itself, once (fewer steps) limited to one thread; per-stage seconds from timers
    wrapped around the oracle's functions (attention rows, controller, the two selections, re-projection + placement)."""
    from collections import defaultdict
    from threadpoolctl import threadpool_info, threadpool_limits
    import oracle.adore_oracle as O
    from tests.helpers import make_oracle
    seqs = min(seqs, w.B)
    ws = w.scaled(B=seqs, T=steps + single_thread_steps + 1)
    orc, inp, _ = make_oracle(ws)
    hs = inp.hidden_store()
    pk, pv = inp.prompt_kv()
    rng = np.random.default_rng(ws.seed)
    prompt_scores = rng.random((ws.B, ws.S), dtype=np.float32)     # skip nothing: init still runs the GRU
    orc.init_cache(pk, pv, hs, hs[0][:, :ws.S], ws.S, score_override=prompt_scores)
    qkvs = [inp.step_qkv(ws.S + t) for t in range(steps + single_thread_steps)]
    stage = defaultdict(float)

    def timed(name, fn):
        def wrapper(*a, **k):
            t = time.perf_counter()
            r = fn(*a, **k)
            stage[name] += time.perf_counter() - t
            return r
        return wrapper

    saved = (O.attention_row, O.release_lowest, O.rebuild_choice)
    O.attention_row = timed("attention", O.attention_row)
    O.release_lowest = timed("release_select", O.release_lowest)
    O.rebuild_choice = timed("rebuild_select", O.rebuild_choice)
    orc._controller = timed("controller", orc._controller)
    orc._place_rebuilt = timed("rebuild_projection_and_placement", orc._place_rebuilt)
    try:
        t0 = time.perf_counter()
        for t in range(steps):
            orc.decode_step(*qkvs[t], hs, hs[0][:, ws.S + t])
        dt = time.perf_counter() - t0
        per_stage = {k: round(v, 3) for k, v in stage.items()}
        per_stage["insert_and_bookkeeping"] = round(dt - sum(stage.values()), 3)
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        with threadpool_limits(limits=1):
            t0 = time.perf_counter()
            for t in range(steps, steps + single_thread_steps):
                orc.decode_step(*qkvs[t], hs, hs[0][:, ws.S + t])
            dt1 = time.perf_counter() - t0
    finally:
        O.attention_row, O.release_lowest, O.rebuild_choice = saved
    return dict(value=seqs * steps / dt, unit="tokens/s/layer", cores=int(threads), kind="oracle",
                sample=f"{seqs} of {w.B} sequences, {steps} steady-state steps after a {ws.S}-token prompt "
                       f"(numpy fp64; BLAS threads for the re-projection, Python loops elsewhere)",
                seconds=round(dt, 2), stage_seconds=per_stage,
                single_thread=dict(value=round(seqs * single_thread_steps / dt1, 2), unit="tokens/s/layer", cores=1,
                                   sample=f"the next {single_thread_steps} steps with every thread pool limited to one thread",
                                   seconds=round(dt1, 2)))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--profile-steps", type=int, default=50, help="extra steps with per-kernel events")
    ap.add_argument("--workload", default="llama7b_layer")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--rescore", action="store_true",
                    help="controller scores every token again at every step (relative position)")
    ap.add_argument("--h2o", action="store_true",
                    help="H2O(Rebuilt) score mode: per-head cumulative attention instead of the controller")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="leave the compact high_batch / long_context records out of the default line")
    ap.add_argument("--rope-base", type=float, default=0.0,
                    help="rotary position embedding with this base on the keys (and forward queries) the library makes")
    ap.add_argument("--topk-attention", action="store_true",
                    help="time adore_topk_attention over the workload's prompts (B * H rows of S tokens)")
    ap.add_argument("--topk", type=int, default=96, help="K of --topk-attention (the paper fine-tunes with 96)")
    ap.add_argument("--forward", type=int, default=0, metavar="LAYERS",
                    help="time the rebuild forward (adore_forward_step) through this many layers of the workload's shape")
    ap.add_argument("--input-order", choices=["ready", "stream"], default="ready",
                    help="ready: inputs are complete in memory at every call (they are, here); stream: the library "
                         "orders its side stream behind the caller's stream at every step (its default)")
    ap.add_argument("--prefill", action="store_true",
                    help="time adore_init_cache over the workload's prompt instead of decode steps")
    args = ap.parse_args()
    global INPUTS_ORDERED
    INPUTS_ORDERED = args.input_order == "stream"
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: this build has no multi-GPU path (the decode step shards by "
                 "sequence or by head with no exchange step). Run with --gpus 1.")
    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU (the HIP path has no CPU fallback)")
    from gen import workload
    w = workload(args.workload)
    if args.rescore:
        w = w.scaled(rescore=True)
    if args.rope_base:
        w = w.scaled(rope_base=args.rope_base)
    if args.h2o:
        w = w.scaled(h2o=True)
    if args.forward:
        print(json.dumps(forward_line(w.scaled(L=args.forward), args)), flush=True)
        return
    if args.prefill:
        print(json.dumps(prefill_line(w, args)), flush=True)
        return
    if args.topk_attention:
        print(json.dumps(topk_line(w, args)), flush=True)
        return
    work = algorithmic_work(w)
    stack = None
    if w.L != 1:
        elapsed, per_kernel_us, el_full, us_full = run_stack(w, args.steps, args.warmup, args.profile_steps)
        n_mid = w.S + args.warmup + args.steps // 2
        full_bytes = 4 * w.B * w.H * (n_mid + 1) * w.d * (2 if w.dtype == "bf16" else 4) // 2
        stack = {"layers": w.L, "ms_per_step_all_layers": round(1e3 * elapsed / args.steps, 4),
                 "full_attention_ms_per_step_all_layers": round(1e3 * el_full / args.steps, 4),
                 "sparse_vs_full_throughput": round(el_full / elapsed, 3),
                 "full_attention_attend_us": round(us_full["attend"] + us_full["attend_combine"], 2),
                 "full_attention_attend_GBs": round(full_bytes / ((us_full["attend"] + us_full["attend_combine"]) * 1e-6) / 1e9, 1),
                 "full_attention_rows_per_head": n_mid + 1}
        elapsed /= w.L                       # the metric is per decode layer
        args.no_cpu_baseline = True          # the oracle sample is defined on the single-layer workloads
    else:
        extra = args.profile_steps + args.warmup + args.steps // 2
        if args.warmup + args.steps + extra > w.T:
            # a longer run than the workload's T decode steps: more positions (the shapes stay; the riding
            # selections keep a sequence's scores in LDS, which bounds the positions at about 4400)
            w = w.scaled(T=max(w.T, min(args.warmup + args.steps + extra, 4400 - w.S)))
        elapsed, per_kernel_us, other = run_gpu(w, args.steps, args.warmup, args.profile_steps,
                                                ordered_steps=args.warmup + args.steps // 2)
    ms_per_step = 1e3 * elapsed / args.steps
    value = w.B * args.steps / elapsed

    att_us = per_kernel_us["attend"]
    gemm_us = per_kernel_us["rebuild_gemm"]
    att_gbs = work["attend_bytes"] / (att_us * 1e-6) / 1e9 if att_us else 0.0
    gemm_tflops = work["gemm_flops"] / (gemm_us * 1e-6) / 1e12 if gemm_us else 0.0
    traffic = recorded_traffic(w)
    roof_att = dict(kernel="attend", bound="hbm", achieved=round(att_gbs, 1), peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=round(att_gbs / HBM_PEAK_GBS, 4), traffic=traffic.get("attend"), us_per_launch=round(att_us, 2),
                    algorithmic_bytes=work["attend_bytes"])
    peak = MFMA_PEAK_TFLOPS[w.dtype]
    roof_gemm = dict(kernel="rebuild_gemm", bound="mfma" if w.dtype == "bf16" else "alu",
                     achieved=round(gemm_tflops, 1), peak=peak, unit="TFLOP/s", frac=round(gemm_tflops / peak, 4),
                     traffic=traffic.get("rebuild_gemm"), us_per_launch=round(gemm_us, 2), algorithmic_flops=work["gemm_flops"])
    dominant = roof_gemm if gemm_us >= att_us else roof_att

    line = {
        "metric": "decoded tokens/sec per decode layer at cache K",
        "value": round(value, 1), "unit": "tokens/s/layer", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "batch": w.B, "heads": w.H, "head_dim": w.d, "hidden": w.D,
                   "cache_slots_K": w.K, "rebuild_budget_R": w.R, "prompt": w.S, "layers": w.L,
                   "score_mode": "h2o" if w.h2o else "rescore" if w.rescore else "static",
                   "input_order": args.input_order, "library_default_input_order": "stream", "rope_base": w.rope_base},
        "roofline": dominant,
        "roofline_attend": roof_att, "roofline_rebuild_gemm": roof_gemm,
        "kernel_us": {k: round(v, 2) for k, v in per_kernel_us.items()},
        "kernel_us_sum": round(sum(per_kernel_us.values()), 2),
    }
    if w.L == 1 and other:
        line["stream_ordered_inputs" if not INPUTS_ORDERED else "ready_inputs"] = {
            "ms_per_step": round(1e3 * other, 4), "value": round(w.B / other, 1)}
    if stack:
        line["stack"] = stack
    default_line = (args.workload == "llama7b_layer" and w.L == 1 and not (args.rescore or args.h2o or args.rope_base))
    if default_line and not args.no_other_workloads:
        # the other single-layer workloads, compactly: high_batch is the one whose cache (546 MB per step) does not
        # fit the 256 MB last-level cache, so its attention figure is the HBM-bound one
        t0 = time.time()
        line["other_workloads"] = [other_workload_entry("high_batch"), other_workload_entry("long_context"),
                                   stack_workload_entry()]
        hb = line["other_workloads"][0]
        traffic_hb = recorded_traffic(workload("high_batch"))
        line["roofline_attend_high_batch"] = dict(
            kernel="attend", bound="hbm", achieved=hb["attend_GBs"], peak=HBM_PEAK_GBS, unit="GB/s",
            frac=hb["attend_frac_of_hbm_peak"], traffic=traffic_hb.get("attend"), us_per_launch=hb["attend_us"],
            algorithmic_bytes=hb["attend_algorithmic_bytes"])
        log(f"other workloads took {time.time() - t0:.1f}s")
        t0 = time.time()
        line["other_paths"] = other_path_entries(workload("llama7b_layer"))
        log(f"other paths took {time.time() - t0:.1f}s")
    if not args.no_cpu_baseline and not w.h2o:
        t0 = time.time()
        line["cpu_baseline"] = run_cpu_baseline(w)
        log(f"cpu baseline took {time.time() - t0:.1f}s in total")
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
