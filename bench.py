#!/usr/bin/env python3
"""Throughput of the prefill-time KV reduction pass on one MI355X.

One step = one pass of the whole hot path over one layer of the 32k-context
workload (the benchmark configuration configs[3]: Mistral-7B-shaped, 8 KV heads x 4 query heads,
head_dim 128, seq_len 32768, fp16, clustered keys/values with drift):
  spindle_compress_deep    (window 64, pool 7, budget 2048)  and
  spindle_compress_shallow (K and V, theta 0.98 / 0.95, codebook cap 2048).
Inputs are resident in HBM before the timed region.  Prints one JSON line.
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

PEAK_MFMA_F16_TFLOPS = 2500.0      # MI355X dense fp16 matrix peak
PEAK_HBM_GBS = 8000.0
PEAK_VALU_F64_TFLOPS = 78.6         # 256 CUs x 64 lanes x 2 flop x 2.4 GHz


# sets of buffers the pipelined steps rotate over (2.60 ms per step with two, 2.56 with three, 2.60 with four)
PIPELINE_SETS = 3


def cpu_baseline(L, wl, max_threads=16):
    """The oracle as it stands, timed on this host on the whole layer the GPU step processes: every
    eviction unit and every codebook problem (K and V of every head) in full, one problem per
    thread (the oracle itself is single-threaded; ctypes releases the interpreter lock).  `value`
    is the layer's tokens over the wall time with `cores` threads; the time the threads spent per
    problem (while the other cores were busy too) is reported beside it."""
    import oracle
    from concurrent.futures import ThreadPoolExecutor
    oracle.lib()
    d = L.head_dim
    scale = float(np.float32(1.0 / np.sqrt(d)))
    try:
        avail = len(os.sched_getaffinity(0))
    except AttributeError:
        avail = os.cpu_count() or 1
    cores = max(1, min(max_threads, avail))
    units = [(b, h) for b in range(L.batch) for h in range(L.n_kv_heads)]
    jobs = [("deep", b, h) for b, h in units] + [(t, b, h) for t in ("k", "v") for b, h in units]

    def run(job):
        kind, b, h = job
        t0 = time.perf_counter()
        if kind == "deep":
            oracle.deep_unit(wl.to_f64(L.Qw[b, h * L.group_size:(h + 1) * L.group_size], L.dtype),
                             wl.to_f64(L.K[b, h], L.dtype), scale, L.pool, L.budget)
        else:
            X = wl.to_f64((L.K if kind == "k" else L.V)[b, h], L.dtype)
            theta = L.theta_k if kind == "k" else L.theta_v
            o = oracle.shallow_unit(X, float(np.float32(theta)), L.max_codes)
            del o
        return kind, time.perf_counter() - t0

    t0 = time.perf_counter()
    with ThreadPoolExecutor(max_workers=cores) as ex:
        times = list(ex.map(run, jobs))
    wall = time.perf_counter() - t0
    t_deep = [t for k, t in times if k == "deep"]
    t_code = [t for k, t in times if k != "deep"]
    busy = sum(t for _, t in times)
    return {"value": L.batch * L.seq_len / wall, "unit": "tokens/s/layer", "cores": cores, "kind": "oracle",
            "sample": f"the whole layer of the timed step, nothing scaled: {len(t_deep)} eviction units and "
                      f"{len(t_code)} codebook problems of {L.seq_len} tokens, one per thread, {cores} threads",
            "wall_s": wall, "thread_s_per_eviction_unit": float(np.mean(t_deep)),
            "thread_s_per_codebook_problem": float(np.mean(t_code)),
            "one_core_value_from_thread_time": L.batch * L.seq_len / busy}


def deep_bytes(units, l, d, esz, kept):
    """Algorithmic HBM bytes of one eviction call: K read once, the kept rows of K and V read and
    written, three words per key of scores (raw, pooled, index)."""
    return units * (l * d * esz + 2 * 2 * kept * d * esz + 3 * 4 * l)


def time_deep_call(torch, plan, K, V, Q, reps=30):
    """Average duration of the whole eviction call (its four kernels back to back on one stream,
    no events between them): one pair of torch events around `reps` calls."""
    for _ in range(3):
        plan.run(K, V, Q)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        plan.run(K, V, Q)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def deep_folded(torch, sb, wl):
    """The 24 eviction layers of the 8192-token stack (configs[2]) folded into the batch dimension of
    ONE call, with the stack's per-layer budgets as per-unit budgets: 192 units."""
    layers = list(range(8, 32))
    Ls = [wl.config3_layer(i) for i in layers]
    K = sb.to_device(np.concatenate([x.K for x in Ls]), "f16")
    V = sb.to_device(np.concatenate([x.V for x in Ls]), "f16")
    Q = sb.to_device(np.concatenate([x.Qw for x in Ls]), "f16")
    H = Ls[0].n_kv_heads
    per_unit = [wl.config3_budget(i) for i in layers for _ in range(H)]
    budgets = torch.tensor(per_unit, dtype=torch.int32, device="cuda")
    plan = sb.plan_deep(K, Ls[0].group_size, "f16", Ls[0].window, Ls[0].pool, Ls[0].window, want_scores=False,
                        budgets=budgets, out_stride=max(per_unit))
    ms = time_deep_call(torch, plan, K, V, Q, reps=20)
    l, d = Ls[0].seq_len, Ls[0].head_dim
    nbytes = deep_bytes(len(per_unit), l, d, 2, float(np.mean(per_unit)))
    gbs = nbytes / (ms * 1e-3) / 1e9
    return {"workload": "configs[2] layers 8-31 as one call: 192 units of 8192 tokens, fp16, budgets 2048 .. 256",
            "ms_per_call": ms, "tokens_per_s": len(layers) * l / (ms * 1e-3), "bound": "hbm", "achieved": gbs,
            "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS}


def config5_layer(torch, sb, wl, cap=4096, steps=8, warmup=3):
    """One layer of configs[4] (batch 4, bf16, half of the tokens isolated noise, budget = cap), the
    two calls one after the other on one stream: a secondary figure of the same run."""
    L = wl.config5_layer(0, cap)
    K, V, Q = (sb.to_device(x, L.dtype) for x in (L.K, L.V, L.Qw))
    deep = sb.plan_deep(K, L.group_size, L.dtype, L.window, L.pool, L.budget, want_scores=False)
    shallow = sb.plan_shallow(K, L.dtype, L.theta_k, L.theta_v, L.max_codes)
    for _ in range(warmup):
        deep.run(K, V, Q)
        shallow.run(K, V)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        deep.run(K, V, Q)
        shallow.run(K, V)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    sb.spindle_profile(1)
    for _ in range(3):
        deep.run(K, V, Q)
        shallow.run(K, V)
    torch.cuda.synchronize()
    per = {}
    for name, t in sb.spindle_profile_read():
        per[name] = per.get(name, 0.0) + t / 3
    sb.spindle_profile(0)
    deep_ms = time_deep_call(torch, deep, K, V, Q, reps=10)
    units = L.batch * L.n_kv_heads
    nbytes = deep_bytes(units, L.seq_len, L.head_dim, 2, min(L.budget, L.seq_len))
    gram_flop = 2 * units * (L.seq_len ** 2 / 2) * L.head_dim * 2
    assert min(shallow.out["n_codes_k"].min().item(), shallow.out["n_codes_v"].min().item()) >= 1
    out = {"workload": f"configs[4], one layer: batch 4 x {L.seq_len}, bf16, pool 15, budget = cap = {cap}; one stream",
           "steps": steps, "ms_per_step": ms, "tokens_per_s": L.batch * L.seq_len / (ms * 1e-3), "kernel_ms": per,
           "deep_call_ms": deep_ms, "deep_frac_of_hbm": nbytes / (deep_ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
           "shallow_gram_frac_of_mfma": gram_flop / (per["shallow_gram"] * 1e-3) / 1e12 / PEAK_MFMA_F16_TFLOPS}
    del deep, shallow, K, V, Q
    torch.cuda.empty_cache()
    return out


def time_reconstruct(torch, sb, L, shallow, reps=20):
    """Eq. 14 on the step's own output (K and V of every unit), outside the timed step: a gather and
    scale bound by HBM.  Algorithmic bytes per token: one row written, index and magnitude read;
    the codebook (cap rows per unit) is read once."""
    o = shallow.out
    units = L.batch * L.n_kv_heads
    outs = {t: torch.empty((L.batch, L.n_kv_heads, L.seq_len, L.head_dim), dtype=o["C_k"].dtype,
                           device=o["C_k"].device) for t in ("k", "v")}

    def once():
        for t in ("k", "v"):
            sb.spindle_reconstruct(units, L.seq_len, L.head_dim, sb._DT[L.dtype], L.max_codes,
                                   o[f"C_{t}"], o[f"ref_{t}"], o[f"mag_{t}"], outs[t])
    once()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        once()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    esz = outs["k"].element_size()
    nbytes = 2 * units * (L.seq_len * (L.head_dim * esz + 8) + L.max_codes * L.head_dim * esz)
    gbs = nbytes / (ms * 1e-3) / 1e9
    return {"ms_k_and_v": ms, "bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
            "frac": gbs / PEAK_HBM_GBS, "tokens_per_s": L.batch * L.seq_len / (ms * 1e-3)}


def time_decode(torch, sb, L, K, shallow, m=256, novel=0.25, reps=10):
    """Decode-time merge on the step's own K codebooks, outside the timed step: m later tokens per
    head (tokens of the layer at random positions with 1 % noise; a quarter replaced by directions
    the layer never saw) merged into the stored entries.  Dominant kernel: the double-precision
    search of the stored entries, 2 x 128 flop per (token, entry) on the vector ALUs."""
    g = torch.Generator(device="cuda").manual_seed(5)
    pos = torch.randint(0, L.seq_len, (m,), generator=g, device="cuda")
    base = K[:, :, pos].float()
    base = base * (1 + 0.01 * torch.randn(base.shape, generator=g, device="cuda"))
    fresh = torch.randn(base.shape, generator=g, device="cuda")
    pick = torch.rand((L.batch, L.n_kv_heads, m, 1), generator=g, device="cuda") < novel
    new = torch.where(pick, fresh, base).to(K.dtype).contiguous()
    cap = L.max_codes + m
    stored = shallow.out["n_codes_k"].to(torch.int32)
    Cb = torch.zeros((L.batch, L.n_kv_heads, cap, L.head_dim), dtype=K.dtype, device="cuda")
    Cb[:, :, :L.max_codes] = shallow.out["C_k"]
    nc = stored.clone()
    out = sb.decode_merge(new, L.dtype, L.theta_k, Cb, nc)          # warm-up
    torch.cuda.synchronize()
    sb.spindle_profile(True)
    for _ in range(reps):
        nc.copy_(stored)
        out = sb.decode_merge(new, L.dtype, L.theta_k, Cb, nc)
    torch.cuda.synchronize()
    recs = sb.spindle_profile_read()
    sb.spindle_profile(False)
    ms = {}
    for name, t in recs:
        ms[name] = ms.get(name, 0.0) + t / reps
    total = sum(ms.values())
    # the usual decode step: one token per head and call, a single launch
    one = new[:, :, :1].contiguous()
    sb.spindle_profile(True)
    for _ in range(reps):
        nc.copy_(stored)
        sb.decode_merge(one, L.dtype, L.theta_k, Cb, nc)
    torch.cuda.synchronize()
    single = [t for name, t in sb.spindle_profile_read() if name == "decode_small"]
    sb.spindle_profile(False)
    flop = 2.0 * L.head_dim * m * float(stored.sum().item())
    tf = flop / (ms["decode_match"] * 1e-3) / 1e12
    return {"new_tokens_per_head": m, "stored_entries": stored.cpu().numpy().ravel().tolist(),
            "merged_with_stored": out["n_matched"].cpu().numpy().ravel().tolist(),
            "entries_after": out["n_found"].cpu().numpy().ravel().tolist(),
            "kernel_ms": ms, "tokens_per_s": L.batch * L.n_kv_heads * m / (total * 1e-3),
            "one_token_per_head_call_us": float(np.mean(single)) * 1e3,
            "roofline": {"kernel": "decode_match", "bound": "alu", "achieved": tf, "peak": PEAK_VALU_F64_TFLOPS,
                         "unit": "TFLOP/s", "frac": tf / PEAK_VALU_F64_TFLOPS}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # the part needs about 0.1 s of load before its clocks settle: a step measured in the first
    # few iterations is 1.5-4 % slower than the steady state
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--seq-len", type=int, default=32768)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-pipeline", action="store_true",
                    help="one step at a time (two streams within the step); default: consecutive steps are "
                         "pipelined over three sets of buffers, the similarity phase of a step beside the codebook "
                         "phase and the eviction call of the step before")
    ap.add_argument("--one-stream", action="store_true",
                    help="time the eviction call and the codebook call one after the other on one stream "
                         "(default: the eviction call runs on a side stream beside the second half of the codebook call)")
    ap.add_argument("--workload", choices=["config4", "config5"], default="config4",
                    help="config4 = the benchmark configuration; config5 = one layer of the batch-4 bf16 stack "
                         "(half of the tokens isolated noise, codebook cut to --cap): a secondary figure")
    ap.add_argument("--cap", type=int, default=4096, help="budget = codebook cap of --workload config5")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run the plain 1 GiB copy (scale reference for the HBM traffic counters) even with --no-extras")
    ap.add_argument("--calibrate", action="store_true",
                    help="run the library's matrix-core and similarity-loop calibrations even with --no-extras")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the secondary measurements (folded eviction call, config-5 layer, reconstruction, decode)")
    ap.add_argument("--traffic-json", default=os.path.join(ROOT, "profiles", "shallow_gram_config4_traffic.json"))
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)")

    import torch
    from paper_2507_06517_amd import binding as sb, workloads as wl
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    sb.lib()
    torch.cuda.set_device(0)

    L = wl.config4(0, seq_len=args.seq_len) if args.workload == "config4" else wl.config5_layer(0, args.cap)
    K, V, Q = (sb.to_device(x, L.dtype) for x in (L.K, L.V, L.Qw))
    deep = sb.plan_deep(K, L.group_size, L.dtype, L.window, L.pool, L.budget, want_scores=False)
    shallow = sb.plan_shallow(K, L.dtype, L.theta_k, L.theta_v, L.max_codes)
    stream = torch.cuda.current_stream()
    mode = "one-stream" if args.one_stream else ("two-streams" if args.no_pipeline else "pipelined")
    layer = sb.OverlappedLayer(deep, shallow)
    first = [(deep, shallow)]
    pipe = sb.PipelinedLayers(lambda: first.pop() if first else (
        sb.plan_deep(K, L.group_size, L.dtype, L.window, L.pool, L.budget, want_scores=False),
        sb.plan_shallow(K, L.dtype, L.theta_k, L.theta_v, L.max_codes)), depth=PIPELINE_SETS) if mode == "pipelined" else None

    def step():
        if mode == "one-stream":
            deep.run(K, V, Q)
            shallow.run(K, V)
        elif mode == "two-streams":
            layer.run(K, V, Q)                       # eviction on a side stream beside the codebook loop
        else:
            pipe.run(K, V, Q)                        # ... and the next step's similarity phase beside both

    def drain():
        if pipe is not None:
            pipe.finish()
        torch.cuda.synchronize()

    for _ in range(args.warmup):
        step()
    drain()
    copy_gbs = None
    if args.calibrate_copy or not args.no_extras:
        # a plain 1 GiB copy by the library's own kernel (`cal_copy` in a profile): what the memory system
        # sustains, and the known size the HBM traffic counters are scaled by
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        copy_gbs = sb.spindle_calibrate_copy(src, dst)
        torch.cuda.synchronize()
        del src, dst

    # timed region: whole-step wall time; the dominant kernel is bracketed by HIP events on the
    # launch stream (two events per step; events around every kernel would cost 5 % of the step)
    sb.spindle_profile(2)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step()
    drain()
    wall = time.perf_counter() - t0
    gram_recs = [ms for name, ms in sb.spindle_profile_read() if name == "shallow_gram"]
    assert len(gram_recs) == args.steps
    gram_ms = float(np.mean(gram_recs))
    ms_step = wall * 1e3 / args.steps

    # for reference (not the reported throughput): the same steps one at a time, two streams within a step
    ms_step_unpipelined = None
    if mode == "pipelined":
        sb.spindle_profile(0)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            layer.run(K, V, Q)
        torch.cuda.synchronize()
        ms_step_unpipelined = (time.perf_counter() - t0) * 1e3 / args.steps

    # breakdown pass (not the reported throughput): the same steps with events around every kernel
    sb.spindle_profile(1)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3 * args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        ev[3 * i].record(stream)
        deep.run(K, V, Q)
        ev[3 * i + 1].record(stream)
        shallow.run(K, V)
        ev[3 * i + 2].record(stream)
    torch.cuda.synchronize()
    ms_step_all_events = (time.perf_counter() - t0) * 1e3 / args.steps
    recs = sb.spindle_profile_read()
    sb.spindle_profile(0)

    ms_deep = float(np.mean([ev[3 * i].elapsed_time(ev[3 * i + 1]) for i in range(args.steps)]))
    ms_shallow = float(np.mean([ev[3 * i + 1].elapsed_time(ev[3 * i + 2]) for i in range(args.steps)]))
    per_kernel = {}
    for name, ms in recs:
        per_kernel.setdefault(name, []).append(ms)
    # per step: some kernels are launched several times per step (merge rounds)
    kernel_ms = {k: float(np.sum(v)) / args.steps for k, v in per_kernel.items()}

    st = shallow.stats()
    n_codes = {t: shallow.out[f"n_found_{t}"].cpu().numpy().ravel().tolist() for t in ("k", "v")}
    assert min(shallow.out["n_codes_k"].min().item(), shallow.out["n_codes_v"].min().item()) >= 1, \
        "codebook construction did not finish"

    tokens = L.batch * L.seq_len
    units = L.batch * L.n_kv_heads
    # dominant kernel: the similarity tiles.  Algorithmic work = each unordered token pair
    # once: n^2/2 pairs x 128 multiply-adds x 2 flop, per (unit, K|V).
    gram_flop = 2 * units * (L.seq_len ** 2 / 2) * L.head_dim * 2
    achieved = gram_flop / (gram_ms * 1e-3) / 1e12
    # HBM bytes per launch of the dominant kernel: not measurable inside this process (it takes two
    # rocprofv3 counter runs); read from the committed summary, with the source commit it names
    traffic, traffic_source = None, None
    if args.workload == "config4" and args.seq_len == 32768 and os.path.exists(args.traffic_json):
        try:
            tj = json.load(open(args.traffic_json))
            traffic = tj.get("hbm_bytes_per_launch")
            traffic_source = {"file": os.path.relpath(args.traffic_json, ROOT), "kernel": tj.get("kernel"),
                              "measured_on_commit": tj.get("measured_on_commit")}
        except Exception:
            traffic = None
    out = {
        "metric": "KV tokens compressed/sec per layer (deep & shallow) at 32k ctx",
        "value": tokens / (ms_step * 1e-3),
        "unit": "tokens/s/layer",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": L.dtype, "data": "synthetic",
        "config": {"workload": (f"configs[3]: Mistral-7B-shaped layer, 8 KV heads x 4 Q heads, head_dim 128, "
                                f"seq_len {L.seq_len}, fp16, 256 drifting clusters; deep: window 64, pool 7, "
                                f"budget 2048; shallow: K and V, theta 0.98/0.95, cap 2048; batch 1")
                   if args.workload == "config4" else
                   (f"configs[4], one layer: batch 4, 8 KV heads x 4 Q heads, head_dim 128, seq_len {L.seq_len}, "
                    f"bf16, half clustered / half noise; deep: window 64, pool 15, budget {L.budget}; "
                    f"shallow: K and V, theta 0.98/0.95, cap {L.max_codes}")},
        "streams": {"one-stream": "one: the eviction call, then the codebook call",
                    "two-streams": "two: the eviction call runs on a side stream beside the second half of the "
                                   "codebook call (spindle_shallow_graph, event, spindle_shallow_codebook)",
                    "pipelined": "consecutive steps pipelined over three sets of buffers: the similarity phase of a "
                                 "step (spindle_shallow_graph) runs beside the codebook phase "
                                 "(spindle_shallow_codebook) and the eviction call of the step before; two "
                                 "similarity phases never overlap"}[mode],
        "breakdown_pass": "deep_ms, shallow_ms and kernel_ms come from a second pass with the two calls one after the "
                          "other on one stream and HIP events around every kernel, which lengthens the step; "
                          "roofline uses the timed steps' own events",
        "ms_per_step_one_at_a_time": ms_step_unpipelined,
        "tokens_per_s_one_at_a_time": tokens / (ms_step_unpipelined * 1e-3) if ms_step_unpipelined else None,
        "ms_per_step_with_all_events": ms_step_all_events,
        "deep_ms": ms_deep, "shallow_ms": ms_shallow,
        "deep_tokens_per_s": tokens / (ms_deep * 1e-3), "shallow_tokens_per_s": tokens / (ms_shallow * 1e-3),
        "kernel_ms": kernel_ms,
        "codebook_entries_found": n_codes,
        "merge_rounds": st[:, 0].tolist(), "pairs_decided_in_f64": int(st[:, 2].sum()),
        "merge_phase_us_unit0": st[0, 4:14].tolist(),
        "roofline": {"kernel": "shallow_gram", "bound": "mfma", "kernel_ms": gram_ms, "achieved": achieved,
                     "peak": PEAK_MFMA_F16_TFLOPS, "unit": "TFLOP/s", "frac": achieved / PEAK_MFMA_F16_TFLOPS,
                     "traffic": traffic, "traffic_source": traffic_source},
    }
    # what the part sustains (measurement aids of the library): a register-resident fp16 MFMA loop, and
    # the similarity kernel's own loop with the packing of the results left out
    if copy_gbs is not None:
        out["hbm_copy_measured"] = {"gb_per_s_read_plus_write": copy_gbs, "frac_of_peak": copy_gbs / PEAK_HBM_GBS,
                                    "bytes": 2 << 30}
    if args.calibrate or not args.no_extras:
        bare = [sb.spindle_calibrate_similarity(shallow) for _ in range(5)][1:]
        bare_nostream = float(np.mean([sb.spindle_calibrate_similarity(shallow, 1) for _ in range(4)][1:]))
        bare_mfma = float(np.mean([sb.spindle_calibrate_similarity(shallow, 2) for _ in range(4)][1:]))
        mfma = max(sb.spindle_calibrate_mfma(4096) for _ in range(3))
        mfma_data = max(sb.spindle_calibrate_mfma(4096, 1) for _ in range(3))
        out["roofline"]["calibration"] = {
            "mfma_f16_register_loop_tflops": mfma, "mfma_f16_register_loop_frac_of_peak": mfma / PEAK_MFMA_F16_TFLOPS,
            "mfma_f16_register_loop_workload_like_operands_tflops": mfma_data,
            "mfma_f16_register_loop_workload_like_operands_frac_of_peak": mfma_data / PEAK_MFMA_F16_TFLOPS,
            "similarity_loop_without_packing_ms": float(np.mean(bare)),
            "similarity_loop_without_packing_frac_of_peak": gram_flop / (float(np.mean(bare)) * 1e-3) / 1e12 / PEAK_MFMA_F16_TFLOPS,
            "similarity_loop_without_packing_and_streaming_loads_ms": bare_nostream,
            "similarity_loop_matrix_instructions_only_ms": bare_mfma,
            "similarity_loop_matrix_instructions_only_frac_of_peak": gram_flop / (bare_mfma * 1e-3) / 1e12 / PEAK_MFMA_F16_TFLOPS,
            "note": "without packing: the kernel's matrix instructions, staging and barriers alone; what is left "
                    "between this and roofline.frac is the vector work on the results.  The next two leave out the "
                    "loads that stream tokens into LDS, then also the fragment reads: the part is power-limited, "
                    "and each of these draws from the same budget as the matrix instructions"}
    # secondary: the eviction call against the HBM roofline, timed on its own without events between
    # its kernels (deep_ms above is the breakdown pass, where every kernel is followed by an event gap)
    esz = K.element_size()
    nbytes = deep_bytes(units, L.seq_len, L.head_dim, esz, min(L.budget, L.seq_len))
    deep_call_ms = time_deep_call(torch, deep, K, V, Q)
    out["deep_roofline"] = {"bound": "hbm", "call_ms": deep_call_ms, "achieved": nbytes / (deep_call_ms * 1e-3) / 1e9,
                            "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": nbytes / (deep_call_ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
                            "tokens_per_s": tokens / (deep_call_ms * 1e-3),
                            "kernels_ms": {k: v for k, v in kernel_ms.items() if k.startswith("deep_")}}
    if not args.no_extras:
        out["reconstruct"] = time_reconstruct(torch, sb, L, shallow)
        out["decode_merge"] = time_decode(torch, sb, L, K, shallow)
    # Eq. 15 on this layer: eviction alone (r1) and replacement alone (r2 r3), each on the full layer
    stored = int(shallow.out["n_codes_k"].sum().item() + shallow.out["n_codes_v"].sum().item())
    bits = 8 * torch.empty(0, dtype=sb.torch_dtype(L.dtype)).element_size()
    # (16-bit references as the library's 65535-token limit allows; the magnitudes it writes are float32)
    r1 = sb.spindle_reserve_ratio(2 * units * min(L.budget, L.seq_len), 2 * units * L.seq_len, 1, L.head_dim, 16, bits, 32)[0]
    _, r2, r3, r23 = sb.spindle_reserve_ratio(2 * units * L.seq_len, 2 * units * L.seq_len, stored, L.head_dim, 16, bits, 32)
    out["reserve_ratio"] = {"eviction_r1": r1, "replacement_r2": r2, "r3": r3, "replacement_r2_r3": r23,
                            "index_bits": 16, "magnitude_bits": 32, "element_bits": bits}
    del pipe, layer
    if not args.no_extras and args.workload == "config4":
        del deep, shallow, K, V, Q
        torch.cuda.empty_cache()
        out["deep_roofline_folded"] = deep_folded(torch, sb, wl)
        out["config5_layer"] = config5_layer(torch, sb, wl)
        deep = shallow = K = V = Q = None
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(L, wl)
    print(json.dumps(out), flush=True)
    # release device memory before interpreter shutdown
    del deep, shallow, K, V, Q
    torch.cuda.synchronize()
    torch.cuda.empty_cache()


if __name__ == "__main__":
    main()
