#!/usr/bin/env python3
"""Benchmark of the SP-MoE verify-layer hot path on one MI355X.

A step = one pass of the whole hot path (gate/top-k -> grouped gate+up GEMM -> grouped down GEMM -> weighted
combine) over one verification batch of synthetic tokens, all expert weights already resident in HBM when the
timed region starts.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

With no --workload the line carries the whole metric "verify-layer us & tokens/s; expert-GEMM HBM GB/s vs peak;
% H2D hidden":
  * the timed steps on the Mixtral-8x7B-shaped layer (d_model 4096, d_ff 14336, 8 experts, top-2, bf16 weights,
    8 tokens) -> value, ms_per_step, latency percentiles, per-kernel times, roofline of the dominant kernel;
  * "layers": the same measurement, shorter, on the other single-GPU layer shapes (DeepSeek-V2-Lite, T = 16;
    Mixtral-8x22B, T = 32 -- the largest configuration);
  * "h2d": one offloaded stack (DeepSeek-V2-Lite shape, cache budget 16 experts per layer, cutoff layer chosen by
    the paper's policy from times measured in the run): share of the prefetch copy time hidden under executing
    kernels, link rate against its measured peak, hit rate;
  * "cpu_baseline": the CPU oracle on the same layer and batches, single thread and OpenMP.
With --workload NAME only that workload runs (resident layers: c1_small, c2_mixtral_8x7b, or any shape with
--resident; offloaded stacks: c3_..., c4_..., c5_..., phi_3_5_moe).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0      # MI355X published HBM3E bandwidth


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def profiled_traffic(workload):
    """HBM bytes per launch of the gate/up kernel as measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (scaled
    by a copy-kernel calibration) and recorded in profiles/verify_layer_<workload>.txt, with the commit that
    summary was measured at.  (None, None) if there is no such record."""
    path = os.path.join(ROOT, "profiles", "verify_layer_%s.txt" % workload)
    traffic = commit = None
    try:
        for line in open(path):
            if line.startswith("gate_up_traffic_bytes_per_launch:"):
                traffic = int(line.split(":")[1])
            if line.startswith("measured at commit:"):
                commit = line.split(":", 1)[1].strip()
    except OSError:
        pass
    return traffic, commit


def union(intervals):
    """Sorted, merged copy of a list of (t0, t1)."""
    out = []
    for a, b in sorted(intervals):
        if out and a <= out[-1][1]:
            out[-1][1] = max(out[-1][1], b)
        else:
            out.append([a, b])
    return out


def measure(intervals):
    return sum(b - a for a, b in intervals)


def intersect(u1, u2):
    """Total overlap of two merged interval lists."""
    i = j = 0
    tot = 0.0
    while i < len(u1) and j < len(u2):
        lo, hi = max(u1[i][0], u2[j][0]), min(u1[i][1], u2[j][1])
        if hi > lo:
            tot += hi - lo
        if u1[i][1] < u2[j][1]:
            i += 1
        else:
            j += 1
    return tot


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


# ---------------------------------------------------------------------------------------------------------------
# resident layer
# ---------------------------------------------------------------------------------------------------------------
def run_resident(name, spec, args, steps, warmup, keep_for_cpu=False):
    """Times `steps` verify-layer calls on one layer of the workload's shape with every expert resident.
    Returns (result block, (workload, host batches) for the CPU baseline or None)."""
    import numpy as np
    import torch
    import spmoe_inputs as si
    from paper_2510_10302_amd import workload as W

    d, f, E, k, T, n_shared = spec["d"], spec["f"], spec["E"], spec["k"], spec["T"], spec["shared"]
    t0 = time.time()
    wl = W.Workload(d=d, f=f, E=E, k=k, shared=n_shared, dtype=spec["dtype"], layers=1, seed=0)
    cfg = W.make_config(wl, max_tokens=T)
    stream = torch.cuda.Stream() if args.graph else torch.cuda.current_stream()
    torch.cuda.set_stream(stream)
    L = W.Loaded(wl, cfg, stream=stream)
    log("bench: workload %s built in %.1f s (expert blob %.1f MiB)" % (name, time.time() - t0, W.sp.expert_blob_bytes(cfg) / 2 ** 20))
    ctx = L.ctx
    elem = 2 if spec["dtype"] == "bf16" else 4
    xs_host = [si.hidden_correlated(1000 + i, T, d, args.token_corr, args.sequences) for i in range(args.batches)]
    xs = [torch.from_numpy(x).cuda() for x in xs_host]
    out = torch.empty((T, d), dtype=torch.float32, device="cuda")

    # routing of each batch (for the algorithmic byte count: only activated experts are streamed)
    idx = torch.empty((T, k), dtype=torch.int32, device="cuda")
    w = torch.empty((T, k), dtype=torch.float32, device="cuda")
    e_act = []
    for x in xs:
        ctx.gate_topk(0, x, k, idx, w)
        ctx.sync()
        e_act.append(len(set(idx.cpu().numpy().reshape(-1).tolist())) + n_shared)

    def step(i):
        ctx.moe_verify_layer(0, xs[i % len(xs)], out)

    # first launches load code objects, size the grids and let the clocks settle: part of the set-up, not of the
    # warm-up the caller asks for
    for i in range(100):
        step(i)
    ctx.sync()
    for i in range(warmup):
        step(i)
    ctx.sync()
    torch.cuda.synchronize()
    if args.graph:
        # one graph = one pass over the batches; a step is still one verify-layer call
        steps = max(len(xs), steps // len(xs) * len(xs))
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            for i in range(len(xs)):
                step(i)
        graph.replay()
        torch.cuda.synchronize()
        t_start = time.perf_counter()
        for _ in range(steps // len(xs)):
            graph.replay()
    else:
        t_start = time.perf_counter()
        for i in range(steps):
            step(i)
    ctx.sync()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    ms_per_step = elapsed * 1e3 / steps

    # latency distribution: each call between its own pair of HIP events on the compute stream (separate pass; the
    # events sit between the layers, not inside them)
    n_lat = 200
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_lat)]
    for i, (a, b) in enumerate(evs):
        a.record(stream)
        step(i)
        b.record(stream)
    torch.cuda.synchronize()
    lat = np.sort(np.array([a.elapsed_time(b) * 1e3 for a, b in evs]))
    pct = {"p10": float(lat[int(0.1 * (n_lat - 1))]), "median": float(np.median(lat)), "p90": float(lat[int(0.9 * (n_lat - 1))]),
           "calls": n_lat}

    # per-kernel durations from HIP events on the compute stream (separate pass: the events sit between kernels)
    kms = np.zeros(4)
    bytes_gu = bytes_dn = 0.0
    n_prof = 3 * len(xs)
    for i in range(n_prof):
        ctx.profile_begin()
        step(i)
        kms += np.array(ctx.last_layer_kernel_ms())
        ctx.profile_collect()
        bytes_gu += e_act[i % len(xs)] * 2.0 * d * f * elem
        bytes_dn += e_act[i % len(xs)] * 1.0 * d * f * elem
    kms /= n_prof
    bytes_gu /= n_prof
    bytes_dn /= n_prof
    gu_gbs = bytes_gu / (kms[1] * 1e-3) / 1e9
    dn_gbs = bytes_dn / (kms[2] * 1e-3) / 1e9
    both_gbs = (bytes_gu + bytes_dn) / ((kms[1] + kms[2]) * 1e-3) / 1e9
    layer_gbs = (bytes_gu + bytes_dn) / (ms_per_step * 1e-3) / 1e9
    log("bench: %s: layer %.1f us | kernels ms route %.4f gate_up %.4f down %.4f combine %.4f | gate_up %.0f GB/s, down %.0f GB/s, "
        "both %.0f GB/s, whole layer %.0f GB/s, mean active experts %.2f"
        % (name, ms_per_step * 1e3, kms[0], kms[1], kms[2], kms[3], gu_gbs, dn_gbs, both_gbs, layer_gbs, float(np.mean(e_act))))
    traffic, commit = profiled_traffic(name)
    plan_gu, plan_dn = (W.sp.gemm_plan(cfg, 0), W.sp.gemm_plan(cfg, 1)) if spec["dtype"] == "bf16" else (None, None)
    block = {
        "value": T * steps / elapsed, "unit": "tokens/s", "steps": steps, "warmup": warmup, "ms_per_step": ms_per_step,
        "verify_layer_us": ms_per_step * 1e3, "verify_layer_us_percentiles": pct, "dtype": spec["dtype"],
        "config": {"workload": name, "d_model": d, "d_ff": f, "n_experts": E, "top_k": k, "n_shared": n_shared,
                   "verify_tokens": T, "experts_resident": True, "mean_active_experts": float(np.mean(e_act)),
                   "token_corr": args.token_corr, "sequences": args.sequences, "hip_graph": bool(args.graph),
                   "gemm_plan_gate_up": plan_gu, "gemm_plan_down": plan_dn},
        "kernels_ms": {"route": float(kms[0]), "gate_up": float(kms[1]), "down": float(kms[2]), "combine": float(kms[3])},
        "expert_gemm_gbs": {"gate_up": gu_gbs, "down": dn_gbs, "both": both_gbs, "frac_of_peak_both": both_gbs / HBM_PEAK_GBS},
        "layer_weight_streaming_gbs": layer_gbs, "layer_frac_of_hbm_peak": layer_gbs / HBM_PEAK_GBS,
        "roofline": {"bound": "hbm", "kernel": "expert_gemm_kernel<gate_up>", "achieved": gu_gbs, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": gu_gbs / HBM_PEAK_GBS, "algorithmic_bytes": bytes_gu, "traffic": traffic,
                     "traffic_source": ("profiles/verify_layer_%s.txt (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an earlier run, "
                                        "measured at commit %s; not measured in this run)" % (name, commit)) if traffic else None},
    }
    keep = (wl, xs_host) if keep_for_cpu else None
    L.close()
    return block, keep


def cpu_baseline(wl, xs_host, T, k, seconds=10.0):
    """The fp32 C oracle on the same layer and batches: single thread, then OpenMP over the FFN rows."""
    import ctypes
    import oracle
    orc = oracle.Oracle("f32")
    omp = ctypes.CDLL("libgomp.so.1")
    nproc = os.cpu_count() or 1
    threads = int(os.environ.get("OMP_NUM_THREADS", nproc))
    legs = {}
    for label, nthr in (("single_thread", 1), ("openmp", threads)):
        omp.omp_set_num_threads(nthr)
        t1 = time.perf_counter()
        n = 0
        while n == 0 or time.perf_counter() - t1 < seconds:
            orc.moe_layer(xs_host[n % len(xs_host)], wl.gate[0], wl.layer_experts(0), k, shared=wl.shared[0])
            n += 1
        dt = time.perf_counter() - t1
        legs[label] = {"value": T * n / dt, "unit": "tokens/s", "threads": nthr, "ms_per_step": dt * 1e3 / n, "batches": n}
    omp.omp_set_num_threads(threads)
    best = legs["openmp"]
    return {"value": best["value"], "unit": "tokens/s", "cores": threads, "kind": "oracle", "ms_per_step": best["ms_per_step"],
            "single_thread": legs["single_thread"], "openmp": legs["openmp"], "nproc": nproc, "cpu_model": cpu_model(),
            "sample": "verify batches of %d tokens of the same layer (the %d seeded batches of the GPU run, cycled for about %.0f s "
                      "per leg: %d batch(es) single-threaded, %d with %d OpenMP threads), fp32 C oracle, one OpenMP loop over "
                      "FFN rows" % (T, len(xs_host), seconds, legs["single_thread"]["batches"], best["batches"], threads)}


def cpu_stack_estimate(wl, xs_host, T, k, stack_layers, evals=4):
    """CPU oracle time of a whole stack of this layer shape: `evals` layer evaluations timed (OpenMP, all host
    threads), scaled linearly to the stack's layer count."""
    import oracle
    orc = oracle.Oracle("f32")
    threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    t1 = time.perf_counter()
    for n in range(evals):
        orc.moe_layer(xs_host[n % len(xs_host)], wl.gate[0], wl.layer_experts(0), k, shared=wl.shared[0])
    per_layer = (time.perf_counter() - t1) / evals
    return {"kind": "oracle", "threads": threads, "ms_per_layer": per_layer * 1e3, "layers_timed": evals,
            "stack_layers": stack_layers, "stack_ms_scaled": per_layer * 1e3 * stack_layers,
            "stack_tokens_per_s_scaled": T / (per_layer * stack_layers),
            "sample": "%d evaluations of one layer of this shape (fp32 C oracle, OpenMP over FFN rows), scaled linearly to the "
                      "%d layers of the stack" % (evals, stack_layers)}


# ---------------------------------------------------------------------------------------------------------------
# offloaded stack
# ---------------------------------------------------------------------------------------------------------------
def run_offload(name, spec, args):
    """Stack with host-offloaded experts: one step = one speculative-decoding iteration on synthetic inputs.

    Drafting stage: for each of the T-1 draft forward passes and each layer, the predictor (target gate on
    the draft hidden state, Alg. 1) and the prefetcher (Alg. 2) run for layers <= cutoff, and a dense
    SwiGLU FFN of the same d x f shape runs on the compute stream as a stand-in for the draft model's layer.
    Verification stage: spmoe_moe_verify_layer on every layer for the T-token batch."""
    import numpy as np
    import torch
    import spmoe_inputs as si
    from paper_2510_10302_amd import workload as W

    d, f, E, k, T, n_shared = spec["d"], spec["f"], spec["E"], spec["k"], spec["T"], spec["shared"]
    layers = args.layers or spec["layers"]
    pred_k = args.pred_k or k
    steps, warmup = min(args.steps, 50), min(args.warmup, 5)
    t0 = time.time()
    wl = W.Workload(d=d, f=f, E=E, k=k, shared=n_shared, dtype="bf16", layers=layers, seed=0,
                    distinct=min(args.distinct, layers * E))
    cutoff_arg = -1 if args.cutoff == "auto" else int(args.cutoff)
    cfg = W.make_config(wl, max_tokens=T, slots=spec["slots"], cutoff_layer=cutoff_arg, pred_k=pred_k)
    L = W.Loaded(wl, cfg, warm=False, keep_canonical=False)
    dwl = W.Workload(d=d, f=args.draft_ff or f, E=1, k=1, shared=0, dtype="bf16", layers=layers, seed=1, distinct=2)
    D = W.Loaded(dwl, W.make_config(dwl, max_tokens=1), keep_canonical=False)
    blob = W.sp.expert_blob_bytes(cfg)
    # profiled inputs of the cutoff policy: per-expert load time, per-layer compute time of the drafting stage
    dx1 = torch.zeros((1, d), dtype=torch.float32, device="cuda")
    dy1 = torch.empty((1, d), dtype=torch.float32, device="cuda")
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    for rep in range(2):
        ev[0].record()
        for l in range(layers):
            D.ctx.moe_verify_layer(l, dx1, dy1)
        ev[1].record()
        torch.cuda.synchronize()
    t_comp_ms = ev[0].elapsed_time(ev[1]) / layers
    t_io_ms = L.ctx.measure_expert_load_ms(0, 0, repeats=3)
    free_b, _total_b = torch.cuda.mem_get_info()
    # The policy's window L_all * t_comp: one pass of the draft model ("pass"), or the whole drafting stage of T - 1
    # passes ("stage"), in which case the k experts predicted per layer are counted once for the stage (successive
    # draft tokens mostly predict the same experts, so the loads of a layer do not grow with the number of passes).
    window_layers = layers if args.draft_window == "pass" else layers * (T - 1)
    suggested = W.sp.suggest_cutoff(layers, window_layers, pred_k, t_comp_ms, t_io_ms, 0.0, float(blob), float(free_b))
    cutoff = suggested if args.cutoff == "auto" else cutoff_arg
    L.ctx.set_cutoff(cutoff)
    log("bench: offload workload %s: %d layers, %d slots/layer, cutoff %d (policy suggests %d over a window of one %s: t_comp %.3f "
        "ms/layer, t_io %.3f ms/expert), sigma %.2f, pred_k %d, built in %.1f s"
        % (name, layers, spec["slots"], cutoff, suggested, args.draft_window, t_comp_ms, t_io_ms, args.sigma, pred_k, time.time() - t0))

    # host link peak: one 1 GiB pinned -> device copy
    pin = torch.empty(2 ** 30, dtype=torch.uint8, pin_memory=True)
    dev = torch.empty(2 ** 30, dtype=torch.uint8, device="cuda")
    dev.copy_(pin, non_blocking=True)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    dev.copy_(pin, non_blocking=True)
    e1.record()
    torch.cuda.synchronize()
    link_gbs = 2 ** 30 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del pin, dev

    n_it = warmup + steps
    xs = [[torch.from_numpy(si.hidden_correlated(7, T, d, args.token_corr, args.sequences, iteration=i, layer=l)).cuda()
           for l in range(layers)] for i in range(n_it)]
    dxs = [[xs[i][l] + torch.from_numpy(si.draft_noise(7, T, d, args.sigma, iteration=i, layer=l)).cuda()
            for l in range(layers)] for i in range(n_it)]
    out = torch.empty((T, d), dtype=torch.float32, device="cuda")
    dout = torch.empty((1, d), dtype=torch.float32, device="cuda")
    ctx, dctx = L.ctx, D.ctx

    def iteration(i):
        for j in range(T - 1):
            for l in range(layers):
                if 0 <= l <= cutoff and args.prefetcher != "none":
                    if args.prefetcher == "worker":
                        ctx.predict_prefetch_async(l, dxs[i][l][j:j + 1])
                    else:
                        ctx.prefetch(l, ctx.predict_experts(l, dxs[i][l][j:j + 1]))
                        if args.prefetcher == "blocking":
                            ctx.sync()
                dctx.moe_verify_layer(l, dxs[i][l][j:j + 1], dout)
        for l in range(layers):
            ctx.moe_verify_layer(l, xs[i][l], out)
        ctx.sync()

    for i in range(warmup):
        iteration(i)
    torch.cuda.synchronize()
    st0 = ctx.expert_cache_stats()
    if args.copy_log:
        ctx.profile_begin(log_only=True)
    t_start = time.perf_counter()
    for i in range(warmup, n_it):
        iteration(i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    st1 = ctx.expert_cache_stats()
    stats = {key: st1[key] - st0[key] for key in st1}
    if args.copy_log:
        kinds = [r["kind"] for r in ctx.profile_collect(cap=500000) if r["kind"] in (1, 2)]
        json.dump({"blob_bytes": blob, "copy_kinds_in_issue_order": kinds, "iterations": steps}, open(args.copy_log, "w"))
        log("bench: wrote %d copy labels to %s" % (len(kinds), args.copy_log))
        L.close()
        D.close()
        return {"metric": "moe_verify_stack_tokens_per_s", "value": T * steps / elapsed, "unit": "tokens/s",
                "ms_per_step": elapsed * 1e3 / steps, "copy_log": args.copy_log, "cache_stats": stats}

    # profiled pass (events around every copy and every expert-GEMM launch) over a few more iterations
    n_prof = min(3, steps)
    ctx.profile_begin(per_kernel=True)     # verify-layer calls wait for copies between their kernels
    dctx.profile_begin(per_kernel=False)   # resident stand-in: one span per layer call, no events between kernels
    for i in range(n_it - n_prof, n_it):
        iteration(i)
    recs = ctx.profile_collect(cap=200000)
    pre = union([(r["t0"], r["t1"]) for r in recs if r["kind"] == 1])
    ond = union([(r["t0"], r["t1"]) for r in recs if r["kind"] == 2])
    drecs = dctx.profile_collect(cap=200000)
    # kernels executing on the compute stream: per-kernel spans of the offloaded stack, whole-call spans of the
    # resident draft stand-in (its calls never wait for a copy)
    busy = union([(r["t0"], r["t1"]) for r in recs if r["kind"] in (3, 4, 5, 6)] +
                 [(r["t0"], r["t1"]) for r in drecs if r["kind"] == 0])
    copy_ms = {"prefetch": measure(pre), "ondemand": measure(ond)}
    hidden = {"prefetch": intersect(pre, busy), "ondemand": intersect(ond, busy)}
    n_pre = sum(1 for r in recs if r["kind"] == 1)
    n_ond = sum(1 for r in recs if r["kind"] == 2)
    h2d_gbs = ((n_pre + n_ond) * blob / 1e9) / (max(measure(union(pre + ond)), 1e-9) * 1e-3)
    # time the compute stream spent, inside verify-layer calls, waiting for a copy to land: for cached experts
    # whose prefetch was still in flight (kind 7) and for on-demand loads (kinds 8, 9)
    wait_pre = sum(r["t1"] - r["t0"] for r in recs if r["kind"] == 7)
    wait_ond = sum(r["t1"] - r["t0"] for r in recs if r["kind"] in (8, 9))

    ms_per_step = elapsed * 1e3 / steps
    hits, misses = stats["hits"], stats["misses"]
    result = {
        "metric": "moe_verify_stack_tokens_per_s", "value": T * steps / elapsed, "unit": "tokens/s", "n_gpus": 1,
        "steps": steps, "warmup": warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": name, "layers": layers, "d_model": d, "d_ff": f, "n_experts": E, "top_k": k,
                   "n_shared": n_shared, "verify_tokens": T, "cache_slots_per_layer": spec["slots"], "cutoff_layer": cutoff,
                   "cutoff_suggested_by_policy": suggested, "policy_window": "one draft " + args.draft_window,
                   "t_comp_ms_per_draft_layer": t_comp_ms, "t_io_ms_per_expert": t_io_ms,
                   "draft_sigma": args.sigma, "pred_k": pred_k, "token_corr": args.token_corr, "sequences": args.sequences,
                   "distinct_blobs": wl.distinct, "prefetcher": args.prefetcher,
                   "draft_stage": "T-1 passes of a dense d x f SwiGLU FFN per layer (stand-in)"},
        "per_layer_verify_us_incl_stalls": ms_per_step * 1e3 / layers,
        "hit_rate": hits / max(hits + misses, 1), "cache_stats": stats,
        "h2d": {"link_peak_gbs_measured": link_gbs, "achieved_gbs_while_copying": h2d_gbs,
                "link_frac_of_measured_peak": h2d_gbs / link_gbs,
                "prefetch_copy_ms": copy_ms["prefetch"], "ondemand_copy_ms": copy_ms["ondemand"],
                "prefetch_hidden_frac": hidden["prefetch"] / max(copy_ms["prefetch"], 1e-9),
                "ondemand_hidden_frac": hidden["ondemand"] / max(copy_ms["ondemand"], 1e-9),
                "prefetch_wait_ms": wait_pre, "ondemand_wait_ms": wait_ond,
                "prefetch_unstalled_frac": 1.0 - wait_pre / max(copy_ms["prefetch"], 1e-9),
                "compute_busy_ms": measure(busy), "profiled_iterations": n_prof},
        "roofline": {"bound": "host-link", "achieved": h2d_gbs, "peak": link_gbs, "unit": "GB/s",
                     "frac": h2d_gbs / link_gbs, "traffic": None},
    }
    L.close()
    D.close()
    return result


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="", help="run only this workload (default: the composite line described above)")
    ap.add_argument("--batches", type=int, default=20, help="distinct synthetic token batches cycled through")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="composite line without the other layer shapes and the offloaded cell")
    ap.add_argument("--graph", action="store_true",
                    help="resident layer only: capture one pass over the batches in a HIP graph and time its replays")
    ap.add_argument("--resident", action="store_true",
                    help="time one layer of the workload's shape with every expert resident (compute-only number)")
    ap.add_argument("--token-corr", type=float, default=0.0, metavar="RHO",
                    help="correlation of the tokens of a sequence (x_t = rho*b_seq + sqrt(1-rho^2)*eps_t); 0 = independent")
    ap.add_argument("--sequences", type=int, default=1, help="sequences the verification batch is split into (with --token-corr)")
    ap.add_argument("--tokens", type=int, default=0, help="verification batch size T (0 = the workload's)")
    ap.add_argument("--slots", type=int, default=0, help="offload workloads: cache slots per layer (0 = the workload's)")
    ap.add_argument("--layers", type=int, default=0, help="offload workloads: number of layers (0 = the config's)")
    ap.add_argument("--cutoff", default="auto", help="offload workloads: cutoff layer L of the prefetcher (-1 = off, "
                    "'auto' (default) = the largest L the paper's memory/overlap constraints admit with the measured times)")
    ap.add_argument("--draft-window", default="pass", choices=["pass", "stage"],
                    help="offload workloads, --cutoff auto: the compute window of the policy's overlap constraint is one pass of "
                         "the draft stand-in over the layers, or the whole drafting stage of T-1 passes")
    ap.add_argument("--draft-ff", type=int, default=0, help="offload workloads: FFN width of the dense draft-layer stand-in (0 = d_ff)")
    ap.add_argument("--sigma", type=float, default=0.1, help="offload workloads: draft-noise std")
    ap.add_argument("--pred-k", type=int, default=0, help="offload workloads: k of the predictor (0 = top_k)")
    ap.add_argument("--prefetcher", default="worker", choices=["worker", "sync", "blocking", "none"],
                    help="offload workloads: worker = queue tasks to the library's prefetch thread (continuous prefetching); "
                         "sync = predict and prefetch on the caller's thread; blocking = sync + wait for the layer's copies "
                         "before the next draft layer (layer-triggered prefetch that synchronises I/O); none = on-demand only")
    ap.add_argument("--distinct", type=int, default=32, help="offload workloads: distinct expert blobs backing the stack")
    ap.add_argument("--copy-log", default="", metavar="PATH",
                    help="offload workloads: instead of the HIP-event pass, log the kind (1 prefetch, 2 on-demand) of every "
                         "expert copy of the timed iterations, in issue order, to PATH (labels for a rocprofv3 copy trace)")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="N",
                    help="only run N plain 1 GiB device copies (counter calibration for rocprofv3 --pmc) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on one GPU only (the path would shard by expert across GPUs, "
            "each GPU would own a subset of the experts, their cache slots and its own host link); --gpus %d is not supported" % args.gpus)
        sys.exit(2)

    import torch
    from paper_2510_10302_amd import workload as W

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        sys.exit(1)
    torch.cuda.set_device(0)
    if args.calibrate_copy:
        # a copy kernel of known traffic: reads 1 GiB, writes 1 GiB per launch (fp32 elementwise copy)
        src = torch.ones(2 ** 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(args.calibrate_copy):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy": args.calibrate_copy, "bytes_read": 2 ** 30, "bytes_written": 2 ** 30}))
        return

    composite = args.workload == ""
    name = args.workload or "c2_mixtral_8x7b"
    spec = dict(W.CONFIGS[name])
    if args.tokens:
        spec["T"] = args.tokens
    if args.slots and spec["slots"]:
        spec["slots"] = args.slots
    if spec["slots"] and not args.resident:
        print(json.dumps(run_offload(name, spec, args)), flush=True)
        return

    block, keep = run_resident(name, spec, args, args.steps, args.warmup, keep_for_cpu=not args.no_cpu_baseline)
    result = {"metric": "moe_verify_layer_tokens_per_s", "value": block["value"], "unit": "tokens/s", "n_gpus": 1,
              "steps": block["steps"], "warmup": block["warmup"], "ms_per_step": block["ms_per_step"],
              "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": block["dtype"], "data": "synthetic"}
    for key in ("verify_layer_us", "verify_layer_us_percentiles", "config", "kernels_ms", "expert_gemm_gbs",
                "layer_weight_streaming_gbs", "layer_frac_of_hbm_peak", "roofline"):
        result[key] = block[key]
    if keep is not None:
        result["cpu_baseline"] = cpu_baseline(keep[0], keep[1], spec["T"], spec["k"])
        if composite:
            # configuration 3 is a 32-layer stack of this layer shape
            result["cpu_baseline"]["stack_c3_mixtral_8x7b"] = {
                "stack_layers": 32, "stack_ms_scaled": result["cpu_baseline"]["ms_per_step"] * 32,
                "stack_tokens_per_s_scaled": spec["T"] / (result["cpu_baseline"]["ms_per_step"] * 1e-3 * 32),
                "sample": "the OpenMP per-layer time above scaled linearly to the 32 layers of the stack"}
        keep = None
    if composite and not args.no_extras:
        # the other single-GPU layer shapes (the Mixtral-8x22B layer is the largest configuration), shorter runs
        result["layers"] = {}
        for other in ("c4_deepseek_v2_lite", "c5_mixtral_8x22b"):
            ospec = dict(W.CONFIGS[other])
            oblock, okeep = run_resident(other, ospec, args, max(100, args.steps // 2), args.warmup,
                                         keep_for_cpu=not args.no_cpu_baseline)
            oblock.pop("dtype")
            if okeep is not None:
                oblock["cpu_baseline_stack"] = cpu_stack_estimate(okeep[0], okeep[1], ospec["T"], ospec["k"], ospec["layers"])
                okeep = None
            result["layers"][other] = oblock
        # the third part of the metric: one offloaded stack at the cutoff the policy admits
        oargs = argparse.Namespace(**vars(args))
        oargs.cutoff, oargs.sigma, oargs.pred_k, oargs.steps, oargs.warmup, oargs.prefetcher = "auto", 0.3, 1, 6, 2, "worker"
        oargs.draft_ff, oargs.draft_window = 11264, "pass"
        off = run_offload("c4_deepseek_v2_lite", dict(W.CONFIGS["c4_deepseek_v2_lite"]), oargs)
        result["h2d"] = dict(off["h2d"], workload=off["config"], hit_rate=off["hit_rate"], cache_stats=off["cache_stats"],
                             ms_per_iteration=off["ms_per_step"], stack_tokens_per_s=off["value"],
                             note="the cell where the paper's overlap constraint admits a cutoff on this machine; at the cache budgets "
                                  "and cutoffs of the benchmark's stack configurations (Mixtral shapes, cutoff 4/8/16) the stacks are "
                                  "link-bound and 2-14 % of the prefetch copy time is hidden (measured cells under profiles/)")
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
