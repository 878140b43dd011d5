#!/usr/bin/env python3
"""Benchmark of the SP-MoE verify-layer hot path on one MI355X.

A step = one pass of the whole hot path (gate/top-k/grouping -> grouped gate+up GEMM -> grouped down
GEMM -> weighted combine) over one verification batch of synthetic tokens, all expert weights already
resident in HBM when the timed region starts.  The default workload is the Mixtral-8x7B-shaped layer
(d_model 4096, d_ff 14336, 8 experts, top-2, bf16 weights, 8 tokens).  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2_mixtral_8x7b]
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


def profiled_traffic(workload, key):
    """HBM bytes per launch of the dominant kernel, as measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
    (scaled by a copy-kernel calibration) and recorded in profiles/verify_layer_<workload>.txt; None if absent."""
    path = os.path.join(ROOT, "profiles", "verify_layer_%s.txt" % workload)
    try:
        for line in open(path):
            if line.startswith(key + ":"):
                return int(line.split(":")[1])
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c2_mixtral_8x7b")
    ap.add_argument("--batches", type=int, default=20, help="distinct synthetic token batches cycled through")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="N",
                    help="only run N plain 1 GiB device copies (counter calibration for rocprofv3 --pmc) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on one GPU only (the path would shard by expert across GPUs, "
            "see DESIGN.md); --gpus %d is not supported" % args.gpus)
        sys.exit(2)

    import numpy as np
    import torch
    import spmoe_inputs as si
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
    spec = dict(W.CONFIGS[args.workload])
    d, f, E, k, T = spec["d"], spec["f"], spec["E"], spec["k"], spec["T"]
    n_shared = spec["shared"]
    # one layer, every expert resident: the compute-only verify layer at the real layer shape
    t0 = time.time()
    wl = W.Workload(d=d, f=f, E=E, k=k, shared=n_shared, dtype=spec["dtype"], layers=1, seed=0)
    cfg = W.make_config(wl, max_tokens=T)
    L = W.Loaded(wl, cfg)
    log("bench: workload %s built in %.1f s (expert blob %.1f MiB)" % (args.workload, time.time() - t0,
                                                                       W.sp.expert_blob_bytes(cfg) / 2 ** 20))
    ctx = L.ctx
    elem = 2 if spec["dtype"] == "bf16" else 4
    xs_host = [si.hidden(1000 + i, T, d) for i in range(args.batches)]
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

    for i in range(args.warmup):
        step(i)
    ctx.sync()
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for i in range(args.steps):
        step(i)
    ctx.sync()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    ms_per_step = elapsed * 1e3 / args.steps
    tokens_per_s = T * args.steps / elapsed

    # per-kernel durations from HIP events on the compute stream (separate pass: the events sit between kernels)
    kms = np.zeros(4)
    bytes_gu = bytes_dn = 0.0
    n_prof = min(args.steps, 5 * len(xs))
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
    log("bench: kernels ms  route %.4f  gate_up %.4f  down %.4f  combine %.4f | gate_up %.0f GB/s, down %.0f GB/s, "
        "both %.0f GB/s, mean active experts %.2f" % (kms[0], kms[1], kms[2], kms[3], gu_gbs, dn_gbs, both_gbs,
                                                       float(np.mean(e_act))))

    result = {
        "metric": "moe_verify_layer_tokens_per_s",
        "value": tokens_per_s,
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "verify_layer_us": ms_per_step * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": spec["dtype"],
        "data": "synthetic",
        "config": {"workload": args.workload, "d_model": d, "d_ff": f, "n_experts": E, "top_k": k, "n_shared": n_shared,
                   "verify_tokens": T, "experts_resident": True, "mean_active_experts": float(np.mean(e_act))},
        "kernels_ms": {"route": float(kms[0]), "gate_up": float(kms[1]), "down": float(kms[2]), "combine": float(kms[3])},
        "expert_gemm_gbs": {"gate_up": gu_gbs, "down": dn_gbs, "both": both_gbs},
        "roofline": {"bound": "hbm", "kernel": "expert_gemm_kernel<gate_up>", "achieved": gu_gbs, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": gu_gbs / HBM_PEAK_GBS, "algorithmic_bytes": bytes_gu,
                     "traffic": profiled_traffic(args.workload, "gate_up_traffic_bytes_per_launch")},
    }

    if not args.no_cpu_baseline:
        import oracle
        orc = oracle.Oracle("f32")
        cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        t1 = time.perf_counter()
        n_cpu = 0
        while n_cpu < len(xs_host) and (n_cpu == 0 or time.perf_counter() - t1 < 10.0):
            orc.moe_layer(xs_host[n_cpu], wl.gate[0], wl.layer_experts(0), k, shared=wl.shared[0])
            n_cpu += 1
        cpu_s = time.perf_counter() - t1
        result["cpu_baseline"] = {"value": T * n_cpu / cpu_s, "unit": "tokens/s", "cores": cores, "kind": "oracle",
                                  "sample": "%d verify batch(es) of %d tokens of the same layer, fp32 C oracle, "
                                            "one OpenMP loop over FFN rows" % (n_cpu, T),
                                  "ms_per_step": cpu_s * 1e3 / n_cpu}
    L.close()
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
