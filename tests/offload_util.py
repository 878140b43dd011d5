"""Helper of the GPU tests of offloaded stacks: drives the library through drafting stages (per-draft-token
prediction + prefetch tasks, Alg. 1 / Alg. 2) and verification passes (teacher-forced seeded x_l per layer),
with the CPU oracle (routing, outputs) and the reference cache/queue model (queue contents, statistics) run
beside every call."""
import numpy as np

import spmoe_inputs as si
from oracle.cache_model import rank_predicted
from parity_util import NEAR_TIE, REL_L2_BF16, check_layer, gpu_layer, oracle_layer

STAT_KEYS = ("hits", "misses", "evictions", "prefetch_issued", "prefetch_used", "prefetch_wasted", "ondemand_loads")


def ranked_prediction(oracle, draft, gate, pred_k, E):
    """Alg. 1's prediction for the draft states of one task, on the oracle: top-pred_k experts per state, ranked
    most-voted first, then larger summed probability, then lower index.  Returns (ranking, smallest logit gap that
    decided a selection)."""
    pidx, plog, pp = oracle.predict_experts(draft, gate, pred_k)
    gap = np.inf
    for t in range(draft.shape[0]):
        top = np.sort(np.asarray(plog[t], np.float64))[::-1][: pred_k + 1]
        if top.size > 1:
            gap = min(gap, float((-np.diff(top)).min()))
    return rank_predicted(pidx, pp, E), gap


def run_offloaded_stack(L, wl, model, oracle, layers, T, sigma, pred_k, seed, iterations, mode,
                        tokens_per_task=1, out_tol=REL_L2_BF16, collect_outputs=None):
    """One drafting stage + one verification pass per iteration, cache state carried from iteration to iteration.

    mode: "sync" (spmoe_predict_experts + spmoe_prefetch on the caller's thread; the predicted list itself is
    compared), "blocking" (as sync, then spmoe_sync after every task) or "worker" (spmoe_predict_prefetch_async; the
    queue contents are compared after every drafting pass, which also waits for the worker).
    Returns per-layer reports of check_layer."""
    import torch
    ctx, E, d = L.ctx, wl.E, wl.d
    reports = []
    for it in range(iterations):
        xs = [si.hidden(seed, T, d, iteration=it, layer=l) for l in range(layers)]
        drafts = [xs[l] + si.draft_noise(seed, T, d, sigma, iteration=it, layer=l) for l in range(layers)]
        ddev = [torch.from_numpy(dr).cuda() for dr in drafts]
        for j in range(0, T - 1, tokens_per_task):                      # drafting stage: T - 1 draft tokens
            rows = slice(j, min(j + tokens_per_task, T - 1))
            for l in range(layers):
                ranked, gap = ranked_prediction(oracle, drafts[l][rows], wl.gate[l], pred_k, E)
                assert gap >= NEAR_TIE, "seeded draft state with a near-tie in the prediction (gap %.2e): pick another seed" % gap
                want = model.filter_cached(l, ranked)
                if mode == "worker":
                    ctx.predict_prefetch_async(l, ddev[l][rows])
                else:
                    ids = ctx.predict_experts(l, ddev[l][rows])
                    assert ids == want, (it, j, l, ids, want)
                    ctx.prefetch(l, ids)
                    if mode == "blocking":
                        ctx.sync()
                model.prefetch(l, want)
                if mode != "worker":
                    assert ctx.expert_cache_contents(l) == model.contents(l), (it, j, l)
            if mode == "worker":
                for l in range(layers):
                    assert ctx.expert_cache_contents(l) == model.contents(l), (it, j, l)
        for l in range(layers):                                           # verification pass
            g = gpu_layer(L, l, xs[l])
            ref = oracle_layer(oracle, wl, l, xs[l])
            rep = check_layer(g, ref, wl.k, out_tol)
            assert not rep["near_ties"], "seeded batch with a routing near-tie: pick another seed"
            if collect_outputs is not None:
                collect_outputs.append(g["out"])
            model.verify(l, sorted(set(ref["idx"].reshape(-1).tolist())))
            assert ctx.expert_cache_contents(l) == model.contents(l), (it, l)
            for e in range(E):
                assert (ctx.expert_cache_lookup(l, e) >= 0) == (e in model.contents(l))
            rep.update(iteration=it, layer=l)
            reports.append(rep)
    st = ctx.expert_cache_stats()
    for key in STAT_KEYS:
        assert st[key] == model.stats[key], (key, st, model.stats)
    blob = 3 * wl.d * wl.f * (2 if wl.dtype == "bf16" else 4)
    assert st["h2d_bytes_prefetch"] == st["prefetch_issued"] * blob
    assert st["h2d_bytes_ondemand"] == st["ondemand_loads"] * blob
    return reports
