"""Helpers shared by the GPU parity tests: run the library and the oracle on the same seeded inputs."""
import numpy as np

import spmoe_inputs as si

NEAR_TIE = 1e-5     # logit gap below which a routing decision is a near-tie (listed, not counted as exact)
REL_L2_BF16 = 1e-2  # bound on relative L2 output error for bf16 weights with fp32 accumulation
REL_L2_F32 = 1e-4   # self-imposed bound for fp32 weights


def rel_l2(a, b):
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def routing_report(idx_gpu, idx_ref, logits_ref, k):
    """Per token: exact match, or a near-tie (some adjacent gap among the top k+1 reference logits
    below NEAR_TIE), or a real mismatch.  Returns (n_exact, near_tie_tokens, mismatch_tokens)."""
    T = idx_ref.shape[0]
    exact, near, bad = 0, [], []
    for t in range(T):
        if np.array_equal(idx_gpu[t], idx_ref[t]):
            exact += 1
            continue
        top = np.sort(np.asarray(logits_ref[t], np.float64))[::-1][: k + 1]
        gaps = -np.diff(top)
        (near if gaps.size and gaps.min() < NEAR_TIE else bad).append(t)
    return exact, near, bad


def oracle_layer(oracle, wl, layer, x):
    return oracle.moe_layer(x, wl.gate[layer], wl.layer_experts(layer), wl.k, shared=wl.shared[layer], renorm=True)


def gpu_layer(loaded, layer, x):
    """Runs spmoe_moe_verify_layer and spmoe_gate_topk on x (numpy [T][d]); returns numpy results."""
    import torch
    cfg, ctx = loaded.cfg, loaded.ctx
    T = x.shape[0]
    dx = torch.from_numpy(np.ascontiguousarray(x, np.float32)).cuda()
    out = torch.full((T, cfg.d_model), float("nan"), dtype=torch.float32, device="cuda")
    ctx.moe_verify_layer(layer, dx, out)
    idx = torch.full((T, cfg.top_k), -1, dtype=torch.int32, device="cuda")
    w = torch.zeros((T, cfg.top_k), dtype=torch.float32, device="cuda")
    logits = torch.zeros((T, cfg.n_experts), dtype=torch.float32, device="cuda")
    ctx.gate_topk(layer, dx, cfg.top_k, idx, w, logits)
    ctx.sync()
    torch.cuda.synchronize()
    return dict(out=out.cpu().numpy(), idx=idx.cpu().numpy(), w=w.cpu().numpy(), logits=logits.cpu().numpy())


def check_layer(gpu, ref, k, out_tol, w_tol=2e-5, logit_tol=2e-4):
    """Asserts the parity bar: indices bit-exact outside near-ties, outputs within out_tol (rel. L2)."""
    exact, near, bad = routing_report(gpu["idx"], ref["idx"], ref["logits"], k)
    assert not bad, "routing mismatch on tokens %s" % bad
    assert np.abs(gpu["logits"] - ref["logits"]).max() < logit_tol
    T = ref["idx"].shape[0]
    good = [t for t in range(T) if t not in near]
    assert np.abs(gpu["w"][good] - ref["w"][good]).max() < w_tol
    assert np.abs(gpu["w"].sum(1) - 1).max() < 1e-5
    err = rel_l2(gpu["out"][good], ref["out"][good])
    assert np.all(np.isfinite(gpu["out"]))
    assert err < out_tol, "rel L2 %.3e >= %.1e" % (err, out_tol)
    return dict(exact=exact, near_ties=near, rel_l2=err)
