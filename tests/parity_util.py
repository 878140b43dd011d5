"""Helpers shared by the GPU parity tests: run the library and the oracle on the same seeded inputs."""
import numpy as np

import spmoe_inputs as si

NEAR_TIE = 1e-5     # logit gap below which a routing decision is a near-tie (listed, not counted as exact)
REL_L2_BF16 = 1e-2  # bound on relative L2 output error for bf16 weights with fp32 accumulation
REL_L2_F32 = 1e-4   # self-imposed bound for fp32 weights
# Element-wise bound beside the norm: |gpu - ref| <= c * rms(ref row).  An output element is a sum of f (then k)
# products whose relative rounding errors are independent, so its absolute error is close to normal with standard
# deviation eps * rms(row), eps being the relative L2 error of the row (measured 2.3e-3 ... 3.1e-3 for bf16).
# The largest of up to 2e5 such errors sits near 5 standard deviations, 1.5e-2 * rms; c = 3e-2 leaves a factor two
# and is 30 times smaller than a typical element, so one dropped, duplicated or garbage element is caught even
# where it would hide inside the L2 norm of a large tensor.
ELEM_C_BF16 = 3e-2
ELEM_C_F32 = 2e-4


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
    worst = check_elements(gpu["out"], ref["out"], good, ELEM_C_F32 if out_tol <= REL_L2_F32 else ELEM_C_BF16, out_tol)
    return dict(exact=exact, near_ties=near, rel_l2=err, max_elem_err_over_rms=worst)


def check_elements(out_gpu, out_ref, rows, c, row_tol):
    """Every listed token row within row_tol (relative L2) and every element of it within c * rms(reference row).
    Returns the largest |gpu - ref| / rms(row) seen."""
    worst = 0.0
    for t in rows:
        g, r = np.asarray(out_gpu[t], np.float64), np.asarray(out_ref[t], np.float64)
        rms = max(float(np.sqrt(np.mean(r * r))), 1e-300)
        dev = np.abs(g - r) / rms
        i = int(np.argmax(dev))
        assert dev[i] <= c, "token %d element %d: |gpu - ref| = %.3e * rms(row) > %.1e (gpu %.6g, ref %.6g)" % (
            t, i, dev[i], c, g[i], r[i])
        row_err = float(np.linalg.norm(g - r) / max(np.linalg.norm(r), 1e-300))
        assert row_err < row_tol, "token %d: rel L2 %.3e >= %.1e" % (t, row_err, row_tol)
        worst = max(worst, float(dev[i]))
    return worst
