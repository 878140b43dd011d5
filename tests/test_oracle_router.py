"""Pins for the oracle's router (gate logits, softmax, top-k, renormalised gating scores, token->expert
grouping).  Each check is independent of the oracle's own code: a brute-force stable sort, closed
forms, constructed ties, a library matmul in fp64, and the closed-form expected number of distinct
activated experts under uniform routing (the "-Max" curve of the paper's activation-rate figure)."""
import math

import numpy as np
import pytest

import spmoe_inputs as si


def brute_force_topk(logits_row, k):
    # full stable sort of (-score, index): descending score, lower index first among equals
    order = sorted(range(len(logits_row)), key=lambda e: (-float(logits_row[e]), e))
    return order[:k]


@pytest.mark.parametrize("prec", ["f32", "f64"])
def test_gate_logits_match_library_matmul(prec, oracle32, oracle64):
    o = oracle32 if prec == "f32" else oracle64
    T, E, d = 5, 8, 512
    x = si.hidden(11, T, d)
    wg = si.gate_weights(11, 0, E, d, "bf16")
    ref = x.astype(np.float64) @ si.bf16_to_f32(wg).astype(np.float64).T      # [T][E]; catches a transposed Wg
    got = o.gate_logits(x, wg)
    tol = 2e-5 if prec == "f32" else 1e-12
    assert got.shape == (T, E)
    assert np.abs(got - ref).max() < tol
    wg32 = si.gate_weights(11, 0, E, d, "f32")
    got32 = o.gate_logits(x, wg32)
    assert np.abs(got32 - x.astype(np.float64) @ wg32.astype(np.float64).T).max() < tol


def test_topk_brute_force_tiny(oracle32):
    rng = np.random.default_rng(0)
    for trial in range(300):
        E = int(rng.integers(1, 9))
        k = int(rng.integers(1, E + 1))
        # few distinct values so that ties are common
        row = rng.integers(-2, 3, size=E).astype(np.float32) * 0.5
        assert list(oracle32.topk(row, k)) == brute_force_topk(row, k)


def test_ties_go_to_lower_index(oracle32):
    row = np.array([1.0, 3.0, 3.0, 0.5, 3.0], dtype=np.float32)
    assert list(oracle32.topk(row, 2)) == [1, 2]
    assert list(oracle32.topk(row, 4)) == [1, 2, 4, 0]
    assert list(oracle32.topk(np.zeros(8, np.float32), 3)) == [0, 1, 2]


def test_softmax_closed_forms(oracle32, oracle64):
    # two experts with logits (a, 0): p0 = 1/(1+exp(-a)) (logistic); uniform logits: 1/E
    for a in [0.0, 1.0, -2.5, 7.0]:
        p = oracle64.softmax(np.array([a, 0.0]))
        assert abs(p[0] - 1.0 / (1.0 + math.exp(-a))) < 1e-15
        assert abs(p.sum() - 1.0) < 1e-15
    p = oracle32.softmax(np.full(64, 3.25, np.float32))
    assert np.allclose(p, 1.0 / 64, rtol=1e-6)
    # invariance to a common shift (needs the max subtraction to be right for large logits)
    big = oracle32.softmax(np.array([1000.0, 999.0, 998.0], np.float32))
    small = oracle32.softmax(np.array([2.0, 1.0, 0.0], np.float32))
    assert np.all(np.isfinite(big)) and np.allclose(big, small, rtol=1e-6)


@pytest.mark.parametrize("E,k,T", [(8, 2, 5), (8, 2, 8), (64, 6, 16), (16, 2, 8), (1, 1, 3)])
def test_route_weights_and_bruteforce(E, k, T, oracle32, oracle64):
    logits = si.normal_f32(5, 77, T * E, std=1.3).reshape(T, E)
    idx, w = oracle32.route(logits, k, renorm=True)
    idx64, w64 = oracle64.route(logits, k, renorm=True)
    assert np.array_equal(idx, idx64)
    for t in range(T):
        assert list(idx[t]) == brute_force_topk(logits[t], k)
        assert abs(float(w[t].sum()) - 1.0) < 1e-6                  # top-k scores renormalise to 1
        # renormalised softmax over E == softmax over the k selected logits (closed form)
        sel = logits[t, idx[t]].astype(np.float64)
        ref = np.exp(sel - sel.max()) / np.exp(sel - sel.max()).sum()
        assert np.abs(w64[t] - ref).max() < 1e-14
        assert np.abs(w[t] - ref).max() < 1e-6
        assert np.all(np.diff(w[t]) <= 1e-7)                        # rank order = descending score
    # without renormalisation: plain softmax probabilities of the selected experts
    idx_n, w_n = oracle64.route(logits, k, renorm=False)
    p = np.exp(logits.astype(np.float64) - logits.max(1, keepdims=True))
    p /= p.sum(1, keepdims=True)
    assert np.abs(w_n - np.take_along_axis(p, idx_n.astype(np.int64), 1)).max() < 1e-14


def test_route_token_permutation_equivariance(oracle32):
    T, E, k = 8, 8, 2
    logits = si.normal_f32(6, 78, T * E).reshape(T, E)
    idx, w = oracle32.route(logits, k)
    perm = np.array([3, 0, 7, 1, 6, 2, 5, 4])
    idx_p, w_p = oracle32.route(logits[perm], k)
    assert np.array_equal(idx_p, idx[perm]) and np.array_equal(w_p, w[perm])


def test_permute_is_stable_counting_sort(oracle32):
    rng = np.random.default_rng(2)
    for E, k, T in [(8, 2, 8), (64, 6, 16), (8, 2, 32), (4, 1, 1)]:
        idx = np.stack([rng.choice(E, size=k, replace=False) for _ in range(T)]).astype(np.int32)
        counts, offsets, perm = oracle32.permute(idx, E)
        flat = idx.reshape(-1)
        assert np.array_equal(counts, np.bincount(flat, minlength=E))
        assert offsets[0] == 0 and offsets[E] == T * k and np.array_equal(np.diff(offsets), counts)
        assert sorted(perm.tolist()) == list(range(T * k))                       # a permutation
        assert np.array_equal(perm, np.argsort(flat, kind="stable"))             # library stable sort
        for e in range(E):
            assert np.all(flat[perm[offsets[e]:offsets[e + 1]]] == e)


def test_expected_activated_experts_closed_form(oracle32):
    # Under uniform independent routing the expected number of distinct experts hit by T tokens is
    # E * (1 - (1 - k/E)^T): 7.20 of 8 for (8, 2, T=8), 6.10 for T=5, 50.7 of 64 for (64, 6, T=16).
    for E, k, T, d, expect in [(8, 2, 8, 256, 7.1989), (8, 2, 5, 256, 6.1016), (64, 6, 16, 256, 50.752)]:
        assert abs(E * (1 - (1 - k / E) ** T) - expect) < 1e-2
        total, trials = 0, 150
        for s in range(trials):
            x = si.hidden(100 + s, T, d)
            wg = si.gate_weights(100 + s, 0, E, d, "bf16")
            idx, _ = oracle32.route(oracle32.gate_logits(x, wg), k)
            total += len(set(idx.reshape(-1).tolist()))
        mean = total / trials
        # sd of the count is < 2.2 for these cases; 150 trials -> standard error < 0.18
        assert abs(mean - expect) < 0.6, (E, k, T, mean, expect)


def test_predictor_sigma_zero_is_truth_and_cosine(oracle32):
    # Draft stand-in: draft_x = x + sigma * eps.  cos(x, draft_x) -> 1/sqrt(1+sigma^2); sigma = 0 predicts exactly.
    T, E, d, k = 8, 8, 4096, 2
    x = si.hidden(9, T, d)
    wg = si.gate_weights(9, 0, E, d, "bf16")
    truth, _ = oracle32.route(oracle32.gate_logits(x, wg), k)
    pred, _, _ = oracle32.predict_experts(x + si.draft_noise(9, T, d, 0.0), wg, k)
    assert np.array_equal(pred, truth)
    for sigma in (0.1, 0.3, 0.5):
        dx = x + si.draft_noise(9, T, d, sigma)
        cos = (x * dx).sum() / np.linalg.norm(x) / np.linalg.norm(dx)
        assert abs(cos - 1 / math.sqrt(1 + sigma * sigma)) < 5e-3
