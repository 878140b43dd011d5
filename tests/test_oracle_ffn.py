"""Pins for the oracle's expert FFN and the weighted combination of Eq. 1.  References used here are
independent of the oracle: torch's fp64 matmul + silu for the dense special case, closed forms,
and invariants (identical experts, linearity in W_down, zero W_down, token order, shared experts)."""
import math

import numpy as np
import pytest
import torch

import spmoe_inputs as si


def dense_swiglu_fp64(x, wg, wu, wd):
    """Textbook dense SwiGLU FFN through torch (fp64): W_down (silu(W_gate x) * (W_up x))."""
    X = torch.from_numpy(np.asarray(x, dtype=np.float64))
    G, U, D = (torch.from_numpy(np.asarray(m, dtype=np.float64)) for m in (wg, wu, wd))
    h = torch.nn.functional.silu(X @ G.T) * (X @ U.T)
    return (h @ D.T).numpy()


def as_f32(m):
    return si.bf16_to_f32(m) if m.dtype == np.uint16 else m


def rel_l2(a, b):
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    return np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300)


def test_silu_closed_form_one_by_one(oracle64):
    # d = f = 1: E(x) = wd * silu(wg*x) * (wu*x).  With wg = wu = wd = 1 and x = 1: silu(1) = 1/(1+e^-1).
    one = np.ones((1, 1), np.float32)
    y = oracle64.expert_ffn(np.array([1.0], np.float32), one, one, one)
    assert abs(y[0] - 1.0 / (1.0 + math.exp(-1.0))) < 1e-15
    # x = -2, wg = 1, wu = 3, wd = 0.5 -> 0.5 * (-2/(1+e^2)) * (-6)
    y = oracle64.expert_ffn(np.array([-2.0], np.float32), one, 3 * one, 0.5 * one)
    assert abs(y[0] - 0.5 * (-2.0 / (1.0 + math.exp(2.0))) * (-6.0)) < 1e-15
    # gate and up are not interchangeable: swapping them changes the value
    y_swapped = oracle64.expert_ffn(np.array([-2.0], np.float32), 3 * one, one, 0.5 * one)
    assert abs(y_swapped[0] - y[0]) > 1e-3


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("d,f", [(64, 96), (512, 1024), (96, 32)])
def test_expert_ffn_vs_library_dense(dtype, d, f, oracle32, oracle64):
    # rectangular, asymmetric matrices: a transposed operand or swapped matrix cannot pass
    wg, wu, wd = si.expert_weights(21, 0, 3, d, f, dtype, std=0.05)
    x = si.hidden(21, 1, d)[0]
    ref = dense_swiglu_fp64(x[None], as_f32(wg), as_f32(wu), as_f32(wd))[0]
    assert rel_l2(oracle64.expert_ffn(x, wg, wu, wd), ref) < 1e-13
    assert rel_l2(oracle32.expert_ffn(x, wg, wu, wd), ref) < 5e-6


def test_single_expert_layer_is_dense_ffn(oracle32, oracle64):
    # E = 1, k = 1: the gating score renormalises to exactly 1 and the block is a dense SwiGLU FFN
    T, d, f = 5, 128, 192
    x = si.hidden(3, T, d)
    wgate = si.gate_weights(3, 0, 1, d, "bf16")
    ex = [si.expert_weights(3, 0, 0, d, f, "bf16", std=0.05)]
    ref = dense_swiglu_fp64(x, *(as_f32(m) for m in ex[0]))
    r64 = oracle64.moe_layer(x, wgate, ex, k=1)
    r32 = oracle32.moe_layer(x, wgate, ex, k=1)
    assert np.all(r64["w"] == 1.0) and np.all(r64["idx"] == 0)
    assert rel_l2(r64["out"], ref) < 1e-13
    assert rel_l2(r32["out"], ref) < 5e-6


def test_identical_experts_give_dense_ffn_whatever_the_routing(oracle64):
    T, d, f, E, k = 6, 64, 96, 8, 2
    x = si.hidden(4, T, d)
    wgate = si.gate_weights(4, 0, E, d, "bf16", std=0.5)
    one = si.expert_weights(4, 0, 0, d, f, "bf16", std=0.05)
    r = oracle64.moe_layer(x, wgate, [one] * E, k=k)
    assert len(set(r["idx"].reshape(-1).tolist())) > 2           # routing is not trivial
    ref = dense_swiglu_fp64(x, *(as_f32(m) for m in one))
    assert rel_l2(r["out"], ref) < 1e-13                          # because the gating scores sum to 1


def test_layer_equals_weighted_sum_of_library_experts(oracle64, oracle32):
    # Eq. 1 assembled outside the oracle: routing from brute force, experts from torch fp64.
    T, d, f, E, k = 5, 64, 96, 8, 2
    x = si.hidden(5, T, d)
    wgate = si.gate_weights(5, 0, E, d, "bf16", std=0.5)
    ex = [si.expert_weights(5, 0, e, d, f, "bf16", std=0.05) for e in range(E)]
    sh = [si.expert_weights(5, 0, s, d, f, "bf16", std=0.05, shared=True) for s in range(2)]
    logits = x.astype(np.float64) @ as_f32(wgate).astype(np.float64).T
    ref = np.zeros((T, d))
    for t in range(T):
        order = sorted(range(E), key=lambda e: (-logits[t, e], e))[:k]
        z = np.exp(logits[t, order] - logits[t, order].max())
        g = z / z.sum()
        for r, e in enumerate(order):
            ref[t] += g[r] * dense_swiglu_fp64(x[t:t + 1], *(as_f32(m) for m in ex[e]))[0]
        for s in sh:
            ref[t] += dense_swiglu_fp64(x[t:t + 1], *(as_f32(m) for m in s))[0]     # shared experts: weight 1
    r = oracle64.moe_layer(x, wgate, ex, k=k, shared=sh)
    assert rel_l2(r["out"], ref) < 1e-13
    assert rel_l2(oracle32.moe_layer(x, wgate, ex, k=k, shared=sh)["out"], ref) < 5e-6
    # leaving the shared experts out, or not renormalising, must be visible
    assert rel_l2(oracle64.moe_layer(x, wgate, ex, k=k)["out"], ref) > 1e-2
    assert rel_l2(oracle64.moe_layer(x, wgate, ex, k=k, shared=sh, renorm=False)["out"], ref) > 1e-3


def test_linearity_and_zero_in_w_down(oracle64):
    T, d, f, E, k = 4, 64, 96, 4, 2
    x = si.hidden(6, T, d)
    wgate = si.gate_weights(6, 0, E, d, "f32", std=0.5)
    ex = [si.expert_weights(6, 0, e, d, f, "f32", std=0.05) for e in range(E)]
    base = oracle64.moe_layer(x, wgate, ex, k=k)["out"]
    scaled = [(g, u, (2.5 * dn).astype(np.float32)) for g, u, dn in ex]
    assert rel_l2(oracle64.moe_layer(x, wgate, scaled, k=k)["out"], 2.5 * base) < 1e-7
    zero = [(g, u, np.zeros_like(dn)) for g, u, dn in ex]
    assert np.all(oracle64.moe_layer(x, wgate, zero, k=k)["out"] == 0.0)


def test_token_order_equivariance(oracle32):
    T, d, f, E, k = 8, 64, 96, 8, 2
    x = si.hidden(7, T, d)
    wgate = si.gate_weights(7, 0, E, d, "bf16", std=0.5)
    ex = [si.expert_weights(7, 0, e, d, f, "bf16", std=0.05) for e in range(E)]
    r = oracle32.moe_layer(x, wgate, ex, k=k)
    perm = np.array([5, 2, 7, 0, 1, 6, 3, 4])
    rp = oracle32.moe_layer(x[perm], wgate, ex, k=k)
    assert np.array_equal(rp["out"], r["out"][perm])              # bit-identical: tokens are independent
    assert np.array_equal(rp["idx"], r["idx"][perm])


def test_fp32_oracle_close_to_fp64_on_small_config(oracle32, oracle64):
    # benchmark configuration 1: d_model 512, d_ff 1024, 8 experts, top-2, 5 tokens, fp32 weights, seed 0
    T, d, f, E, k = 5, 512, 1024, 8, 2
    x = si.hidden(0, T, d)
    wgate = si.gate_weights(0, 0, E, d, "f32")
    ex = [si.expert_weights(0, 0, e, d, f, "f32") for e in range(E)]
    r32 = oracle32.moe_layer(x, wgate, ex, k=k)
    r64 = oracle64.moe_layer(x, wgate, ex, k=k)
    assert np.array_equal(r32["idx"], r64["idx"])
    assert rel_l2(r32["out"], r64["out"]) < 2e-6
    assert np.abs(r32["logits"] - r64["logits"]).max() < 1e-5


def test_expert_byte_sizes_match_paper():
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "expert_sizes.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for name, d, f, b, mib in rows:
        d, f, b = int(d), int(f), int(b)
        wg, wu, wd = (d * f, d * f, d * f)
        assert (wg + wu + wd) * b == float(mib) * 2 ** 20, name
