"""The pins must be able to fail: each plausible mistake is planted in a copy of the oracle's source
(on the CPU, in a temporary build), and at least one pin has to notice it.  The pins used here are the
same independent references as in test_oracle_router.py / test_oracle_ffn.py."""
import ctypes
import math
import os
import subprocess
import tempfile

import numpy as np
import pytest
import torch

import oracle as oracle_pkg
import spmoe_inputs as si

SRC = os.path.join(os.path.dirname(oracle_pkg.__file__), "spmoe_oracle.c")

MUTANTS = {
    "silu_sign": ("real silu = g / ((real)1 + real_exp(-g));", "real silu = g / ((real)1 + real_exp(g));"),
    "gate_up_swapped": ("h[n] = silu * u;", "h[n] = (u / ((real)1 + real_exp(-u))) * g;"),
    "down_transposed": ("acc += h[n] * wload(w_down, (size_t)i * f + n, wdtype);",
                        "acc += h[n] * wload(w_down, (size_t)n * d + i, wdtype);"),
    "gate_transposed": ("acc += (real)x[j] * wload(w, row * n + j, dtype);",
                        "acc += (real)x[j] * wload(w, (j * 7 + row) % (n * 2), dtype);"),
    "no_renorm": ("w[(size_t)t * k + r] = renorm ? pr / s : pr;", "w[(size_t)t * k + r] = pr;"),
    "tie_to_higher_index": ("if (best < 0 || scores[e] > scores[best]) best = e;",
                            "if (best < 0 || scores[e] >= scores[best]) best = e;"),
    "topk_smallest": ("if (best < 0 || scores[e] > scores[best]) best = e;",
                      "if (best < 0 || scores[e] < scores[best]) best = e;"),
    "softmax_no_max": ("p[e] = real_exp(logits[e] - m);", "p[e] = real_exp(logits[e]);"),
    "shared_dropped": ("for (int i = 0; i < d; ++i) ot[i] += y[i];", "for (int i = 0; i < d; ++i) ot[i] += 0 * y[i];"),
    "weight_dropped": ("for (int i = 0; i < d; ++i) ot[i] += g * y[i];", "for (int i = 0; i < d; ++i) ot[i] += y[i];"),
    "dropped_last_term": ("for (size_t j = 0; j < n; ++j) acc +=", "for (size_t j = 0; j + 1 < n; ++j) acc +="),
    "bf16_shift": ("uint32_t u = (uint32_t)((const uint16_t*)w)[i] << 16;", "uint32_t u = (uint32_t)((const uint16_t*)w)[i] << 15;"),
    "perm_unstable": ("if (idx[a] == e) perm[pos++] = a;", "if (idx[T * k - 1 - a] == e) perm[pos++] = T * k - 1 - a;"),
}


def _build(tmp, name, old, new):
    text = open(SRC).read()
    assert text.count(old) == 1, "mutation site for %s not found exactly once" % name
    path = os.path.join(tmp, name + ".c")
    open(path, "w").write(text.replace(old, new))
    so = os.path.join(tmp, name + ".so")
    subprocess.check_call(["gcc", "-O1", "-fPIC", "-shared", "-fopenmp", "-std=c99", "-DORACLE_REAL=double", path, "-o", so, "-lm"])
    o = oracle_pkg.Oracle.__new__(oracle_pkg.Oracle)
    o.precision, o.real, o.lib = "f64", np.float64, ctypes.CDLL(so)
    for fn in ("oracle_gate_logits", "oracle_softmax", "oracle_topk", "oracle_route", "oracle_permute",
               "oracle_expert_ffn", "oracle_moe_layer"):
        getattr(o.lib, fn).restype = None
    return o


def _f32(m):
    return si.bf16_to_f32(m) if m.dtype == np.uint16 else m


def _dense(x, wg, wu, wd):
    X = torch.from_numpy(np.asarray(x, np.float64))
    G, U, D = (torch.from_numpy(np.asarray(_f32(m), np.float64)) for m in (wg, wu, wd))
    return ((torch.nn.functional.silu(X @ G.T) * (X @ U.T)) @ D.T).numpy()


def pins_pass(o):
    """True iff the oracle object `o` passes this reduced set of independent pins."""
    try:
        # routing: library matmul for logits, stable sort for top-k incl. ties, closed-form weights
        T, E, d, k = 6, 8, 96, 2
        x = si.hidden(31, T, d)
        wg = si.gate_weights(31, 0, E, d, "bf16", std=0.5)
        logits = o.gate_logits(x, wg)
        if np.abs(logits - x.astype(np.float64) @ _f32(wg).astype(np.float64).T).max() > 1e-9:
            return False
        if list(o.topk(np.array([1.0, 3.0, 3.0, 0.5, 3.0]), 2)) != [1, 2]:
            return False
        big = o.softmax(np.array([1000.0, 999.0, 998.0]))
        if not np.all(np.isfinite(big)) or abs(big.sum() - 1) > 1e-12:
            return False
        idx, w = o.route(logits, k)
        for t in range(T):
            order = sorted(range(E), key=lambda e: (-logits[t, e], e))[:k]
            if list(idx[t]) != order or abs(w[t].sum() - 1) > 1e-12:
                return False
        rng = np.random.default_rng(1)
        ridx = np.stack([rng.choice(E, size=k, replace=False) for _ in range(T)]).astype(np.int32)
        if not np.array_equal(o.permute(ridx, E)[2], np.argsort(ridx.reshape(-1), kind="stable")):
            return False
        # experts: closed form, library dense FFN on rectangular matrices, Eq. 1 with shared experts
        one = np.ones((1, 1), np.float32)
        if abs(o.expert_ffn(np.array([-2.0], np.float32), one, 3 * one, 0.5 * one)[0]
               - 0.5 * (-2.0 / (1.0 + math.exp(2.0))) * (-6.0)) > 1e-12:
            return False
        f = 160
        ex = [si.expert_weights(31, 0, e, d, f, "bf16", std=0.05) for e in range(E)]
        sh = [si.expert_weights(31, 0, 0, d, f, "bf16", std=0.05, shared=True)]
        if np.linalg.norm(o.expert_ffn(x[0], *ex[3]) - _dense(x[:1], *ex[3])[0]) > 1e-9:
            return False
        ref = np.zeros((T, d))
        for t in range(T):
            order = sorted(range(E), key=lambda e: (-logits[t, e], e))[:k]
            z = np.exp(logits[t, order] - logits[t, order].max())
            for r, e in enumerate(order):
                ref[t] += z[r] / z.sum() * _dense(x[t:t + 1], *ex[e])[0]
            ref[t] += _dense(x[t:t + 1], *sh[0])[0]
        got = o.moe_layer(x, wg, ex, k, shared=sh)["out"]
        return bool(np.linalg.norm(got - ref) / np.linalg.norm(ref) < 1e-9)
    except Exception:
        return False


def test_unmodified_oracle_passes_the_pins(oracle64):
    assert pins_pass(oracle64)


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_planted_mistake_is_caught(name):
    old, new = MUTANTS[name]
    with tempfile.TemporaryDirectory() as tmp:
        mutant = _build(tmp, name, old, new)
        assert not pins_pass(mutant), "the pins did not notice the planted mistake '%s'" % name
