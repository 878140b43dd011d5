"""CPU oracle of the SP-MoE hot path: ctypes wrapper over ``spmoe_oracle.c``.  TEST INFRASTRUCTURE.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may import
this package.  It does not import, load or call anything of the GPU library.

``Oracle("f32")`` is the fp32 oracle; ``Oracle("f64")`` is the same source built with
``real = double``, used to bound the fp32 oracle's rounding error and as a tighter reference.
bf16 weights are passed as ``uint16`` bit patterns, fp32 weights as ``float32`` arrays, all in the
canonical row-major layout (Wg[E][d]; W_gate[f][d], W_up[f][d], W_down[d][f]).
"""
import ctypes
import os
import subprocess

import numpy as np

from .cache_model import CacheModel  # noqa: F401  (re-export)

_DIR = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_DIR, "spmoe_oracle.c")
_SO = {"f32": os.path.join(_DIR, "libspmoe_oracle_f32.so"),
       "f64": os.path.join(_DIR, "libspmoe_oracle_f64.so")}
_CTYPE = {"f32": "float", "f64": "double"}
_NP = {"f32": np.float32, "f64": np.float64}

F32, BF16 = 0, 1


def build():
    """Compile both precisions of the oracle with gcc (host code only)."""
    for prec, so in _SO.items():
        cmd = ["gcc", "-O2", "-fPIC", "-shared", "-fopenmp", "-std=c99", "-ffp-contract=off",
               "-DORACLE_REAL=" + _CTYPE[prec], _SRC, "-o", so, "-lm"]
        subprocess.check_call(cmd)


def _wdtype(a):
    if a.dtype == np.uint16:
        return BF16
    if a.dtype == np.float32:
        return F32
    raise TypeError("weights must be uint16 (bf16 bits) or float32, got %s" % a.dtype)


def _ptr_array(arrays):
    arr = (ctypes.c_void_p * max(len(arrays), 1))()
    for i, a in enumerate(arrays):
        assert a.flags.c_contiguous
        arr[i] = a.ctypes.data
    return arr


class Oracle:
    def __init__(self, precision="f32"):
        if not os.path.exists(_SO[precision]):
            build()
        self.precision = precision
        self.real = _NP[precision]
        self.lib = ctypes.CDLL(_SO[precision])
        assert self.lib.oracle_real_bytes() == np.dtype(self.real).itemsize
        for name in ("oracle_gate_logits", "oracle_softmax", "oracle_topk", "oracle_route",
                     "oracle_permute", "oracle_expert_ffn", "oracle_moe_layer"):
            getattr(self.lib, name).restype = None

    # -- routing ------------------------------------------------------------------------------
    def gate_logits(self, x, wg):
        x = np.ascontiguousarray(x, dtype=np.float32)
        T, d = x.shape
        E = wg.shape[0]
        assert wg.shape == (E, d) and wg.flags.c_contiguous
        logits = np.empty((T, E), dtype=self.real)
        self.lib.oracle_gate_logits(ctypes.c_void_p(x.ctypes.data), ctypes.c_void_p(wg.ctypes.data),
                                    _wdtype(wg), T, E, d, ctypes.c_void_p(logits.ctypes.data))
        return logits

    def softmax(self, logits_row):
        lg = np.ascontiguousarray(logits_row, dtype=self.real)
        p = np.empty_like(lg)
        self.lib.oracle_softmax(ctypes.c_void_p(lg.ctypes.data), lg.size, ctypes.c_void_p(p.ctypes.data))
        return p

    def topk(self, scores_row, k):
        s = np.ascontiguousarray(scores_row, dtype=self.real)
        idx = np.empty(k, dtype=np.int32)
        self.lib.oracle_topk(ctypes.c_void_p(s.ctypes.data), s.size, k, ctypes.c_void_p(idx.ctypes.data))
        return idx

    def route(self, logits, k, renorm=True):
        lg = np.ascontiguousarray(logits, dtype=self.real)
        T, E = lg.shape
        idx = np.empty((T, k), dtype=np.int32)
        w = np.empty((T, k), dtype=self.real)
        self.lib.oracle_route(ctypes.c_void_p(lg.ctypes.data), T, E, k, int(bool(renorm)),
                              ctypes.c_void_p(idx.ctypes.data), ctypes.c_void_p(w.ctypes.data))
        return idx, w

    def permute(self, idx, E):
        idx = np.ascontiguousarray(idx, dtype=np.int32)
        T, k = idx.shape
        counts = np.empty(E, dtype=np.int32)
        offsets = np.empty(E + 1, dtype=np.int32)
        perm = np.empty(T * k, dtype=np.int32)
        self.lib.oracle_permute(ctypes.c_void_p(idx.ctypes.data), T, k, E, ctypes.c_void_p(counts.ctypes.data),
                                ctypes.c_void_p(offsets.ctypes.data), ctypes.c_void_p(perm.ctypes.data))
        return counts, offsets, perm

    # -- experts ------------------------------------------------------------------------------
    def expert_ffn(self, x_row, w_gate, w_up, w_down):
        x = np.ascontiguousarray(x_row, dtype=np.float32)
        f, d = w_gate.shape
        assert x.shape == (d,) and w_up.shape == (f, d) and w_down.shape == (d, f)
        assert w_gate.flags.c_contiguous and w_up.flags.c_contiguous and w_down.flags.c_contiguous
        assert w_gate.dtype == w_up.dtype == w_down.dtype
        y = np.empty(d, dtype=self.real)
        self.lib.oracle_expert_ffn(ctypes.c_void_p(x.ctypes.data), ctypes.c_void_p(w_gate.ctypes.data),
                                   ctypes.c_void_p(w_up.ctypes.data), ctypes.c_void_p(w_down.ctypes.data),
                                   _wdtype(w_gate), d, f, ctypes.c_void_p(y.ctypes.data))
        return y

    def moe_layer(self, x, wg, experts, k, shared=(), renorm=True):
        """experts / shared: sequences of (W_gate[f][d], W_up[f][d], W_down[d][f]).
        Returns dict(out[T][d], idx[T][k], w[T][k], logits[T][E])."""
        x = np.ascontiguousarray(x, dtype=np.float32)
        T, d = x.shape
        E = len(experts)
        f = experts[0][0].shape[0]
        assert wg.shape == (E, d) and wg.flags.c_contiguous
        wdt = _wdtype(wg)
        for trip in list(experts) + list(shared):
            assert trip[0].shape == (f, d) and trip[1].shape == (f, d) and trip[2].shape == (d, f)
            assert all(_wdtype(m) == wdt for m in trip)
        out = np.empty((T, d), dtype=self.real)
        idx = np.empty((T, k), dtype=np.int32)
        w = np.empty((T, k), dtype=self.real)
        logits = np.empty((T, E), dtype=self.real)
        self.lib.oracle_moe_layer(
            ctypes.c_void_p(x.ctypes.data), T, d, f, E, k, len(shared), int(bool(renorm)), wdt,
            ctypes.c_void_p(wg.ctypes.data),
            _ptr_array([e[0] for e in experts]), _ptr_array([e[1] for e in experts]),
            _ptr_array([e[2] for e in experts]),
            _ptr_array([s[0] for s in shared]), _ptr_array([s[1] for s in shared]),
            _ptr_array([s[2] for s in shared]),
            ctypes.c_void_p(out.ctypes.data), ctypes.c_void_p(idx.ctypes.data),
            ctypes.c_void_p(w.ctypes.data), ctypes.c_void_p(logits.ctypes.data))
        return {"out": out, "idx": idx, "w": w, "logits": logits}

    def predict_experts(self, draft_x, wg, pred_k):
        """Alg. 1, prediction half: per draft token the top-pred_k experts of the target gate.
        Returns (idx[n][pred_k], logits[n][E], p[n][E])."""
        logits = self.gate_logits(draft_x, wg)
        idx = np.stack([self.topk(row, pred_k) for row in logits])
        p = np.stack([self.softmax(row) for row in logits])
        return idx, logits, p
