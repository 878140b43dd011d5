"""Seeded synthetic inputs for the SP-MoE hot path (tests, benchmark, smoke check).

This module is the only code shared by the CPU oracle's tests and the GPU path's tests.  It
contains no arithmetic of the method itself: only a counter-based normal generator (``gen.c``)
and helpers that lay tensors out in the *canonical* (row-major) form both sides accept:

* gate weights ``Wg[E][d]``
* per expert ``W_gate[f][d]``, ``W_up[f][d]``, ``W_down[d][f]`` (3-matrix SwiGLU expert; the
  3*d*f*2-byte size reproduces the per-expert sizes quoted in the paper's latency analysis)
* hidden states ``x[T][d]`` in fp32

Weights are N(0, 0.02^2), hidden states N(0, 1).  bf16 tensors are returned as ``uint16`` bit
patterns (rounded to nearest-even once, here), so both sides read identical weight bits.
"""
import ctypes
import os
import subprocess

import numpy as np

_DIR = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_DIR, "libspmoe_gen.so")
_lib = None

# stream ids inside one seed: keep tensors of one workload disjoint
STREAM_X = 1 << 40          # + iteration * 4096 + layer
STREAM_GATE = 2 << 40       # + layer
STREAM_EXPERT = 3 << 40     # + ((layer * 4096 + expert) * 4 + {0: gate, 1: up, 2: down})
STREAM_NOISE = 4 << 40      # + iteration * 4096 + layer
STREAM_SHARED = 5 << 40     # + ((layer * 64 + idx) * 4 + matrix)


def build():
    """Compile gen.c into libspmoe_gen.so (host only, no GPU code)."""
    cmd = ["gcc", "-O2", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off", "-std=c99",
           os.path.join(_DIR, "gen.c"), "-o", _SO, "-lm"]
    subprocess.check_call(cmd)


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_SO):
            build()
        lib = ctypes.CDLL(_SO)
        u64 = ctypes.c_uint64
        lib.spmoe_gen_normal_f32.argtypes = [u64, u64, u64, u64, ctypes.c_float, ctypes.c_float, ctypes.c_void_p]
        lib.spmoe_gen_normal_f32.restype = None
        lib.spmoe_gen_normal_bf16.argtypes = [u64, u64, u64, u64, ctypes.c_float, ctypes.c_void_p]
        lib.spmoe_gen_normal_bf16.restype = None
        lib.spmoe_gen_round_bf16.argtypes = [ctypes.c_void_p, u64, ctypes.c_void_p]
        lib.spmoe_gen_round_bf16.restype = None
        _lib = lib
    return _lib


def normal_f32(seed, stream, n, std=1.0, mean=0.0, offset=0, out=None):
    """Elements offset..offset+n-1 of the fp32 N(mean, std^2) tensor named (seed, stream)."""
    lib = _load()
    if out is None:
        out = np.empty(int(n), dtype=np.float32)
    assert out.dtype == np.float32 and out.flags.c_contiguous and out.size == n
    lib.spmoe_gen_normal_f32(seed, stream, offset, n, mean, std, out.ctypes.data)
    return out


def normal_bf16(seed, stream, n, std=1.0, offset=0, out=None):
    """Same values as normal_f32 (mean 0), rounded to bf16; returned as uint16 bit patterns."""
    lib = _load()
    if out is None:
        out = np.empty(int(n), dtype=np.uint16)
    assert out.dtype == np.uint16 and out.flags.c_contiguous and out.size == n
    lib.spmoe_gen_normal_bf16(seed, stream, offset, n, std, out.ctypes.data)
    return out


def round_bf16(a):
    """fp32 array -> bf16 bit patterns (uint16), round to nearest even."""
    lib = _load()
    a = np.ascontiguousarray(a, dtype=np.float32)
    out = np.empty(a.shape, dtype=np.uint16)
    lib.spmoe_gen_round_bf16(a.ctypes.data, a.size, out.ctypes.data)
    return out


def bf16_to_f32(bits):
    """Exact upcast of bf16 bit patterns (uint16) to fp32 values (test helper, no rounding)."""
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def _weights(seed, stream, shape, dtype, std):
    n = int(np.prod(shape))
    if dtype == "bf16":
        return normal_bf16(seed, stream, n, std).reshape(shape)
    if dtype == "f32":
        return normal_f32(seed, stream, n, std).reshape(shape)
    raise ValueError(dtype)


def hidden(seed, T, d, iteration=0, layer=0):
    """x[T][d] fp32 ~ N(0,1)."""
    return normal_f32(seed, STREAM_X + iteration * 4096 + layer, T * d).reshape(T, d)


def hidden_correlated(seed, T, d, rho, n_seq=1, iteration=0, layer=0):
    """x[T][d] fp32 with unit variance whose rows share a per-sequence component:
    x_t = rho * b_seq(t) + sqrt(1 - rho^2) * eps_t, T split evenly into n_seq sequences.  rho = 0 gives hidden().
    Neighbouring tokens of a sequence then tend to pick the same experts (the paper's Observation I)."""
    eps = hidden(seed, T, d, iteration=iteration, layer=layer)
    base = normal_f32(seed, STREAM_X + (1 << 36) + iteration * 4096 + layer, n_seq * d).reshape(n_seq, d)
    per = (T + n_seq - 1) // n_seq
    seq = np.minimum(np.arange(T) // per, n_seq - 1)
    return (np.float32(rho) * base[seq] + np.float32(np.sqrt(1.0 - rho * rho)) * eps).astype(np.float32)


def draft_noise(seed, T, d, sigma, iteration=0, layer=0):
    """sigma * eps[T][d]: the additive noise that turns a target hidden state into a stand-in draft one."""
    return normal_f32(seed, STREAM_NOISE + iteration * 4096 + layer, T * d, std=sigma).reshape(T, d)


def gate_weights(seed, layer, E, d, dtype, std=0.02):
    """Wg[E][d] of one layer."""
    return _weights(seed, STREAM_GATE + layer, (E, d), dtype, std)


def expert_weights(seed, layer, expert, d, f, dtype, std=0.02, shared=False):
    """(W_gate[f][d], W_up[f][d], W_down[d][f]) of one routed (or shared) expert, canonical row-major."""
    if shared:
        base = STREAM_SHARED + (layer * 64 + expert) * 4
    else:
        base = STREAM_EXPERT + (layer * 4096 + expert) * 4
    return (_weights(seed, base + 0, (f, d), dtype, std),
            _weights(seed, base + 1, (f, d), dtype, std),
            _weights(seed, base + 2, (d, f), dtype, std))
