"""CPU-side checks of the C-ABI library: it loads, exports every symbol the header declares, and its
host-only entry points (sizes, packing, argument validation) behave as documented.  No kernel runs."""
import ctypes
import os
import re

import numpy as np
import pytest

import spmoe_inputs as si

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def sp():
    import paper_2510_10302_amd as sp
    if not os.path.exists(sp.lib_path()):
        from paper_2510_10302_amd import build
        build.build()
    sp.load_library()
    return sp


def test_header_symbols_are_exported(sp):
    header = open(os.path.join(ROOT, "include", "spmoe.h")).read()
    declared = sorted(set(re.findall(r"^(?:spmoe_status|size_t|const char\*)\s+(spmoe_[a-z_0-9]+)\(", header, re.M)))
    assert declared == sorted(sp.DECLARED_SYMBOLS)
    lib = ctypes.CDLL(sp.lib_path())
    for name in declared:
        assert hasattr(lib, name), name


def test_blob_bytes_match_paper_expert_sizes(sp):
    # 336 MB / 150 MB / 16.5 MB per expert (16-bit), the sizes quoted in the paper's latency analysis
    for d, f, mib in [(4096, 14336, 336), (4096, 6400, 150), (2048, 1408, 16.5)]:
        cfg = sp.Config(d_model=d, d_ff=f, n_experts=8, top_k=2)
        assert sp.expert_blob_bytes(cfg) == mib * 2 ** 20
    assert sp.expert_blob_bytes(sp.Config(d_model=100, d_ff=64, n_experts=8, top_k=2)) == 0      # d not a multiple of 32
    assert sp.expert_blob_bytes(sp.Config(d_model=64, d_ff=64, n_experts=8, top_k=9)) == 0       # k > limits


def test_pack_is_a_permutation_of_the_canonical_weights(sp):
    d, f = 96, 160
    cfg = sp.Config(d_model=d, d_ff=f, n_experts=4, top_k=2)
    g, u, dn = si.expert_weights(1, 0, 0, d, f, "bf16")
    blob = sp.pack_expert(cfg, g, u, dn).view(np.uint16)
    assert blob.size == 3 * d * f
    assert np.array_equal(np.sort(blob), np.sort(np.concatenate([g.ravel(), u.ravel(), dn.ravel()])))
    # tile (nt, ks) of the gate/up region: lane l holds row nt*16 + (l & 15), K = ks*32 + 8*(l >> 4) .. +7
    tiles = blob[: 2 * d * f].reshape(f // 16, d // 32, 2, 64, 8)
    for nt, ks, lane in [(0, 0, 0), (3, 2, 37), (9, 1, 63)]:
        r, k0 = nt * 16 + (lane & 15), ks * 32 + 8 * (lane >> 4)
        assert np.array_equal(tiles[nt, ks, 0, lane], g[r, k0:k0 + 8])
        assert np.array_equal(tiles[nt, ks, 1, lane], u[r, k0:k0 + 8])
    dt = blob[2 * d * f:].reshape(d // 16, f // 32, 64, 8)
    for nt, ks, lane in [(0, 0, 0), (5, 4, 21)]:
        r, k0 = nt * 16 + (lane & 15), ks * 32 + 8 * (lane >> 4)
        assert np.array_equal(dt[nt, ks, lane], dn[r, k0:k0 + 8])
    # fp32: the three matrices back to back
    cfg32 = sp.Config(d_model=d, d_ff=f, n_experts=4, top_k=2, weight_dtype=sp.F32)
    g32, u32, d32 = si.expert_weights(1, 0, 0, d, f, "f32")
    b32 = sp.pack_expert(cfg32, g32, u32, d32).view(np.float32)
    assert np.array_equal(b32, np.concatenate([g32.ravel(), u32.ravel(), d32.ravel()]))


def test_argument_validation_without_a_gpu(sp):
    lib = sp.load_library()
    handle = ctypes.c_void_p()
    assert lib.spmoe_create(None, None, ctypes.byref(handle)) == 1                      # SPMOE_EINVAL
    bad = sp.Config(d_model=64, d_ff=64, n_experts=4, top_k=2, max_tokens=1000)
    assert lib.spmoe_create(ctypes.byref(bad), None, ctypes.byref(handle)) == 2         # SPMOE_ERANGE
    assert lib.spmoe_destroy(None) == 0
    assert lib.spmoe_last_error(None) == b""
    cfg = sp.Config(d_model=64, d_ff=64, n_experts=4, top_k=2)
    assert lib.spmoe_pack_expert(ctypes.byref(cfg), None, None, None, None) == 1
    assert lib.spmoe_sync(None) == 1
    with pytest.raises(ValueError):
        sp.pack_expert(cfg, np.zeros((64, 64), np.float32), np.zeros((64, 64), np.float32), np.zeros((64, 64), np.float32))
