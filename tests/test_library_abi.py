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


def test_cutoff_policy_hand_worked(sp):
    # "Cutoff layer design": N = (L+1)k; m_peak + N*m_exp < m_gpu; max{(L-1)t_c + k*t_io, N*t_io} <= L_all*t_c.
    # Hand-worked: L_all = 32, t_c = 1, t_io = 2, k = 1, no memory pressure: N*t_io = 2(L+1) <= 32 -> L = 15.
    assert sp.suggest_cutoff(32, 32, 1, 1.0, 2.0, 0.0, 1.0, 1e9) == 15
    # memory binds first: 10 + (L+1)*1 < 20 -> L + 1 <= 9 -> L = 8
    assert sp.suggest_cutoff(32, 32, 1, 1.0, 2.0, 10.0, 1.0, 20.0) == 8
    # k = 2: 2(L+1)*2 <= 32 -> L = 7
    assert sp.suggest_cutoff(32, 32, 2, 1.0, 2.0, 0.0, 1.0, 1e9) == 7
    # fast link: I/O never binds, every layer qualifies ((L-1) + k*t_io <= 32 holds up to L = 31)
    assert sp.suggest_cutoff(32, 32, 1, 1.0, 0.01, 0.0, 1.0, 1e9) == 31
    # first term binds: t_io = 20, k = 1: N*t_io = 20(L+1) <= 32 -> L = 0; (L-1) + 20 <= 32 fine
    assert sp.suggest_cutoff(32, 32, 1, 1.0, 20.0, 0.0, 1.0, 1e9) == 0
    # loading one expert takes longer than the whole drafting stage: nothing can be hidden
    assert sp.suggest_cutoff(32, 32, 1, 1.0, 40.0, 0.0, 1.0, 1e9) == -1
    # a Mixtral-8x7B-shaped expert over a ~57 GB/s link (6.2 ms) against 32 draft layers of 75 us: none
    assert sp.suggest_cutoff(32, 32, 1, 0.075, 6.2, 0.0, 0.336, 288.0) == -1
    lib = sp.load_library()
    assert lib.spmoe_suggest_cutoff(0, 32, 1, 1.0, 1.0, 0.0, 1.0, 1.0, None) == 1


def test_bench_refuses_more_than_one_gpu():
    import subprocess, sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_bench_finds_the_recorded_counter_traffic():
    # the roofline block quotes HBM traffic from the committed rocprofv3 summaries: each benchmark shape must have
    # one that still parses, names the commit it was measured at, and lies between one expert's gate/up bytes and
    # those of all the layer's experts (+ 2 %): more would mean re-reads were recorded
    import importlib.util
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    shapes = {"c2_mixtral_8x7b": (4096, 14336, 8, 0), "c4_deepseek_v2_lite": (2048, 1408, 64, 2),
              "c5_mixtral_8x22b": (6144, 16384, 8, 0)}
    for name, (d, f, E, shared) in shapes.items():
        traffic, commit = bench.profiled_traffic(name)
        assert traffic and commit, name
        experts = traffic / (2.0 * d * f * 2)
        assert 1.0 <= experts <= (E + shared) * 1.02, (name, experts)
    assert bench.profiled_traffic("no_such_workload") == (None, None)


def test_no_cpu_fallback_when_the_library_is_missing(sp, monkeypatch):
    from paper_2510_10302_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", os.path.join(ROOT, "does_not_exist", "libspmoe.so"))
    with pytest.raises(ImportError):
        binding.load_library()


def test_header_is_plain_c_and_cpp(tmp_path):
    # the boundary is a C ABI: the header must compile as strict C99 and as C++ with no extra includes
    import subprocess
    inc = os.path.join(ROOT, "include")
    src = ('#include "spmoe.h"\n'
           'int main(void) { spmoe_config c; spmoe_stats s; spmoe_profile_record r; (void)c; (void)s; (void)r;\n'
           '  return (int)sizeof(spmoe_status) + SPMOE_MAX_TOKENS * 0; }\n')
    c_file, cpp_file = tmp_path / "abi.c", tmp_path / "abi.cpp"
    c_file.write_text(src)
    cpp_file.write_text(src)
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", inc, "-c", str(c_file),
                           "-o", str(tmp_path / "abi_c.o")])
    subprocess.check_call(["g++", "-std=c++11", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", inc, "-c", str(cpp_file),
                           "-o", str(tmp_path / "abi_cpp.o")])


def test_gemm_plans_fit_what_the_kernels_assume(sp):
    # Host logic that sizes every bf16 expert-GEMM launch: for every shape the library accepts, the plan must
    # cover the contraction, keep the workgroup within the kernels' launch bounds (16 waves; 8 waves when a
    # wave holds more than 14 k-steps of the token tile in registers), divide the N tiles evenly and fit the
    # LDS of a CU.  A plan outside these limits would launch a kernel whose indexing does not match its grid.
    exact_steps = {4, 8, 10, 11, 12, 14, 16, 24, 28, 32}
    shapes = [(d, f) for d in range(32, 8193, 32) for f in (32, 64, 96, 1408, 4096, 6400, 14336, 16384)]
    shapes += [(d, f) for d in (32, 512, 2048, 4096, 6144, 8192) for f in range(32, 32769, 32)]
    for d, f, T in [(d, f, T) for d, f in shapes for T in (16, 32)]:
        cfg = sp.Config(d_model=d, d_ff=f, n_experts=8, top_k=2, weight_dtype=sp.BF16, max_tokens=T)
        for proj, (k_len, n_units) in enumerate([(d // 32, f // 16), (f // 32, d // 32)]):
            p = sp.gemm_plan(cfg, proj)
            waves = p["k_waves"] * p["n_sub"]
            assert 1 <= waves <= 16 and (p["k_steps"] <= 14 or waves <= 8), (d, f, proj, p)
            if p["tokens_per_pass"] == 32:
                # the instances that take 32 tokens of an expert in one weight pass (batches of more than 16 tokens
                # only) have at most 8 waves, one N sub-tile, and no more k-steps per wave than their registers hold
                assert T > 16 and waves <= 8 and p["n_sub"] == 1, (d, f, proj, p)
                assert not p["exact"] or p["k_steps"] <= (28 if proj == 0 else 32), (d, f, proj, p)
            assert n_units % p["n_sub"] == 0, (d, f, proj, p)
            assert p["lds_bytes"] <= 160 * 1024 // 2, (d, f, proj, p)     # two workgroups per CU still fit its 160 KB
            if proj == 0:
                assert p["splits"] == 1, (d, f, p)         # SiLU needs the whole contraction in one workgroup
            if p["exact"]:
                assert p["k_steps"] in exact_steps, (d, f, proj, p)
                assert p["splits"] * p["k_waves"] * p["k_steps"] == k_len, (d, f, proj, p)
            else:
                per = -(-k_len // p["splits"])
                assert p["k_steps"] == 32 and p["k_waves"] <= 8 and p["k_waves"] * 32 >= per, (d, f, proj, p)
    # the benchmark shapes use the plans the measurements were made with
    c2 = sp.Config(d_model=4096, d_ff=14336, n_experts=8, top_k=2, weight_dtype=sp.BF16, max_tokens=8)
    assert (sp.gemm_plan(c2, 0)["k_waves"], sp.gemm_plan(c2, 0)["k_steps"]) == (8, 16)
    p = sp.gemm_plan(c2, 1)
    assert (p["splits"], p["k_waves"], p["k_steps"]) == (2, 16, 14)
    c5 = sp.Config(d_model=6144, d_ff=16384, n_experts=8, top_k=2, weight_dtype=sp.BF16, max_tokens=32)
    p = sp.gemm_plan(c5, 0)
    assert (p["k_waves"], p["k_steps"], p["tokens_per_pass"]) == (8, 24, 32)
    p = sp.gemm_plan(c5, 1)
    assert (p["splits"], p["k_waves"], p["k_steps"], p["tokens_per_pass"]) == (2, 8, 32, 32)
    with pytest.raises(sp.SpmoeError):
        sp.gemm_plan(sp.Config(d_model=512, d_ff=1024, n_experts=8, top_k=2, weight_dtype=sp.F32), 0)
    with pytest.raises(sp.SpmoeError):
        sp.gemm_plan(c2, 2)
