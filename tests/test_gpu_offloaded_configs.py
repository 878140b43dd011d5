"""GPU parity of the benchmark configurations that are offloaded stacks, in their stated form: real layer
shapes, the stated cache budget, draft noise and cutoff layer, experts in pinned host memory, per-draft-token
prediction tasks, cache state carried from one iteration to the next.  Routing and outputs are compared with the
CPU oracle, queue contents and statistics with the reference cache model, after every call.  Stacks are shortened
to a few layers around the cutoff and backed by a few distinct expert blobs (cache identities stay distinct) to
bound host memory and oracle time."""
import numpy as np
import pytest

from oracle.cache_model import CacheModel
from offload_util import run_offloaded_stack

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mixtral_stack():
    # configuration 3: Mixtral-8x7B layers, 3 cache slots per layer; 18 layers cover every stated cutoff (4, 8, 16)
    from paper_2510_10302_amd import workload as W
    wl = W.Workload(d=4096, f=14336, E=8, k=2, shared=0, dtype="bf16", layers=18, seed=0, distinct=8)
    L = W.Loaded(wl, W.make_config(wl, max_tokens=8, slots=3, cutoff_layer=-1, pred_k=2), warm=False)
    yield wl, L
    L.close()


@pytest.mark.parametrize("sigma,cutoff,mode", [
    (0.1, 4, "sync"), (0.5, 4, "worker"), (0.1, 8, "worker"), (0.5, 8, "sync"), (0.1, 16, "worker"), (0.5, 16, "worker"),
])
def test_c3_mixtral_8x7b_offloaded_cells(mixtral_stack, oracle32, sigma, cutoff, mode):
    wl, L = mixtral_stack
    layers = cutoff + 2                                  # layers 0..cutoff are prefetched, the last one is not
    L.ctx.expert_cache_reset()
    L.ctx.set_cutoff(cutoff)
    model = CacheModel(wl.n_layers, wl.E, 3, cutoff_layer=cutoff)
    reps = run_offloaded_stack(L, wl, model, oracle32, layers=layers, T=8, sigma=sigma, pred_k=2,
                               seed=300 + cutoff, iterations=2, mode=mode)
    st = L.ctx.expert_cache_stats()
    print("c3 sigma %.1f cutoff %d %s: worst rel L2 %.2e, worst element %.2e rms, stats %s"
          % (sigma, cutoff, mode, max(r["rel_l2"] for r in reps), max(r["max_elem_err_over_rms"] for r in reps), st))
    assert st["prefetch_issued"] > 0 and st["hits"] > 0 and st["misses"] > 0 and st["evictions"] > 0
    assert L.ctx.expert_cache_contents(layers - 1) == model.contents(layers - 1)
    # beyond the cutoff nothing was prefetched: that layer's loads are all on demand
    assert all(len(model.unused_prefetch[l]) == 0 for l in range(cutoff + 1, wl.n_layers))


def test_c4_deepseek_v2_lite_offloaded_stack(oracle32):
    # configuration 4: d=2048, f=1408, 64 routed experts top-6 + 2 shared, 16 tokens, 16 slots per layer, prediction
    # with the top 6 (the paper's k for this model), one task per draft token through the prefetch worker
    from paper_2510_10302_amd import workload as W
    layers, cutoff, T = 4, 2, 16
    wl = W.Workload(d=2048, f=1408, E=64, k=6, shared=2, dtype="bf16", layers=layers, seed=0)
    L = W.Loaded(wl, W.make_config(wl, max_tokens=T, slots=16, cutoff_layer=cutoff, pred_k=6), warm=False)
    model = CacheModel(layers, 64, 16, cutoff_layer=cutoff)
    reps = run_offloaded_stack(L, wl, model, oracle32, layers=layers, T=T, sigma=0.3, pred_k=6, seed=400,
                               iterations=3, mode="worker")
    st = L.ctx.expert_cache_stats()
    print("c4 offloaded: worst rel L2 %.2e, worst element %.2e rms, stats %s"
          % (max(r["rel_l2"] for r in reps), max(r["max_elem_err_over_rms"] for r in reps), st))
    assert st["prefetch_used"] > 0 and st["misses"] > 0 and st["evictions"] > 0
    L.close()


def test_c5_mixtral_8x22b_offloaded_stack(oracle32):
    # configuration 5: d=6144, f=16384, 8 experts top-2, 32 tokens (4 sequences x 8), 2 slots per layer, draft
    # noise 0.3; 3 layers with the cutoff at layer 1, so the last layer is loaded on demand only
    from paper_2510_10302_amd import workload as W
    layers, cutoff, T = 3, 1, 32
    wl = W.Workload(d=6144, f=16384, E=8, k=2, shared=0, dtype="bf16", layers=layers, seed=0, distinct=8)
    L = W.Loaded(wl, W.make_config(wl, max_tokens=T, slots=2, cutoff_layer=cutoff, pred_k=2), warm=False)
    model = CacheModel(layers, 8, 2, cutoff_layer=cutoff)
    reps = run_offloaded_stack(L, wl, model, oracle32, layers=layers, T=T, sigma=0.3, pred_k=2, seed=500,
                               iterations=2, mode="worker")
    st = L.ctx.expert_cache_stats()
    print("c5 offloaded: worst rel L2 %.2e, worst element %.2e rms, stats %s"
          % (max(r["rel_l2"] for r in reps), max(r["max_elem_err_over_rms"] for r in reps), st))
    # 8 experts activated, 2 slots: every batch evicts experts it has itself just used
    assert st["misses"] >= 6 * layers and st["evictions"] > st["misses"] // 2 and st["prefetch_issued"] > 0
    L.close()


@pytest.mark.parametrize("io_chunks,mode,tokens_per_task", [
    ("1", "worker", 1), ("3", "sync", 1), ("16", "worker", 3), ("1", "blocking", 1), ("16", "blocking", 2),
])
def test_ablation_knobs_change_neither_results_nor_bookkeeping(oracle32, monkeypatch, io_chunks, mode, tokens_per_task):
    # the prefetcher modes of the ablation (caller's thread, caller's thread + wait for the copies, worker thread)
    # and the number of pieces an expert is copied in (1 = batched I/O) must leave outputs bit-identical, and
    # queue contents, statistics and bytes moved equal to the reference model's
    from paper_2510_10302_amd import workload as W
    layers, cutoff, T = 4, 2, 8
    wl = W.Workload(d=512, f=1408, E=8, k=2, shared=1, dtype="bf16", layers=layers, seed=17, gate_std=0.05, std=0.05)
    monkeypatch.delenv("SPMOE_IO_CHUNKS", raising=False)
    base = W.Loaded(wl, W.make_config(wl, max_tokens=T, slots=3, cutoff_layer=cutoff, pred_k=2), warm=False)
    want = []
    run_offloaded_stack(base, wl, CacheModel(layers, 8, 3, cutoff_layer=cutoff), oracle32, layers=layers, T=T, sigma=0.4,
                        pred_k=2, seed=600, iterations=3, mode="sync", collect_outputs=want)
    base_stats = base.ctx.expert_cache_stats()
    base.close()
    monkeypatch.setenv("SPMOE_IO_CHUNKS", io_chunks)
    L = W.Loaded(wl, W.make_config(wl, max_tokens=T, slots=3, cutoff_layer=cutoff, pred_k=2), warm=False)
    got = []
    model = CacheModel(layers, 8, 3, cutoff_layer=cutoff)
    if tokens_per_task == 1:
        run_offloaded_stack(L, wl, model, oracle32, layers=layers, T=T, sigma=0.4, pred_k=2, seed=600, iterations=3,
                            mode=mode, collect_outputs=got)
        st = L.ctx.expert_cache_stats()
        for key in base_stats:
            if key != "late_hits":                                  # timing-dependent
                assert st[key] == base_stats[key], key
        assert all(np.array_equal(a.view(np.uint32), b.view(np.uint32)) for a, b in zip(got, want))
    else:
        # several draft states per task: the ranking by votes decides the task; outputs still cannot change
        run_offloaded_stack(L, wl, model, oracle32, layers=layers, T=T, sigma=0.4, pred_k=2, seed=600, iterations=3,
                            mode=mode, tokens_per_task=tokens_per_task, collect_outputs=got)
        assert all(np.array_equal(a.view(np.uint32), b.view(np.uint32)) for a, b in zip(got, want))
    L.close()
