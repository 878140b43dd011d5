"""GPU tests of the expert cache, prediction and prefetch: results never depend on the cache state
(policy invariance), and the bookkeeping matches the reference cache/queue model call by call."""
import numpy as np
import pytest

import spmoe_inputs as si
from oracle.cache_model import CacheModel, rank_predicted
from parity_util import REL_L2_BF16, gpu_layer, oracle_layer, rel_l2

pytestmark = pytest.mark.gpu


def _setup(slots, cutoff, layers=3, E=8, k=2, d=256, f=192, T=8, pred_k=2, shared=0, seed=12):
    from paper_2510_10302_amd import workload as W
    wl = W.Workload(d=d, f=f, E=E, k=k, shared=shared, dtype="bf16", layers=layers, seed=seed, gate_std=0.05, std=0.05)
    L = W.Loaded(wl, W.make_config(wl, max_tokens=T, slots=slots, cutoff_layer=cutoff, pred_k=pred_k))
    return wl, L


def test_policy_invariance_outputs_do_not_depend_on_cache_state():
    T = 8
    wl, ref = _setup(slots=None, cutoff=-1)
    xs = [si.hidden(12, T, 256, iteration=i, layer=l) for i in range(3) for l in range(3)]
    want = [gpu_layer(ref, j % 3, x)["out"] for j, x in enumerate(xs)]
    ref.close()
    for slots in (1, 2, 3, 5):
        wl2, L = _setup(slots=slots, cutoff=1)
        rng = np.random.default_rng(slots)
        for j, x in enumerate(xs):
            layer = j % 3
            L.ctx.prefetch(layer, rng.integers(0, 8, size=3).tolist())     # arbitrary (mostly wrong) prefetches
            got = gpu_layer(L, layer, x)["out"]
            assert np.array_equal(got, want[j]), (slots, j)                 # bit-identical: fixed summation order
        st = L.ctx.expert_cache_stats()
        assert st["misses"] == st["ondemand_loads"] and st["hits"] + st["misses"] > 0
        L.close()


def test_bookkeeping_matches_cache_model(oracle32):
    T, E, k, slots, cutoff, n_layers = 8, 8, 2, 3, 1, 3
    wl, L = _setup(slots=slots, cutoff=cutoff, layers=n_layers)
    model = CacheModel(n_layers, E, slots, cutoff_layer=cutoff)
    import torch
    for it in range(4):
        for layer in range(n_layers):
            x = si.hidden(12, T, 256, iteration=it, layer=layer)
            draft = x + si.draft_noise(12, T, 256, 0.3, iteration=it, layer=layer)
            # Alg. 1 on the library ...
            ids = L.ctx.predict_experts(layer, torch.from_numpy(draft).cuda())
            # ... and on the reference: top-pred_k per draft token, ranked by votes / probability / index
            if layer <= cutoff:
                pidx, plog, pp = oracle32.predict_experts(draft, wl.gate[layer], 2)
                assert ids == model.filter_cached(layer, rank_predicted(pidx, pp, E))
            else:
                assert ids == []
            L.ctx.prefetch(layer, ids)
            model.prefetch(layer, ids)
            assert L.ctx.expert_cache_contents(layer) == model.contents(layer)
        for layer in range(n_layers):
            x = si.hidden(12, T, 256, iteration=it, layer=layer)
            g = gpu_layer(L, layer, x)
            ref = oracle_layer(oracle32, wl, layer, x)
            assert np.array_equal(g["idx"], ref["idx"])
            assert rel_l2(g["out"], ref["out"]) < REL_L2_BF16
            model.verify(layer, sorted(set(ref["idx"].reshape(-1).tolist())))
            assert L.ctx.expert_cache_contents(layer) == model.contents(layer), (it, layer)
            for e in range(E):
                assert (L.ctx.expert_cache_lookup(layer, e) >= 0) == (e in model.contents(layer))
    st = L.ctx.expert_cache_stats()
    for key in ("hits", "misses", "evictions", "prefetch_issued", "prefetch_used", "prefetch_wasted", "ondemand_loads"):
        assert st[key] == model.stats[key], (key, st, model.stats)
    nbytes = 3 * 256 * 192 * 2
    assert st["h2d_bytes_prefetch"] == st["prefetch_issued"] * nbytes
    assert st["h2d_bytes_ondemand"] == st["ondemand_loads"] * nbytes
    L.ctx.expert_cache_reset()
    assert L.ctx.expert_cache_contents(0) == [] and L.ctx.expert_cache_stats()["hits"] == 0
    L.close()


def test_shared_experts_with_offload(oracle32):
    # DeepSeek-like arity, offloaded routed experts, shared experts always resident
    wl, L = _setup(slots=16, cutoff=1, layers=2, E=64, k=6, d=256, f=160, T=16, pred_k=6, shared=2, seed=13)
    import torch
    for layer in range(2):
        x = si.hidden(13, 16, 256, layer=layer)
        ids = L.ctx.predict_experts(layer, torch.from_numpy(x).cuda())   # sigma = 0: prediction is the truth
        L.ctx.prefetch(layer, ids)
        g = gpu_layer(L, layer, x)
        ref = oracle_layer(oracle32, wl, layer, x)
        assert np.array_equal(g["idx"], ref["idx"])
        assert rel_l2(g["out"], ref["out"]) < REL_L2_BF16
    st = L.ctx.expert_cache_stats()
    assert st["prefetch_used"] == st["prefetch_issued"] == 32 and st["hits"] >= 32
    L.close()


def test_profile_records_cover_copies_and_layers():
    wl, L = _setup(slots=2, cutoff=0, layers=2)
    import torch
    L.ctx.profile_begin()
    L.ctx.prefetch(0, [1, 2])
    x = torch.from_numpy(si.hidden(12, 8, 256)).cuda()
    out = torch.empty((8, 256), device="cuda")
    L.ctx.moe_verify_layer(0, x, out)
    ms = L.ctx.last_layer_kernel_ms()
    recs = L.ctx.profile_collect()
    kinds = [r["kind"] for r in recs]
    assert kinds.count(1) == 2 and kinds.count(0) == 1 and kinds.count(2) >= 1
    assert all(r["t1"] >= r["t0"] >= 0 for r in recs)
    # every wait of the compute stream for a copy is recorded: one per on-demand load (kind 9); prefetched experts
    # the batch uses are either already there or waited for (kind 7), never loaded twice
    assert kinds.count(9) == kinds.count(2)
    waited = {r["expert"] for r in recs if r["kind"] == 7}
    assert waited <= {1, 2} and not (waited & {r["expert"] for r in recs if r["kind"] == 2})
    assert kinds.count(8) == 0
    assert len(ms) == 4 and all(m >= 0 for m in ms) and ms[1] > 0 and ms[2] > 0
    L.close()


def test_async_worker_matches_synchronous_calls(oracle32):
    # The worker-thread path (predict + prefetch queued without blocking) must leave the cache, the
    # statistics and the outputs exactly as the same calls made synchronously do.
    import torch
    T, n_layers = 8, 3
    results = []
    for mode in ("sync", "async"):
        wl, L = _setup(slots=3, cutoff=1, layers=n_layers)
        outs, contents = [], []
        for it in range(5):
            xs = [si.hidden(12, T, 256, iteration=it, layer=l) for l in range(n_layers)]
            drafts = [torch.from_numpy(xs[l] + si.draft_noise(12, T, 256, 0.3, iteration=it, layer=l)).cuda()
                      for l in range(n_layers)]
            for j in range(T - 1):                     # one task per draft token and layer, as in the drafting stage
                for l in range(n_layers):
                    if mode == "sync":
                        L.ctx.prefetch(l, L.ctx.predict_experts(l, drafts[l][j:j + 1]))
                    else:
                        L.ctx.predict_prefetch_async(l, drafts[l][j:j + 1])
            for l in range(n_layers):
                outs.append(gpu_layer(L, l, xs[l])["out"])
                contents.append(L.ctx.expert_cache_contents(l))
        L.ctx.prefetch_drain()
        results.append((outs, contents, L.ctx.expert_cache_stats()))
        L.close()
    (o1, c1, s1), (o2, c2, s2) = results
    assert c1 == c2
    for key in s1:
        if key != "late_hits":                         # timing-dependent: how many copies were still in flight
            assert s1[key] == s2[key], key
    assert all(np.array_equal(a, b) for a, b in zip(o1, o2))
    assert s2["prefetch_issued"] > 0


def test_measured_load_time_and_suggested_cutoff():
    import paper_2510_10302_amd as sp
    wl, L = _setup(slots=2, cutoff=0, layers=2, d=1024, f=2048)
    ms = L.ctx.measure_expert_load_ms(0, 1, repeats=3)
    nbytes = 3 * 1024 * 2048 * 2
    gbs = nbytes / (ms * 1e-3) / 1e9
    print("expert load %.3f ms -> %.1f GB/s" % (ms, gbs))
    assert 1.0 < gbs < 200.0
    # with a per-layer compute time of 4 loads, the overlap constraint (L+1)*k*t_io <= L_all*t_comp gives L = 7 of 2 layers -> capped
    assert sp.suggest_cutoff(2, 2, 1, 4 * ms, ms, 0.0, nbytes, 1e12) == 1
    assert sp.suggest_cutoff(2, 2, 1, 0.25 * ms, ms, 0.0, nbytes, 1e12) == -1
    L.close()


@pytest.mark.parametrize("copy_streams", ["default", "1", "2", "4"])
def test_stress_small_budgets_random_order_async(copy_streams, monkeypatch):
    # copy_streams: how many copy streams the context uses (default: one for prefetches, two alternating for
    # on-demand loads); a slot may be rewritten over a different stream than the one that filled it last
    if copy_streams != "default":
        monkeypatch.setenv("SPMOE_COPY_STREAMS", copy_streams)
    # slot hazards: 1-2 slots per layer, layers visited in random order, worker-thread prefetches racing with
    # verify calls; every output must stay bit-identical to the all-resident run
    import torch
    T, n_layers = 8, 4
    wl, ref = _setup(slots=None, cutoff=-1, layers=n_layers)
    rng = np.random.default_rng(99)
    plan = [(int(rng.integers(0, n_layers)), int(rng.integers(0, 50))) for _ in range(40)]
    xs = {p: si.hidden(12, T, 256, iteration=p[1], layer=p[0]) for p in plan}
    want = {p: gpu_layer(ref, p[0], xs[p])["out"] for p in plan}
    ref.close()
    for slots in (1, 2):
        wl2, L = _setup(slots=slots, cutoff=n_layers - 1, layers=n_layers, pred_k=2)
        for step, p in enumerate(plan):
            nxt = plan[(step + 1) % len(plan)]
            L.ctx.predict_prefetch_async(nxt[0], torch.from_numpy(xs[nxt][:3]).cuda())    # prefetch for a later call
            if step % 3 == 0:
                L.ctx.prefetch(p[0], rng.integers(0, 8, size=2).tolist())
            got = gpu_layer(L, p[0], xs[p])["out"]
            assert np.array_equal(got, want[p]), (slots, step, p)
        st = L.ctx.expert_cache_stats()
        assert st["evictions"] > 0 and st["prefetch_issued"] > 0
        L.close()


def test_contexts_release_their_memory_and_threads():
    # create / use / destroy repeatedly: HBM returns to the pool, worker threads are joined
    import threading
    import torch
    from paper_2510_10302_amd import workload as W
    wl = W.Workload(d=512, f=1024, E=8, k=2, shared=1, dtype="bf16", layers=4, seed=51)
    threads0 = threading.active_count()
    x = torch.from_numpy(si.hidden(51, 8, 512)).cuda()
    out = torch.empty((8, 512), device="cuda")

    def cycle(n):
        for rep in range(n):
            L = W.Loaded(wl, W.make_config(wl, max_tokens=8, slots=3, cutoff_layer=3), warm=False)
            for l in range(4):
                L.ctx.predict_prefetch_async(l, x[:2])      # starts the worker thread
            for l in range(4):
                L.ctx.moe_verify_layer(l, x, out)
            L.close()
        torch.cuda.synchronize()
        return torch.cuda.mem_get_info()[0]

    free_warm = cycle(2)          # first uses load code objects and grow the runtime's own pools
    free_end = cycle(8)
    print("free HBM after 2 cycles %.1f MiB, after 10 cycles %.1f MiB" % (free_warm / 2 ** 20, free_end / 2 ** 20))
    assert free_warm - free_end < 8 * 2 ** 20, "leaked %.1f MiB over 8 create/destroy cycles" % ((free_warm - free_end) / 2 ** 20)
    assert threading.active_count() == threads0


def test_unregistered_expert_is_reported_not_dereferenced():
    import torch
    import paper_2510_10302_amd as sp
    from paper_2510_10302_amd import workload as W
    wl = W.Workload(d=128, f=128, E=4, k=2, shared=0, dtype="bf16", layers=1, seed=52)
    cfg = W.make_config(wl, max_tokens=8, slots=2)
    ctx = sp.Context(cfg)
    x = torch.from_numpy(si.hidden(52, 8, 128)).cuda()
    out = torch.empty((8, 128), device="cuda")
    with pytest.raises(sp.SpmoeError) as e:
        ctx.moe_verify_layer(0, x, out)                   # gate not set
    assert e.value.status_name == "SPMOE_ESTATE"
    g = torch.from_numpy(wl.gate[0].view(np.int16)).cuda()
    ctx.set_gate(0, g)
    with pytest.raises(sp.SpmoeError) as e:
        ctx.moe_verify_layer(0, x, out)                   # experts needed but none registered
    assert e.value.status_name == "SPMOE_ESTATE" and "not registered" in str(e.value)
    with pytest.raises(sp.SpmoeError) as e:
        ctx.expert_cache_warm(0, [1])
    assert e.value.status_name == "SPMOE_ESTATE"
    ctx.destroy()


def test_resident_layer_can_be_captured_in_a_hip_graph():
    # With every expert resident a verify-layer call needs nothing on the host: four kernel launches on the
    # compute stream, no memset, no synchronisation (the routing kernel re-zeroes its own counters).  It can
    # therefore be captured once and replayed.  Each replay, with eager work and synchronisations in between
    # and with new inputs written into the captured buffers, must equal the eager result bit for bit.
    import torch
    from paper_2510_10302_amd import workload as W
    wl = W.Workload(d=512, f=1408, E=16, k=2, shared=1, dtype="bf16", layers=2, seed=21, gate_std=0.05, std=0.05)
    T = 8
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        L = W.Loaded(wl, W.make_config(wl, max_tokens=T), stream=stream)
        xs = [torch.from_numpy(si.hidden(300 + i, T, wl.d)).cuda() for i in range(4)]
        x_in = torch.zeros_like(xs[0])
        mid = torch.zeros_like(xs[0])
        out = torch.zeros_like(xs[0])

        def two_layers(src, tmp, dst):
            L.ctx.moe_verify_layer(0, src, tmp)
            L.ctx.moe_verify_layer(1, tmp, dst)

        eager = []
        for x in xs:                                   # also the warm-up that sizes the launches
            o = torch.empty_like(x)
            two_layers(x, mid, o)
            eager.append(o.clone())
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            two_layers(x_in, mid, out)
        for rep in range(3):
            for i, x in enumerate(xs):
                x_in.copy_(x)
                graph.replay()
                got = out.clone()
                # eager work of the same context between replays
                o = torch.empty_like(x)
                two_layers(xs[(i + 1) % 4], mid, o)
                stream.synchronize()
                assert torch.equal(got.view(torch.int32), eager[i].view(torch.int32)), (rep, i)
                assert torch.equal(o.view(torch.int32), eager[(i + 1) % 4].view(torch.int32)), (rep, i)
    L.close()
