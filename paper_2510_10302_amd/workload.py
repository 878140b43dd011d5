"""Synthetic SP-MoE workloads (the five benchmark configurations: a small fp32 layer, Mixtral-8x7B, DeepSeek-V2-Lite and Mixtral-8x22B shapes) laid out for the library.

This is plumbing around the C ABI for the tests, the smoke check and the benchmark: it draws seeded
tensors from ``spmoe_inputs``, packs experts into pinned host blobs (``spmoe_pack_expert``), uploads
gates, registers everything with a context.  It performs none of the path's arithmetic.

To bound host memory and generation time, a stack may use *aliased backing*: only ``distinct`` expert
blobs are generated and routed expert (layer, e) uses blob ``(layer * E + e) % distinct``.  Cache
identities stay distinct, so copy traffic and LRU behaviour are those of the full model.
"""
import numpy as np

import spmoe_inputs as si

from . import binding as sp

CONFIGS = {
    # name: d, f, E, k, shared, T, dtype, layers, slots (None = all resident)
    "c1_small":        dict(d=512,  f=1024,  E=8,  k=2, shared=0, T=5,  dtype="f32",  layers=1,  slots=None),
    "c2_mixtral_8x7b": dict(d=4096, f=14336, E=8,  k=2, shared=0, T=8,  dtype="bf16", layers=1,  slots=None),
    "c3_mixtral_8x7b_offload": dict(d=4096, f=14336, E=8, k=2, shared=0, T=8, dtype="bf16", layers=32, slots=3),
    "c4_deepseek_v2_lite": dict(d=2048, f=1408, E=64, k=6, shared=2, T=16, dtype="bf16", layers=26, slots=16),
    # third model pair of the paper's Table 1 (not one of the five benchmark configurations)
    "phi_3_5_moe": dict(d=4096, f=6400, E=16, k=2, shared=0, T=8, dtype="bf16", layers=32, slots=4),
    "c5_mixtral_8x22b": dict(d=6144, f=16384, E=8, k=2, shared=0, T=32, dtype="bf16", layers=56, slots=2),
}


class Workload:
    """Canonical weights (numpy, for whoever wants to check results) + what the library needs."""

    def __init__(self, d, f, E, k, shared, dtype, layers, seed=0, distinct=None, gate_std=0.02, std=0.02):
        self.d, self.f, self.E, self.k, self.n_shared, self.dtype, self.n_layers, self.seed = d, f, E, k, shared, dtype, layers, seed
        self.distinct = distinct if distinct else layers * E
        self.gate = [si.gate_weights(seed, l, E, d, dtype, std=gate_std) for l in range(layers)]
        # distinct routed experts are generated as (layer 0.., expert 0..) in aliasing order
        self._experts = {}
        self._std = std
        self.shared = [[si.expert_weights(seed, l, s, d, f, dtype, std=std, shared=True) for s in range(shared)]
                       for l in range(layers)]

    def blob_index(self, layer, expert):
        return (layer * self.E + expert) % self.distinct

    def expert(self, layer, expert):
        """Canonical (W_gate, W_up, W_down) of routed expert (layer, expert)."""
        b = self.blob_index(layer, expert)
        if b not in self._experts:
            self._experts[b] = si.expert_weights(self.seed, b // self.E, b % self.E, self.d, self.f, self.dtype, std=self._std)
        return self._experts[b]

    def layer_experts(self, layer):
        return [self.expert(layer, e) for e in range(self.E)]

    def drop_canonical(self):
        self._experts = {}


def make_config(wl, max_tokens, slots=None, cutoff_layer=-1, pred_k=None, renorm=True):
    return sp.Config(n_layers=wl.n_layers, d_model=wl.d, d_ff=wl.f, n_experts=wl.E, top_k=wl.k, n_shared=wl.n_shared,
                     max_tokens=max_tokens, cache_slots_per_layer=slots if slots else wl.E,
                     weight_dtype=sp.BF16 if wl.dtype == "bf16" else sp.F32, renorm_topk=1 if renorm else 0,
                     pred_k=pred_k if pred_k is not None else wl.k, cutoff_layer=cutoff_layer)


class Loaded:
    """A context with every gate uploaded and every expert registered (pinned blobs kept alive here)."""

    def __init__(self, wl, cfg, stream=None, warm=True, keep_canonical=True):
        import torch
        self.wl, self.cfg = wl, cfg
        self.ctx = sp.Context(cfg, stream=stream)
        self.blobs = {}
        nbytes = sp.expert_blob_bytes(cfg)
        for l in range(wl.n_layers):
            g = torch.from_numpy(wl.gate[l].view(np.int16) if wl.dtype == "bf16" else wl.gate[l]).cuda()
            self.ctx.set_gate(l, g)
        for l in range(wl.n_layers):
            for e in range(wl.E):
                b = wl.blob_index(l, e)
                if b not in self.blobs:
                    pinned = torch.empty(nbytes, dtype=torch.uint8, pin_memory=True)
                    sp.pack_expert(cfg, *wl.expert(l, e), out=pinned.numpy())
                    self.blobs[b] = pinned
                    if not keep_canonical:
                        wl.drop_canonical()
                self.ctx.expert_cache_register(l, e, self.blobs[b])
            for s in range(wl.n_shared):
                pinned = torch.empty(nbytes, dtype=torch.uint8, pin_memory=True)
                sp.pack_expert(cfg, *wl.shared[l][s], out=pinned.numpy())
                self.ctx.expert_cache_register_shared(l, s, pinned)
        if warm and cfg.cache_slots_per_layer == wl.E:
            for l in range(wl.n_layers):
                self.ctx.expert_cache_warm(l, list(range(wl.E)))

    def close(self):
        self.ctx.destroy()
        self.blobs = {}
