"""ctypes binding of libspmoe.so.  Same names as the C ABI (include/spmoe.h) minus the ``spmoe_`` prefix."""
import ctypes
import os

import numpy as np

_DIR = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_DIR, "libspmoe.so")
_lib = None

F32, BF16 = 0, 1
MAX_TOKENS, MAX_EXPERTS, MAX_SHARED, MAX_TOPK = 32, 128, 8, 8

_STATUS = {0: "SPMOE_OK", 1: "SPMOE_EINVAL", 2: "SPMOE_ERANGE", 3: "SPMOE_ENOMEM", 4: "SPMOE_ESTATE",
           5: "SPMOE_EHIP", 6: "SPMOE_ENOTIMPL"}

# every symbol include/spmoe.h declares
DECLARED_SYMBOLS = [
    "spmoe_create", "spmoe_destroy", "spmoe_sync", "spmoe_last_error", "spmoe_expert_blob_bytes",
    "spmoe_pack_expert", "spmoe_set_gate", "spmoe_expert_cache_register", "spmoe_expert_cache_register_shared",
    "spmoe_expert_cache_warm", "spmoe_expert_cache_lookup", "spmoe_expert_cache_contents",
    "spmoe_expert_cache_reset", "spmoe_expert_cache_stats", "spmoe_set_cutoff", "spmoe_gate_topk",
    "spmoe_token_permutation", "spmoe_predict_experts", "spmoe_prefetch", "spmoe_moe_verify_layer",
    "spmoe_profile_begin", "spmoe_profile_collect", "spmoe_last_layer_kernel_ms",
    "spmoe_suggest_cutoff", "spmoe_measure_expert_load_ms", "spmoe_predict_prefetch_async", "spmoe_prefetch_drain",
    "spmoe_gemm_plan", "spmoe_moe_layer_resident_static",
]


class SpmoeError(RuntimeError):
    def __init__(self, status, where, detail=""):
        self.status = status
        self.status_name = _STATUS.get(status, str(status))
        super().__init__("%s failed: %s %s" % (where, self.status_name, detail))


class Config(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "n_layers", "d_model", "d_ff", "n_experts", "top_k", "n_shared", "max_tokens",
        "cache_slots_per_layer", "weight_dtype", "renorm_topk", "pred_k", "cutoff_layer")]

    def __init__(self, n_layers=1, d_model=0, d_ff=0, n_experts=0, top_k=0, n_shared=0, max_tokens=32,
                 cache_slots_per_layer=None, weight_dtype=BF16, renorm_topk=1, pred_k=None, cutoff_layer=-1):
        super().__init__(n_layers, d_model, d_ff, n_experts, top_k, n_shared, max_tokens,
                         n_experts if cache_slots_per_layer is None else cache_slots_per_layer,
                         weight_dtype, renorm_topk, top_k if pred_k is None else pred_k, cutoff_layer)


class Stats(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int64) for n in (
        "hits", "misses", "late_hits", "evictions", "prefetch_issued", "prefetch_used", "prefetch_wasted",
        "ondemand_loads", "h2d_bytes_prefetch", "h2d_bytes_ondemand")]

    def as_dict(self):
        return {n: int(getattr(self, n)) for n, _ in self._fields_}


class ProfileRecord(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("layer", ctypes.c_int32), ("expert", ctypes.c_int32),
                ("reserved", ctypes.c_int32), ("t_begin_ms", ctypes.c_float), ("t_end_ms", ctypes.c_float)]


def lib_path():
    return _LIB_PATH


def load_library():
    """Loads libspmoe.so.  torch is imported first so that the HIP runtime the library binds to is the
    one torch already loaded (streams and device pointers are shared with it)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError("libspmoe.so is not built: run `python -m paper_2510_10302_amd.build` "
                          "(there is no CPU fallback for the SP-MoE hot path)")
    import torch  # noqa: F401
    lib = ctypes.CDLL(_LIB_PATH, mode=ctypes.RTLD_GLOBAL)
    vp, i32, cp = ctypes.c_void_p, ctypes.c_int, ctypes.POINTER(Config)
    sig = {
        "spmoe_create": (i32, [cp, vp, ctypes.POINTER(vp)]),
        "spmoe_destroy": (i32, [vp]),
        "spmoe_sync": (i32, [vp]),
        "spmoe_last_error": (ctypes.c_char_p, [vp]),
        "spmoe_expert_blob_bytes": (ctypes.c_size_t, [cp]),
        "spmoe_pack_expert": (i32, [cp, vp, vp, vp, vp]),
        "spmoe_set_gate": (i32, [vp, i32, vp]),
        "spmoe_expert_cache_register": (i32, [vp, i32, i32, vp]),
        "spmoe_expert_cache_register_shared": (i32, [vp, i32, i32, vp]),
        "spmoe_expert_cache_warm": (i32, [vp, i32, vp, i32]),
        "spmoe_expert_cache_lookup": (i32, [vp, i32, i32, vp]),
        "spmoe_expert_cache_contents": (i32, [vp, i32, vp, vp]),
        "spmoe_expert_cache_reset": (i32, [vp]),
        "spmoe_expert_cache_stats": (i32, [vp, ctypes.POINTER(Stats)]),
        "spmoe_set_cutoff": (i32, [vp, i32]),
        "spmoe_gate_topk": (i32, [vp, i32, vp, i32, i32, vp, vp, vp]),
        "spmoe_token_permutation": (i32, [vp, vp, i32, i32, vp, vp, vp]),
        "spmoe_predict_experts": (i32, [vp, i32, vp, i32, vp, vp]),
        "spmoe_prefetch": (i32, [vp, i32, vp, i32]),
        "spmoe_moe_verify_layer": (i32, [vp, i32, vp, i32, vp]),
        "spmoe_profile_begin": (i32, [vp, i32]),
        "spmoe_profile_collect": (i32, [vp, vp, i32, vp]),
        "spmoe_last_layer_kernel_ms": (i32, [vp, vp]),
        "spmoe_suggest_cutoff": (i32, [i32, i32, i32, ctypes.c_double, ctypes.c_double, ctypes.c_double,
                                       ctypes.c_double, ctypes.c_double, vp]),
        "spmoe_measure_expert_load_ms": (i32, [vp, i32, i32, i32, vp]),
        "spmoe_predict_prefetch_async": (i32, [vp, i32, vp, i32]),
        "spmoe_prefetch_drain": (i32, [vp]),
        "spmoe_gemm_plan": (i32, [cp, i32, vp]),
        "spmoe_moe_layer_resident_static": (i32, [cp, vp, vp, vp, vp, i32, vp]),
    }
    assert sorted(sig) == sorted(DECLARED_SYMBOLS)
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    _lib = lib
    return lib


def expert_blob_bytes(cfg):
    return int(load_library().spmoe_expert_blob_bytes(ctypes.byref(cfg)))


def pack_expert(cfg, w_gate, w_up, w_down, out=None):
    """Canonical row-major numpy matrices (uint16 bf16 bits or float32) -> packed blob (uint8 numpy array,
    or written into `out`, any writable buffer exposing ``ctypes.data``/``data_ptr`` of the right size)."""
    lib = load_library()
    nbytes = expert_blob_bytes(cfg)
    if nbytes == 0:
        raise SpmoeError(1, "spmoe_expert_blob_bytes", "bad config")
    want = np.uint16 if cfg.weight_dtype == BF16 else np.float32
    mats = []
    for m, shape in ((w_gate, (cfg.d_ff, cfg.d_model)), (w_up, (cfg.d_ff, cfg.d_model)), (w_down, (cfg.d_model, cfg.d_ff))):
        m = np.ascontiguousarray(m)
        if m.dtype != want or m.shape != shape:
            raise ValueError("expert matrix must be %s of shape %s, got %s %s" % (want.__name__, shape, m.dtype, m.shape))
        mats.append(m)
    if out is None:
        out = np.empty(nbytes, dtype=np.uint8)
    ptr = _host_ptr(out)
    st = lib.spmoe_pack_expert(ctypes.byref(cfg), mats[0].ctypes.data, mats[1].ctypes.data, mats[2].ctypes.data, ptr)
    if st != 0:
        raise SpmoeError(st, "spmoe_pack_expert")
    return out


def suggest_cutoff(n_layers, n_layers_draft, k, t_comp, t_io, m_peak, m_expert, m_gpu):
    """Largest cutoff layer allowed by the paper's memory and overlap constraints (-1: none)."""
    out = ctypes.c_int32(-2)
    st = load_library().spmoe_suggest_cutoff(n_layers, n_layers_draft, k, t_comp, t_io, m_peak, m_expert, m_gpu,
                                             ctypes.addressof(out))
    if st != 0:
        raise SpmoeError(st, "spmoe_suggest_cutoff")
    return out.value


def gemm_plan(cfg, projection):
    """Tiling of the gate/up (0) or down (1) expert GEMM: dict(splits, k_waves, k_steps, n_sub, exact, tokens_per_pass, lds_bytes)."""
    out = (ctypes.c_int32 * 6)()
    st = load_library().spmoe_gemm_plan(ctypes.byref(cfg), projection, ctypes.addressof(out))
    if st != 0:
        raise SpmoeError(st, "spmoe_gemm_plan")
    return dict(splits=out[0], k_waves=out[1], k_steps=out[2], n_sub=out[3], exact=bool(out[4] & 1),
                tokens_per_pass=32 if out[4] & 2 else 16, lds_bytes=out[5])


def moe_layer_resident_static(cfg, dev_gate, dev_blobs, dev_x, dev_out, stream=None):
    """The resident verify layer without a context and without any allocation (fixed device scratch array).
    dev_blobs: device tensors holding the packed routed experts 0..E-1, then the shared ones."""
    import torch
    lib = load_library()
    if len(dev_blobs) != cfg.n_experts + cfg.n_shared:
        raise ValueError("expected %d blobs" % (cfg.n_experts + cfg.n_shared))
    ptrs = (ctypes.c_void_p * len(dev_blobs))(*[_dev_ptr(b) for b in dev_blobs])
    stream = stream if stream is not None else torch.cuda.current_stream()
    st = lib.spmoe_moe_layer_resident_static(ctypes.byref(cfg), ctypes.c_void_p(stream.cuda_stream), _dev_ptr(dev_gate),
                                             ptrs, _dev_ptr(dev_x, torch.float32), dev_x.shape[0],
                                             _dev_ptr(dev_out, torch.float32))
    if st != 0:
        raise SpmoeError(st, "spmoe_moe_layer_resident_static")


def _host_ptr(buf):
    if isinstance(buf, np.ndarray):
        return buf.ctypes.data
    return buf.data_ptr()          # a (pinned) CPU torch tensor


def _dev_ptr(t, dtype=None):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous device tensor")
    if dtype is not None and t.dtype != dtype:
        raise ValueError("expected dtype %s, got %s" % (dtype, t.dtype))
    return t.data_ptr()


class Context:
    """Owns one spmoe_ctx.  Keeps references to every borrowed tensor (gates, pinned blobs) alive."""

    def __init__(self, cfg, stream=None):
        import torch
        self.lib = load_library()
        self.cfg = cfg
        self._torch = torch
        self._keep = []
        self.stream = stream if stream is not None else torch.cuda.current_stream()
        handle = ctypes.c_void_p()
        st = self.lib.spmoe_create(ctypes.byref(cfg), ctypes.c_void_p(self.stream.cuda_stream), ctypes.byref(handle))
        if st != 0:
            raise SpmoeError(st, "spmoe_create")
        self.h = handle

    def _check(self, st, where):
        if st != 0:
            raise SpmoeError(st, where, self.lib.spmoe_last_error(self.h).decode())

    def destroy(self):
        if self.h is not None:
            self.lib.spmoe_destroy(self.h)
            self.h = None
            self._keep = []

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def sync(self):
        self._check(self.lib.spmoe_sync(self.h), "spmoe_sync")

    # ---- storage -----------------------------------------------------------------------------------
    def set_gate(self, layer, dev_wg):
        self._keep.append(dev_wg)
        self._check(self.lib.spmoe_set_gate(self.h, layer, _dev_ptr(dev_wg)), "spmoe_set_gate")

    def expert_cache_register(self, layer, expert, pinned_blob):
        self._keep.append(pinned_blob)
        self._check(self.lib.spmoe_expert_cache_register(self.h, layer, expert, _host_ptr(pinned_blob)),
                    "spmoe_expert_cache_register")

    def expert_cache_register_shared(self, layer, idx, pinned_blob):
        self._check(self.lib.spmoe_expert_cache_register_shared(self.h, layer, idx, _host_ptr(pinned_blob)),
                    "spmoe_expert_cache_register_shared")

    def expert_cache_warm(self, layer, experts):
        arr = np.ascontiguousarray(experts, dtype=np.int32)
        self._check(self.lib.spmoe_expert_cache_warm(self.h, layer, arr.ctypes.data, arr.size), "spmoe_expert_cache_warm")

    def expert_cache_lookup(self, layer, expert):
        out = ctypes.c_int32(-2)
        self._check(self.lib.spmoe_expert_cache_lookup(self.h, layer, expert, ctypes.addressof(out)),
                    "spmoe_expert_cache_lookup")
        return out.value

    def expert_cache_contents(self, layer):
        buf = np.empty(max(self.cfg.cache_slots_per_layer, 1), dtype=np.int32)
        n = ctypes.c_int32(0)
        self._check(self.lib.spmoe_expert_cache_contents(self.h, layer, buf.ctypes.data, ctypes.addressof(n)),
                    "spmoe_expert_cache_contents")
        return buf[: n.value].tolist()

    def expert_cache_reset(self):
        self._check(self.lib.spmoe_expert_cache_reset(self.h), "spmoe_expert_cache_reset")

    def expert_cache_stats(self):
        s = Stats()
        self._check(self.lib.spmoe_expert_cache_stats(self.h, ctypes.byref(s)), "spmoe_expert_cache_stats")
        return s.as_dict()

    def set_cutoff(self, cutoff_layer):
        self._check(self.lib.spmoe_set_cutoff(self.h, cutoff_layer), "spmoe_set_cutoff")
        self.cfg.cutoff_layer = cutoff_layer

    # ---- hot path ----------------------------------------------------------------------------------
    def gate_topk(self, layer, dev_x, k, dev_idx, dev_w, dev_logits=None):
        t = self._torch
        T = dev_x.shape[0]
        self._check(self.lib.spmoe_gate_topk(self.h, layer, _dev_ptr(dev_x, t.float32), T, k, _dev_ptr(dev_idx, t.int32),
                                             _dev_ptr(dev_w, t.float32), _dev_ptr(dev_logits, t.float32)),
                    "spmoe_gate_topk")

    def token_permutation(self, dev_idx, dev_counts, dev_offsets, dev_perm):
        t = self._torch
        T, k = dev_idx.shape
        self._check(self.lib.spmoe_token_permutation(self.h, _dev_ptr(dev_idx, t.int32), T, k, _dev_ptr(dev_counts, t.int32),
                                                     _dev_ptr(dev_offsets, t.int32), _dev_ptr(dev_perm, t.int32)),
                    "spmoe_token_permutation")

    def predict_experts(self, layer, dev_draft_x):
        n = dev_draft_x.shape[0]
        ids = np.empty(self.cfg.n_experts, dtype=np.int32)
        cnt = ctypes.c_int32(0)
        self._check(self.lib.spmoe_predict_experts(self.h, layer, _dev_ptr(dev_draft_x, self._torch.float32), n,
                                                   ids.ctypes.data, ctypes.addressof(cnt)), "spmoe_predict_experts")
        return ids[: cnt.value].tolist()

    def prefetch(self, layer, experts):
        arr = np.ascontiguousarray(experts, dtype=np.int32)
        self._check(self.lib.spmoe_prefetch(self.h, layer, arr.ctypes.data, arr.size), "spmoe_prefetch")

    def predict_prefetch_async(self, layer, dev_draft_x):
        self._check(self.lib.spmoe_predict_prefetch_async(self.h, layer, _dev_ptr(dev_draft_x, self._torch.float32),
                                                          dev_draft_x.shape[0]), "spmoe_predict_prefetch_async")

    def prefetch_drain(self):
        self._check(self.lib.spmoe_prefetch_drain(self.h), "spmoe_prefetch_drain")

    def moe_verify_layer(self, layer, dev_x, dev_out):
        t = self._torch
        self._check(self.lib.spmoe_moe_verify_layer(self.h, layer, _dev_ptr(dev_x, t.float32), dev_x.shape[0],
                                                    _dev_ptr(dev_out, t.float32)), "spmoe_moe_verify_layer")

    # ---- measurement -------------------------------------------------------------------------------
    def profile_begin(self, per_kernel=True, log_only=False):
        mode = 2 if log_only else (1 if per_kernel else 0)
        self._check(self.lib.spmoe_profile_begin(self.h, mode), "spmoe_profile_begin")

    def profile_collect(self, cap=65536):
        recs = (ProfileRecord * cap)()
        n = ctypes.c_int32(0)
        self._check(self.lib.spmoe_profile_collect(self.h, ctypes.addressof(recs), cap, ctypes.addressof(n)),
                    "spmoe_profile_collect")
        return [dict(kind=r.kind, layer=r.layer, expert=r.expert, t0=r.t_begin_ms, t1=r.t_end_ms)
                for r in recs[: min(n.value, cap)]]

    def measure_expert_load_ms(self, layer, expert, repeats=3):
        ms = ctypes.c_float(0)
        self._check(self.lib.spmoe_measure_expert_load_ms(self.h, layer, expert, repeats, ctypes.addressof(ms)),
                    "spmoe_measure_expert_load_ms")
        return ms.value

    def last_layer_kernel_ms(self):
        ms = (ctypes.c_float * 4)()
        self._check(self.lib.spmoe_last_layer_kernel_ms(self.h, ctypes.addressof(ms)), "spmoe_last_layer_kernel_ms")
        return list(ms)
