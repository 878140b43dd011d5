// spmoe_moe_layer_resident_static: the verify layer with every expert resident, for callers that cannot
// allocate device memory.  It runs the same four kernels as spmoe_moe_verify_layer; what that entry point
// keeps in buffers allocated by spmoe_create (the routing result, the unit counters, the intermediate h and the
// K-split partial outputs) lives here in one file-scope device array.
#include <hip/hip_runtime.h>

#include <mutex>

#include "spmoe_internal.h"

// Each GPU the library runs on holds its own copy of this array, at its own address, until the process ends.
static __device__ __align__(256) unsigned char scratch[SPMOE_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_mu;
unsigned char* g_scratch_ptr[kMaxDevices];   // device address of `scratch` on each device, once looked up

// The name `scratch` is only a handle in host code; the address kernels may use comes from the runtime.
hipError_t scratch_address(unsigned char** out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lk(g_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = static_cast<unsigned char*>(p);
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

size_t round256(size_t v) { return (v + 255) & ~(size_t)255; }

}  // namespace

extern "C" spmoe_status spmoe_moe_layer_resident_static(const spmoe_config* cfg, void* stream, const void* dev_gate,
                                                        const void* const* host_dev_blobs, const float* dev_x, int T,
                                                        float* dev_out) {
    const char* why = "";
    if (!spmoe_config_ok(cfg, &why)) return SPMOE_EINVAL;
    if (T < 0 || T > cfg->max_tokens) return SPMOE_ERANGE;
    if (T == 0) return SPMOE_OK;
    if (!dev_gate || !host_dev_blobs || !dev_x || !dev_out) return SPMOE_EINVAL;
    const int E = cfg->n_experts, n_shared = cfg->n_shared, k = cfg->top_k, d = cfg->d_model, f = cfg->d_ff;
    const int E_tot = E + n_shared;
    auto misaligned = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; };
    if (misaligned(dev_gate) || misaligned(dev_x) || misaligned(dev_out)) return SPMOE_EINVAL;
    for (int e = 0; e < E_tot; ++e)
        if (!host_dev_blobs[e] || misaligned(host_dev_blobs[e])) return SPMOE_EINVAL;

    // carve the array: unit counters first, then the routing result, h and the partial outputs of this call's T.
    // Nothing in it has to survive from call to call: the routing kernel zeroes the two counters (with plain
    // stores, so the call can be recorded into a HIP graph) and every other byte is written before it is read.
    const int dt = cfg->weight_dtype;
    const int splits = spmoe_down_splits(dt, d, f, T);
    const size_t A_tot = (size_t)T * k + (size_t)n_shared * T;
    size_t off = 0;
    auto take = [&](size_t bytes) { const size_t at = off; off += round256(bytes); return at; };
    const size_t o_counters = take(2 * sizeof(int32_t));
    const size_t o_idx = take(sizeof(int32_t) * T * k);
    const size_t o_w = take(sizeof(float) * T * k);
    const size_t o_logits = take(sizeof(float) * T * E);
    const size_t o_xb = take(sizeof(uint16_t) * T * d);
    const size_t o_h = take(A_tot * f * (dt == SPMOE_BF16 ? 2 : 4));
    const size_t o_ypart = take(sizeof(float) * splits * A_tot * d);
    if (off > (size_t)SPMOE_STATIC_SCRATCH_BYTES) return SPMOE_ERANGE;

    unsigned char* base = nullptr;
    if (scratch_address(&base) != hipSuccess) {
        (void)hipGetLastError();
        return SPMOE_EHIP;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    SpmoeRouting r;
    r.steal = reinterpret_cast<int32_t*>(base + o_counters);
    r.idx = reinterpret_cast<int32_t*>(base + o_idx);
    r.w = reinterpret_cast<float*>(base + o_w);
    r.logits = reinterpret_cast<float*>(base + o_logits);
    r.xb = base + o_xb;
    void* h = base + o_h;
    float* ypart = reinterpret_cast<float*>(base + o_ypart);

    SpmoeExpertList list;
    list.n = 0;
    for (int s = 0; s < n_shared; ++s) { list.id[list.n] = (uint16_t)(E + s); list.blob[list.n] = host_dev_blobs[E + s]; list.n += 1; }
    for (int e = 0; e < E; ++e) { list.id[list.n] = (uint16_t)e; list.blob[list.n] = host_dev_blobs[e]; list.n += 1; }
    const SpmoeShape sh{T, k, E, n_shared, d, f};

    if (spmoe_launch_gate_topk(st, dt, dev_x, dev_gate, T, E, d, k, cfg->renorm_topk, r.idx, r.w, r.logits, r.steal, r.xb) !=
        hipSuccess) return SPMOE_EHIP;
    if (spmoe_launch_gate_up(st, dt, sh, list, r, dev_x, h, r.steal) != hipSuccess) return SPMOE_EHIP;
    if (spmoe_launch_down(st, dt, sh, list, r, h, ypart, splits, r.steal + 1) != hipSuccess) return SPMOE_EHIP;
    if (spmoe_launch_combine(st, sh, r, ypart, splits, dev_out) != hipSuccess) return SPMOE_EHIP;
    return SPMOE_OK;
}
