// Internal declarations shared by the host runtime and the kernel launchers of libspmoe.
#ifndef SPMOE_INTERNAL_H
#define SPMOE_INTERNAL_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "spmoe.h"

#define SPMOE_MAX_ETOT (SPMOE_MAX_EXPERTS + SPMOE_MAX_SHARED)

// Byte offsets inside one packed expert blob.
//   bf16: [GU region: (f/16) N-tiles x (d/32) k-steps x {gate tile, up tile} x 1 KiB]
//         [D  region: (d/32) N-tile pairs x (f/32) k-steps x {tile of N-tile 2p, tile of N-tile 2p+1} x 1 KiB]
//         one 1 KiB tile = 64 lanes x 8 bf16; lane l holds row (l & 15), K elements 8*(l >> 4) .. +7
//         of the 16 x 32 block, i.e. exactly the A operand of v_mfma_f32_16x16x32_bf16.
//   fp32: W_gate[f][d], W_up[f][d], W_down[d][f] back to back, row-major.
static inline size_t spmoe_down_region_offset(int d, int f, int dtype) {
    return (size_t)2 * d * f * (dtype == SPMOE_BF16 ? 2 : 4);
}

// Device-side routing scratch of one context (reused by every layer).
struct SpmoeRouting {
    int32_t* idx;      // [Tmax][k]       selected experts, rank order
    float* w;          // [Tmax][k]       gating scores
    float* logits;     // [Tmax][E]
    void* xb;          // [Tmax][d]       the batch's hidden states rounded to bf16 (written by the routing kernel)
    int32_t* steal;    // [2] unit counters of the two expert GEMMs, zeroed by the routing kernel
};

// List of experts one GEMM launch works on, passed by value as a kernel argument.
struct SpmoeExpertList {
    int32_t n;
    uint16_t id[SPMOE_MAX_ETOT];        // expert id (routed: 0..E-1, shared: E..E+n_shared-1)
    const void* blob[SPMOE_MAX_ETOT];   // its packed weights in HBM
};

struct SpmoeShape {
    int32_t T, k, E, n_shared, d, f;
};

// Launchers (spmoe_kernels.hip).  All asynchronous on `stream`; return hipGetLastError().
hipError_t spmoe_launch_gate_topk(hipStream_t stream, int dtype, const float* x, const void* wg, int T, int E, int d,
                                  int k, int renorm, int32_t* idx, float* w, float* logits, int32_t* steal, void* xb);
hipError_t spmoe_launch_permute(hipStream_t stream, const int32_t* idx, int T, int k, int E, int32_t* counts,
                                int32_t* offsets, int32_t* perm);
hipError_t spmoe_launch_gate_up(hipStream_t stream, int dtype, const SpmoeShape& s, const SpmoeExpertList& list,
                                const SpmoeRouting& r, const float* x, void* h, int32_t* steal);
hipError_t spmoe_launch_down(hipStream_t stream, int dtype, const SpmoeShape& s, const SpmoeExpertList& list,
                             const SpmoeRouting& r, const void* h, float* ypart, int splits, int32_t* steal);
hipError_t spmoe_launch_combine(hipStream_t stream, const SpmoeShape& s, const SpmoeRouting& r, const float* ypart,
                                int splits, float* out);
// True if spmoe_create would accept the configuration; otherwise *why names the first offending field.
bool spmoe_config_ok(const spmoe_config* cfg, const char** why);
// Number of K-splits (partial-sum planes of ypart) the down projection uses for this shape and batch size
// (batches of more than 16 tokens use other instances of the kernel, which may split differently).
int spmoe_down_splits(int dtype, int d, int f, int T);
// plan of the bf16 expert GEMM of `projection` (0 gate/up, 1 down) for a batch of T tokens:
// splits, kw, ksw, nw, exact, LDS bytes
void spmoe_describe_plan(int projection, int d, int f, int T, int32_t out[6]);

#endif
