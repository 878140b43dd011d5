// HIP kernels of the SP-MoE verify-layer hot path for gfx950 (CDNA4, wave64).
//
//   gate_topk_kernel     gate logits + softmax + top-k + gating scores (Eq. 1's G(x); Alg. 1's
//                        Gates[l](s) and TopK_Index), one workgroup per token; also leaves the batch
//                        rounded to bf16 for the expert path.
//   expert_gemm_kernel   the grouped SwiGLU expert FFN (Eq. 1's E_i(x)) as two skinny GEMMs whose A
//                        operand is the streamed weight tile and whose B operand is the token tile
//                        (16 tokens held in registers; a second 16 re-read from L2 in the instances for
//                        batches of more than 16 tokens); bf16 x bf16 -> fp32 on v_mfma_f32_16x16x32_bf16.
//                        Its prologue groups the assignments by expert in LDS.
//   expert_gemm_f32_kernel  the same contraction for fp32 weights on the vector ALU.
//   combine_kernel       out[t] = sum_r w[t][r] * y[t][r] (+ shared experts), fixed summation order.
//
// The expert GEMMs are bound by streaming each active expert's weights from HBM exactly once: with a
// handful of tokens per expert every weight byte feeds one MFMA.  Weights are therefore stored
// pre-tiled (see spmoe_internal.h) so that one wave-wide 16-byte-per-lane load is a contiguous 1 KiB
// line group that is already in MFMA A-operand order, and the two tiles of a k-step are adjacent; no LDS
// staging of weights is needed.
#include <hip/hip_runtime.h>
#include <limits.h>
#include <math.h>
#include <stdio.h>
#include <stdlib.h>

#include <type_traits>

#include "spmoe_internal.h"

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

// ---------------------------------------------------------------------------------------------
// wave-level helpers (DPP within rows of 16 lanes, readlane across the four rows)
// ---------------------------------------------------------------------------------------------
#define DPP_QUAD_SWAP1 0xB1      // quad_perm [1,0,3,2]
#define DPP_QUAD_SWAP2 0x4E      // quad_perm [2,3,0,1]
#define DPP_ROW_HALF_MIRROR 0x141
#define DPP_ROW_MIRROR 0x140

template <int CTRL>
__device__ __forceinline__ float dpp_mov_f(float v) {
    int i = __builtin_bit_cast(int, v);
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(i, i, CTRL, 0xF, 0xF, false));
}
template <int CTRL>
__device__ __forceinline__ int dpp_mov_i(int v) {
    return __builtin_amdgcn_update_dpp(v, v, CTRL, 0xF, 0xF, false);
}
__device__ __forceinline__ float readlane_f(float v, int lane) {
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}

// Sum over the 64 lanes; every lane gets the same value, the order of additions is fixed.
__device__ __forceinline__ float wave_sum(float v) {
    v += dpp_mov_f<DPP_QUAD_SWAP1>(v);
    v += dpp_mov_f<DPP_QUAD_SWAP2>(v);
    v += dpp_mov_f<DPP_ROW_HALF_MIRROR>(v);
    v += dpp_mov_f<DPP_ROW_MIRROR>(v);
    return (readlane_f(v, 0) + readlane_f(v, 16)) + (readlane_f(v, 32) + readlane_f(v, 48));
}
__device__ __forceinline__ float wave_max(float v) {
    v = fmaxf(v, dpp_mov_f<DPP_QUAD_SWAP1>(v));
    v = fmaxf(v, dpp_mov_f<DPP_QUAD_SWAP2>(v));
    v = fmaxf(v, dpp_mov_f<DPP_ROW_HALF_MIRROR>(v));
    v = fmaxf(v, dpp_mov_f<DPP_ROW_MIRROR>(v));
    return fmaxf(fmaxf(readlane_f(v, 0), readlane_f(v, 16)), fmaxf(readlane_f(v, 32), readlane_f(v, 48)));
}
__device__ __forceinline__ int wave_min_i(int v) {
    v = min(v, dpp_mov_i<DPP_QUAD_SWAP1>(v));
    v = min(v, dpp_mov_i<DPP_QUAD_SWAP2>(v));
    v = min(v, dpp_mov_i<DPP_ROW_HALF_MIRROR>(v));
    v = min(v, dpp_mov_i<DPP_ROW_MIRROR>(v));
    return min(min(__builtin_amdgcn_readlane(v, 0), __builtin_amdgcn_readlane(v, 16)),
               min(__builtin_amdgcn_readlane(v, 32), __builtin_amdgcn_readlane(v, 48)));
}

// Inclusive prefix sum over the 64 lanes: Hillis-Steele inside each row of 16 (row_shr, lanes without a
// source keep 0), then the last lane of row 0 / row 2 is added to row 1 / row 3 (row_bcast:15) and lane 31
// to rows 2 and 3 (row_bcast:31).
__device__ __forceinline__ int wave_inclusive_scan(int v) {
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xF, 0xF, false);   // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xF, 0xF, false);   // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xF, 0xF, false);   // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xF, 0xF, false);   // row_shr:8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xA, 0xF, false);   // row_bcast:15 into rows 1 and 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xC, 0xF, false);   // row_bcast:31 into rows 2 and 3
    return v;
}

// 16-byte load from a pointer known to be device memory.  Pointers that reach a kernel inside a struct are generic
// to the compiler, and loads through them become flat loads, which count against both memory counters (so a wait
// for LDS also waits for them) and keep their addresses in register pairs.
__device__ __forceinline__ u32x4 load_global_16(const void* p) {
    return *reinterpret_cast<const __attribute__((address_space(1))) u32x4*>(
        (const __attribute__((address_space(1))) void*)p);
}

template <typename T>
__device__ __forceinline__ void store_global(T* p, T v) {
    *reinterpret_cast<__attribute__((address_space(1))) T*>((__attribute__((address_space(1))) void*)p) = v;
}

// fp32 -> bf16 bits, round to nearest even (finite inputs)
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
    uint32_t u = __builtin_bit_cast(uint32_t, f);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    return f32_to_bf16_bits(lo) | (f32_to_bf16_bits(hi) << 16);
}

// ---------------------------------------------------------------------------------------------
// Token -> expert grouping of T*k routed assignments (+ n_shared*T shared-expert assignments).
// Runs inside one workgroup (256 or 512 threads); s_idx / s_cnt / s_scan are workgroup LDS arrays.
//   counts[e], offsets[e] (exclusive prefix, E_tot + 1 entries), perm = assignment ids a = t*k + r
//   expert by expert, ascending inside an expert (a stable counting sort).  Shared expert s owns the
//   assignments T*k + s*T + t, t = 0..T-1.
// ---------------------------------------------------------------------------------------------
#define GROUP_MAX_A (SPMOE_MAX_TOKENS * SPMOE_MAX_TOPK)   // 256 routed assignments at most

__device__ void group_assignments(const int32_t* idx, int T, int k, int E, int n_shared, int32_t* counts,
                                  int32_t* offsets, int32_t* perm, int* s_idx, int* s_cnt, int* s_scan) {
    const int tid = threadIdx.x, nthr = blockDim.x;
    const int A = T * k;
    const int E_tot = E + n_shared;
    for (int e = tid; e < 2 * 256; e += nthr) s_cnt[e] = 0;
    __syncthreads();
    for (int a = tid; a < A; a += nthr) {
        int e = __hip_atomic_load(idx + a, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        e = min(max(e, 0), E - 1);
        s_idx[a] = e;
        atomicAdd(&s_cnt[e], 1);
    }
    for (int s = tid; s < n_shared; s += nthr) s_cnt[E + s] = T;
    __syncthreads();
    // exclusive scan of the counts by wave 0: four consecutive experts per lane, DPP scan of the lane totals
    if (tid < 64) {
        int c[4];
        int tot = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) { c[q] = s_cnt[4 * tid + q]; tot += c[q]; }
        int run = wave_inclusive_scan(tot) - tot;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int e = 4 * tid + q;
            if (e < E_tot) { counts[e] = c[q]; offsets[e] = run; }
            s_scan[e] = run;                  // s_scan now holds the offsets
            run += c[q];
        }
        if (tid == 0) offsets[E_tot] = A + n_shared * T;
    }
    __syncthreads();
    for (int a = tid; a < A; a += nthr) {
        const int e = s_idx[a];
        int rank = 0;
#pragma unroll 8
        for (int b = 0; b < a; ++b) rank += (s_idx[b] == e);
        perm[s_scan[e] + rank] = a;
    }
    for (int a = A + tid; a < A + n_shared * T; a += nthr) perm[a] = a;
}

// ---------------------------------------------------------------------------------------------
// K1: gate logits + softmax + top-k.  Grid = T, block = 4 or 8 waves.  The token-to-expert grouping
// is not done here: every workgroup of the expert GEMMs derives it from idx in LDS (a few hundred integers),
// which costs less than a second pass over all tokens behind a device-wide arrival counter would.
// ---------------------------------------------------------------------------------------------
// Raw 8-element weight chunk (16 bytes of bf16 or 32 bytes of fp32) and its dot product with 8 x values.
template <typename WT> struct Chunk8;
template <> struct Chunk8<uint16_t> {
    u32x4 v;
    __device__ __forceinline__ void load(const uint16_t* p) { v = *reinterpret_cast<const u32x4*>(p); }
    __device__ __forceinline__ float dot(const float4& xa, const float4& xb, float a) const {
        a = fmaf(xa.x, __builtin_bit_cast(float, v[0] << 16), a); a = fmaf(xa.y, __builtin_bit_cast(float, v[0] & 0xFFFF0000u), a);
        a = fmaf(xa.z, __builtin_bit_cast(float, v[1] << 16), a); a = fmaf(xa.w, __builtin_bit_cast(float, v[1] & 0xFFFF0000u), a);
        a = fmaf(xb.x, __builtin_bit_cast(float, v[2] << 16), a); a = fmaf(xb.y, __builtin_bit_cast(float, v[2] & 0xFFFF0000u), a);
        a = fmaf(xb.z, __builtin_bit_cast(float, v[3] << 16), a); a = fmaf(xb.w, __builtin_bit_cast(float, v[3] & 0xFFFF0000u), a);
        return a;
    }
};
template <> struct Chunk8<float> {
    float4 lo, hi;
    __device__ __forceinline__ void load(const float* p) {
        lo = *reinterpret_cast<const float4*>(p);
        hi = *reinterpret_cast<const float4*>(p + 4);
    }
    __device__ __forceinline__ float dot(const float4& xa, const float4& xb, float a) const {
        a = fmaf(xa.x, lo.x, a); a = fmaf(xa.y, lo.y, a); a = fmaf(xa.z, lo.z, a); a = fmaf(xa.w, lo.w, a);
        a = fmaf(xb.x, hi.x, a); a = fmaf(xb.y, hi.y, a); a = fmaf(xb.z, hi.z, a); a = fmaf(xb.w, hi.w, a);
        return a;
    }
};

// logits[e] = sum_j x[j] * Wg[e][j] for the experts of this wave: EPW experts per pass and wave.
// xb_row (may be NULL): wave 0 also stores its x chunks rounded to bf16 there, for the expert GEMMs' token tiles.
template <typename WT, int EPW>
__device__ __forceinline__ void gate_logits_pass(const float* __restrict__ xt, const WT* __restrict__ wg, int E, int d,
                                                 int wave, int lane, float* s_logit, uint16_t* __restrict__ xb_row) {
    constexpr int KI = (sizeof(WT) == 2 ? 16 : 8) / EPW;      // chunks per lane and round
    const int nwaves = blockDim.x >> 6;
    for (int e0 = wave * EPW; e0 < E; e0 += nwaves * EPW) {
        float acc[EPW];
#pragma unroll
        for (int q = 0; q < EPW; ++q) acc[q] = 0.f;
        for (int jb = 0; jb < d; jb += 64 * 8 * KI) {
            float4 xa[KI], xb[KI];
            Chunk8<WT> w[KI][EPW];
#pragma unroll
            for (int i = 0; i < KI; ++i) {
                const int j = jb + (i * 64 + lane) * 8;
                if (j < d) {
                    xa[i] = *reinterpret_cast<const float4*>(xt + j);
                    xb[i] = *reinterpret_cast<const float4*>(xt + j + 4);
#pragma unroll
                    for (int q = 0; q < EPW; ++q)
                        if (e0 + q < E) w[i][q].load(wg + (size_t)(e0 + q) * d + j);
                }
            }
            if (xb_row != nullptr && e0 == 0) {          // wave 0, its first pass: every chunk of the row once
#pragma unroll
                for (int i = 0; i < KI; ++i) {
                    const int j = jb + (i * 64 + lane) * 8;
                    if (j < d)
                        *reinterpret_cast<u32x4*>(xb_row + j) = u32x4{pack_bf16x2(xa[i].x, xa[i].y), pack_bf16x2(xa[i].z, xa[i].w),
                                                                      pack_bf16x2(xb[i].x, xb[i].y), pack_bf16x2(xb[i].z, xb[i].w)};
                }
            }
#pragma unroll
            for (int i = 0; i < KI; ++i) {
                const int j = jb + (i * 64 + lane) * 8;
                if (j < d) {
#pragma unroll
                    for (int q = 0; q < EPW; ++q)
                        if (e0 + q < E) acc[q] = w[i][q].dot(xa[i], xb[i], acc[q]);
                }
            }
        }
#pragma unroll
        for (int q = 0; q < EPW; ++q)
            if (e0 + q < E) {
                const float sum = wave_sum(acc[q]);
                if (lane == 0) s_logit[e0 + q] = sum;
            }
    }
}

template <typename WT, int EPW, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void gate_topk_kernel(const float* __restrict__ x, const WT* __restrict__ wg,
                                                        int T, int E, int d, int k, int renorm,
                                                        int32_t* __restrict__ idx_out, float* __restrict__ w_out,
                                                        float* __restrict__ logits_out, int32_t* steal,
                                                        uint16_t* __restrict__ xb_out) {
    __shared__ float s_logit[SPMOE_MAX_EXPERTS];

    const int t = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float* xt = x + (size_t)t * d;
    // the unit counters of the two expert GEMMs that follow start at zero
    if (steal != nullptr && t == 0 && tid < 2) steal[tid] = 0;

    // ---- gate logits: each wave scores EPW experts per pass; all loads of a round (KI chunks of 8
    //      elements per lane, for every expert of the pass) are issued before the arithmetic starts
    uint16_t* xb_row = (xb_out != nullptr && wave == 0) ? xb_out + (size_t)t * d : nullptr;
    gate_logits_pass<WT, EPW>(xt, wg, E, d, wave, lane, s_logit, xb_row);
    __syncthreads();
    if (wave != 0) return;

    // ---- wave 0: softmax and k rounds of wave-wide argmax (lane l owns experts l and l + 64)
    float v[2];
    bool taken[2];
    float lmax = -INFINITY;
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        const int e = lane + 64 * q;
        float l = (e < E) ? s_logit[e] : -INFINITY;
        if (e < E && logits_out) logits_out[(size_t)t * E + e] = l;
        if (!(l == l)) l = -INFINITY;            // NaN never wins
        v[q] = l;
        taken[q] = !(e < E);
        lmax = fmaxf(lmax, l);
    }
    const float m = wave_max(lmax);
    float psum = 0.f;
#pragma unroll
    for (int q = 0; q < 2; ++q) psum += (lane + 64 * q < E) ? expf(v[q] - m) : 0.f;
    const float denom = wave_sum(psum);

    int sel_i[SPMOE_MAX_TOPK];
    float sel_p[SPMOE_MAX_TOPK];
    float sel_sum = 0.f;
#pragma unroll
    for (int r = 0; r < SPMOE_MAX_TOPK; ++r) {
        sel_i[r] = 0; sel_p[r] = 0.f;
        if (r < k) {
            // best untaken candidate of this lane; the lower index wins a tie
            float bv = -INFINITY;
            int bi = INT_MAX;
#pragma unroll
            for (int q = 1; q >= 0; --q)
                if (!taken[q] && (v[q] >= bv)) { bv = v[q]; bi = lane + 64 * q; }
            const float best = wave_max(bi == INT_MAX ? -INFINITY : bv);
            int win;
            if (E <= 64) {
                // one expert per lane: the lowest set bit of the ballot is the lowest index
                const unsigned long long b = __builtin_amdgcn_ballot_w64(bi != INT_MAX && bv == best);
                win = b ? (__builtin_ctzll(b)) : INT_MAX;
            } else {
                win = wave_min_i((bi != INT_MAX && bv == best) ? bi : INT_MAX);
            }
            if (win == INT_MAX) win = 0;          // cannot happen for k <= E; keeps the index in range
            if ((win & 63) == lane) {
                if (win >> 6) taken[1] = true; else taken[0] = true;
            }
            const float p = expf(best - m) / denom;
            sel_i[r] = win;
            sel_p[r] = p;
            sel_sum += p;
        }
    }
    // lane r writes the r-th selection (one store instruction for the whole row)
#pragma unroll
    for (int r = 0; r < SPMOE_MAX_TOPK; ++r)
        if (r < k && lane == r) {
            idx_out[(size_t)t * k + r] = sel_i[r];
            w_out[(size_t)t * k + r] = renorm ? sel_p[r] / sel_sum : sel_p[r];
        }
}

// Stand-alone grouping of a routing result (one workgroup).
__global__ __launch_bounds__(256) void permute_kernel(const int32_t* idx, int T, int k, int E, int32_t* counts,
                                                      int32_t* offsets, int32_t* perm) {
    __shared__ int s_idx[GROUP_MAX_A];
    __shared__ int s_cnt[512];
    __shared__ int s_scan[256];
    group_assignments(idx, T, k, E, 0, counts, offsets, perm, s_idx, s_cnt, s_scan);
}

// ---------------------------------------------------------------------------------------------
// K2 / K3: grouped skinny GEMM on MFMA, persistent workgroups.
//
// Work unit = (group, K-split, N-tile): a group is one expert of the launch's list together with a
// tile of <= 16 of its tokens; an N-tile is 16 weight rows.  All units of a launch are numbered
// group-major and cut into gridDim.x equal contiguous ranges, one per workgroup, so every workgroup
// streams the same number of weight bytes whatever the routing was; launches of 8-wave workgroups keep the
// last eighth of the units out of the ranges and hand them out one by one through an atomic counter.
//
// Inside a workgroup the W waves split the K range of a unit (KSW k-steps each, 1 KiB per matrix per
// k-step).  A wave keeps its slice of the token tile as the MFMA B operand in registers (reloaded only
// when the group or K-split changes), streams weight tiles from HBM through a register ring of PF
// k-steps that runs across unit boundaries, and the W partial 16x16 results of a unit are summed
// through a double-buffered LDS area in wave order (deterministic), one barrier per unit.
//
// MODE_GU   : A = interleaved W_gate / W_up tiles, B = x rows gathered through perm (fp32 -> bf16 on
//             load); epilogue h[a][n] = silu(g) * u stored as bf16.  A unit covers one N-tile.
// MODE_DOWN : A = W_down tiles of two consecutive N-tiles, B = h rows (bf16); epilogue
//             ypart[split][a][n] = partial y (fp32).  A unit covers 32 weight rows.
//
// MFMA 16x16x32 operand layout used here: A lane l = row (l & 15), K = 8*(l >> 4) .. +7; B lane l =
// column (l & 15), same K; D lane l = column (l & 15), rows 4*(l >> 4) .. +3.
//
// The MFMA chain is branch-free: k-steps past the end of a ragged K range run with zero operands.
// ---------------------------------------------------------------------------------------------
enum { MODE_GU = 0, MODE_DOWN = 1 };

#define GEMM_MAX_GROUPS (2 * SPMOE_MAX_ETOT)
#define GEMM_MAX_ASSIGN (SPMOE_MAX_TOKENS * (SPMOE_MAX_TOPK + SPMOE_MAX_SHARED))

struct GemmParams {
    const int32_t* idx;   // [T][k] routing result: expert of assignment a = t*k + r
    const float* x;       // MODE_GU input  [T][d] (fp32-weight kernels)
    const uint16_t* xb;   // MODE_GU input  [T][d] rounded to bf16 by the routing kernel (MFMA kernels)
    uint16_t* h;          // [A_tot][f] bf16 bits: MODE_GU output, MODE_DOWN input
    float* ypart;         // MODE_DOWN output [splits][A_tot][d]
    int32_t T, k, d, f;
    int32_t A_tot;        // T*k + n_shared*T
    int32_t E;            // routed experts
    int32_t E_tot;        // routed + shared experts
    int32_t ks_total;     // k-steps of the contraction: d/32 (GU), f/32 (DOWN)
    int32_t ks_split;     // k-steps per K-split
    int32_t splits;       // K-splits
    int32_t n_tiles;      // units along N: (f/16)/nw (GU), (d/32)/nw (DOWN)
    int32_t waves;        // waves per workgroup = kw * nw
    int32_t kw;           // waves that split the K range of one N sub-tile
    int32_t nw;           // N sub-tiles a workgroup works on side by side (each kw waves)
    int32_t* steal;       // zeroed counter handing out the last units of the launch one by one, or NULL
    int32_t dyn_div;      // the last 1/dyn_div of the units goes through that counter
    int32_t dyn_force;    // 1: use the counter whatever the launch shape (testing)
};

// largest divisor of ksw that is <= limit (the ring must divide the per-unit step count so that ring
// slots keep static register indices across units)
constexpr int ring_depth(int ksw, int limit) {
    int best = 1;
    for (int v = 1; v <= limit; ++v)
        if (ksw % v == 0) best = v;
    return best;
}

template <int MODE, int KSW, bool EXACT, int NTOK>
__global__ __launch_bounds__(((KSW > 14 || NTOK == 2) ? 8 : 16) * 64) void expert_gemm_kernel(const SpmoeExpertList list,
                                                                                               const GemmParams p) {
    // Two weight tiles are in flight per k-step, adjacent KiB of the blob that share the B operand: gate and up
    // tile of one N-tile in MODE_GU, the tiles of two consecutive N-tiles in MODE_DOWN.
    constexpr int NMAT = 2;
    constexpr int PF = ring_depth(KSW, 4);
    constexpr int STEP = 128;                             // 16-byte units between consecutive k-steps of a stream
    constexpr size_t soff = 64;                           // second tile of the k-step
    extern __shared__ float s_mem[];
    float* s_red = s_mem;                                 // [2][waves][NMAT][NTOK][64 lanes][4]
    const void** s_blob = reinterpret_cast<const void**>(s_mem + 2 * p.waves * NMAT * NTOK * 256);   // [SPMOE_MAX_ETOT] copy of list.blob
    int* s_grp = reinterpret_cast<int*>(s_blob + SPMOE_MAX_ETOT);             // [GEMM_MAX_GROUPS + 1]
    int* s_base = s_grp + GEMM_MAX_GROUPS + 1;            // [SPMOE_MAX_ETOT] start of the expert's run in s_perm, -1: not in this launch
    int* s_cnt = s_base + SPMOE_MAX_ETOT;                 // [SPMOE_MAX_ETOT] assignments of the expert
    unsigned* s_mask = reinterpret_cast<unsigned*>(s_cnt + SPMOE_MAX_ETOT);   // [SPMOE_MAX_EXPERTS] bit t: token t chose the expert
    int* s_idx = reinterpret_cast<int*>(s_mask + SPMOE_MAX_EXPERTS);          // [GROUP_MAX_A] expert of each routed assignment
    int* s_perm = s_idx + GROUP_MAX_A;                    // [GEMM_MAX_ASSIGN] assignments expert by expert, in list order
    int* s_next = s_perm + GEMM_MAX_ASSIGN;               // [2] unit handed to the workgroup two iterations ahead
    int* s_lid = s_next + 2;                              // [SPMOE_MAX_ETOT] copy of list.id

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform over the wave: keeps unit addressing in SGPRs
    const int n = lane & 15, kg = lane >> 4;
    const int kslice = wave % p.kw, nsub = wave / p.kw;  // this wave's K slice and N sub-tile of the unit
    const int K = (MODE == MODE_GU) ? p.d : p.f;          // contraction length
    const int N = (MODE == MODE_GU) ? p.f : p.d;          // output features
    const int upg = p.splits * p.n_tiles;                 // units per group
    const int A = p.T * p.k;                              // routed assignments

    // ---- token -> expert grouping, by every workgroup for itself (T <= 32 tokens, so one 32-bit mask per expert
    //      says which tokens chose it: its popcount is the expert's load, the popcount below bit t the rank of
    //      token t's assignment inside the expert -- a stable counting sort without a second pass over idx)
    //      Everything the prologue needs from global memory is requested at once: the routing result and the
    //      launch list (kernel arguments indexed at run time are memory loads too).
    int ev[4];                                            // A <= 256 assignments, >= 64 threads
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int a = tid + q * blockDim.x;
        ev[q] = (a < A) ? p.idx[a] : 0;
    }
    for (int i = tid; i < list.n; i += blockDim.x) {
        s_lid[i] = list.id[i];
        s_blob[i] = list.blob[i];
    }
    for (int e = tid; e < p.E_tot; e += blockDim.x) {
        if (e < p.E) s_mask[e] = 0u;
        s_base[e] = -1;
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int a = tid + q * blockDim.x;
        if (a < A) {
            const int e = min(max(ev[q], 0), p.E - 1);
            s_idx[a] = e;
            atomicOr(&s_mask[e], 1u << (a / p.k));
        }
    }
    __syncthreads();
    // ---- wave 0: the launch's experts in list order -> runs in s_perm, active groups (list entry, token tile of
    //      <= 16 tokens), and the unit schedule of this workgroup
    long long U = 0;
    int U_dyn = 0, U_st = 0, u1 = 0;
    // thread 0 only: takes the next unit off the counter, -1 once they are all handed out
    auto grab = [&]() -> int {
        if (U_dyn == 0) return -1;
        const int v = U_st + atomicAdd(p.steal, 1);
        return v < (int)U ? v : -1;
    };
    // thread 0 only: the unit after u in this workgroup's schedule, -1 at its end
    auto successor = [&](int u) -> int {
        if (u < 0) return -1;
        return (u + 1 < u1) ? u + 1 : grab();
    };
    if (wave == 0) {
        int base = 0;                                     // packed running totals: groups << 16 | assignments
        for (int i0 = 0; i0 < list.n; i0 += 64) {
            const int i = i0 + lane;
            int e = 0, cnt = 0;
            if (i < list.n) {
                e = s_lid[i];
                cnt = (e < p.E) ? __builtin_popcount(s_mask[e]) : p.T;
            }
            // NTOK = 1: a group is a tile of <= 16 of the expert's tokens; NTOK = 2: all (<= 32) of them
            const int tiles = (NTOK == 2) ? (cnt > 0 ? 1 : 0) : ((cnt + 15) >> 4);
            const int both = (tiles << 16) | cnt;         // <= 2 tiles and <= 32 assignments per entry: no carry
            const int excl = wave_inclusive_scan(both) - both + base;
            if (i < list.n) {
                s_base[e] = excl & 0xFFFF;
                s_cnt[e] = cnt;
                for (int t = 0; t < tiles; ++t) s_grp[(excl >> 16) + t] = i * 2 + t;
            }
            base = __builtin_amdgcn_readlane(excl + both, 63);
        }
        // Unit schedule: the first units are cut into gridDim.x equal contiguous ranges; the last 1/dyn_div is handed
        // out one unit at a time through an atomic counter, so workgroups that stream faster (the XCDs do not all
        // see the same bandwidth) take more of it and all finish together.  Which workgroup computes a unit does
        // not change its value.  A stolen unit usually costs a reload of the token tile, so the tail only pays
        // where finish times spread widely.  Measured, that is the launches with one 8-wave workgroup per CU
        // (down projection at d = 6144, f = 16384: 8 % faster); with 11- and 16-wave workgroups it changed the
        // gate/up projection by -1 % ... +1 % and slowed the down projection by 3 %, so those keep the static split.
        U = (long long)(base >> 16) * upg;
        const bool dyn = p.steal != nullptr && (p.dyn_force || (U >= 10ll * gridDim.x && blockDim.x <= 512));
        U_dyn = dyn ? (int)(U / p.dyn_div) : 0;
        U_st = (int)U - U_dyn;
        const int u0 = (int)((long long)U_st * blockIdx.x / gridDim.x);
        u1 = (int)((long long)U_st * (blockIdx.x + 1) / gridDim.x);
        if (lane == 0) {
            const int first = (u0 < u1) ? u0 : grab();
            s_next[0] = first;
            s_next[1] = successor(first);
        }
    }
    __syncthreads();
    int cur = s_next[0], nxt = s_next[1];
    if (cur < 0) return;                                  // uniform over the workgroup

    const bf16x8 zero8 = __builtin_bit_cast(bf16x8, u32x4{0u, 0u, 0u, 0u});
    const size_t region = (MODE == MODE_DOWN) ? (size_t)2 * p.d * p.f * sizeof(uint16_t) : 0;

    // weight stream address of unit u for this wave (16-byte units), and its live k-step count
    auto unit_ptr = [&](int u, int& nks) -> const bf16x8* {
        const int g = u / upg, rem = u - g * upg;
        const int s = rem / p.n_tiles, nt = rem - s * p.n_tiles;
        const int li = s_grp[g] >> 1;
        const int ks_lo = s * p.ks_split + kslice * KSW;
        const int ks_hi = min(min(ks_lo + KSW, (s + 1) * p.ks_split), p.ks_total);
        nks = EXACT ? KSW : max(ks_hi - ks_lo, 0);
        const char* blob = static_cast<const char*>(s_blob[li]) + region;
        const size_t sub = (size_t)nt * p.nw + nsub;                                   // this wave's sub-tile (pair of tiles)
        return reinterpret_cast<const bf16x8*>(blob) + (sub * p.ks_total + ks_lo) * STEP + lane;
    };

    int nks = KSW;
    const bf16x8* wp = unit_ptr(cur, nks);
    bf16x8 ring[PF][NMAT];
#pragma unroll
    for (int j = 0; j < PF; ++j) {
#pragma unroll
        for (int m = 0; m < NMAT; ++m) {
            ring[j][m] = zero8;
            if (EXACT || j < nks) ring[j][m] = __builtin_nontemporal_load(wp + (size_t)j * STEP + m * soff);
        }
    }

    // ---- while the first weight tiles are on their way: the runs of s_perm.  Routed assignments by rank inside
    //      their expert, shared experts' assignments in token order (shared expert s owns A + s*T + t).
    for (int a = tid; a < A; a += blockDim.x) {
        const int e = s_idx[a];
        const int b = s_base[e];
        if (b >= 0) s_perm[b + __builtin_popcount(s_mask[e] & ((1u << (a / p.k)) - 1u))] = a;
    }
    for (int a = A + tid; a < p.A_tot; a += blockDim.x) {
        const int sidx = (a - A) / p.T;
        const int b = s_base[p.E + sidx];
        if (b >= 0) s_perm[b + (a - A) - sidx * p.T] = a;
    }
    // LDS writes done, then workgroup barrier (s_next is rewritten inside the loop); the weight loads keep flying
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");

    bf16x8 xr[KSW];
    int cur_gs = -1;                                      // group * splits + split held in xr
    int beg = 0, cnt = 0;
    int a_out = -1;                                       // assignment this thread writes in the epilogue
    int buf = 0;
    // NTOK = 2 only: the B operand of the group's second token tile (tokens 16..31) does not fit in registers
    // beside the first one; it is re-read for every unit, k-step by k-step, through a small ring of its own.  It
    // is the same KSW KiB per wave for every unit of a group, so these loads hit in the L2 and cost no HBM traffic.
    constexpr int PF1 = (NTOK == 2) ? ((KSW > 28 && PF >= 2) ? 2 : PF) : 1;   // 32 k-steps of first tile leave room for 2
    bf16x8 ring1[PF1];
    const uint16_t* brow1 = nullptr;                      // this lane's row of the second tile, NULL: no such token
    bool two = false;                                     // the current group has more than 16 tokens

    for (int it = 0; cur >= 0; ++it) {
        const int u = cur;
        const int g = u / upg, rem = u - g * upg;
        const int s = rem / p.n_tiles, nt = rem - s * p.n_tiles;
        int succ = -1;
        if (tid == 0) succ = successor(nxt);             // its latency hides behind this unit's k-steps

        // ---- token tile (B operand) of this wave's K range; reloaded when the group or split changes
        if (g * p.splits + s != cur_gs) {
            cur_gs = g * p.splits + s;
            const int gi = s_grp[g];
            const int e = s_lid[gi >> 1];
            beg = s_base[e] + 16 * (gi & 1);
            cnt = min(16 * NTOK, s_cnt[e] - 16 * (gi & 1));
            const int ks_lo = s * p.ks_split + kslice * KSW;
            const int a_n = (n < min(cnt, 16)) ? s_perm[beg + n] : -1;
            {   // the output this thread writes first in the epilogue: token (tid & 255) >> 4 of tile tid >> 8
                const int tok = ((NTOK == 2) ? (tid >> 8) * 16 : 0) + ((tid & 255) >> 4);
                a_out = (tok < cnt && ((tid & 255) >> 4) < 16) ? s_perm[beg + tok] : -1;
            }
            // rows of the B operand: the token's hidden state (rounded to bf16 by the routing kernel) for gate/up,
            // the assignment's intermediate h for down
            const int routed = p.T * p.k;
            auto row_of = [&](int a) -> int {
                if (a < 0) return 0;
                if (MODE == MODE_DOWN) return a;
                return a < routed ? a / p.k : (a - routed) % p.T;
            };
            const uint16_t* bsrc = ((MODE == MODE_GU) ? p.xb : p.h) + ks_lo * 32 + kg * 8;
            const uint16_t* brow = bsrc + (size_t)row_of(a_n) * K;
#pragma unroll
            for (int j = 0; j < KSW; ++j) {
                u32x4 packed = {0u, 0u, 0u, 0u};
                if (a_n >= 0 && (EXACT || j < nks)) packed = load_global_16(brow + j * 32);
                xr[j] = __builtin_bit_cast(bf16x8, packed);
            }
            if (NTOK == 2) {
                two = cnt > 16;
                const int a_1 = (two && n < cnt - 16) ? s_perm[beg + 16 + n] : -1;
                brow1 = (a_1 >= 0) ? bsrc + (size_t)row_of(a_1) * K : nullptr;
#pragma unroll
                for (int j = 0; j < PF1; ++j) {
                    u32x4 packed = {0u, 0u, 0u, 0u};
                    if (brow1 != nullptr && (EXACT || j < nks)) packed = load_global_16(brow1 + j * 32);
                    ring1[j] = __builtin_bit_cast(bf16x8, packed);
                }
            }
        }

        // ---- stream the unit's KSW k-steps; the ring refills from this unit, then from the next one
        int nks_next = 0;
        const bf16x8* wp_next = (nxt >= 0) ? unit_ptr(nxt, nks_next) : nullptr;
        f32x4 acc[NMAT], acc1[NMAT];
#pragma unroll
        for (int m = 0; m < NMAT; ++m) { acc[m] = f32x4{0.f, 0.f, 0.f, 0.f}; acc1[m] = f32x4{0.f, 0.f, 0.f, 0.f}; }
        // one straight-line MFMA chain per case (a branch per k-step would sit between the MFMAs)
        auto k_steps = [&](auto second_tile) __attribute__((always_inline)) {
            constexpr bool SECOND = decltype(second_tile)::value;
#pragma unroll
            for (int j = 0; j < KSW; ++j) {
                bf16x8 a[NMAT];
#pragma unroll
                for (int m = 0; m < NMAT; ++m) a[m] = ring[j % PF][m];
                if (j + PF < KSW) {
#pragma unroll
                    for (int m = 0; m < NMAT; ++m) {
                        ring[j % PF][m] = zero8;
                        if (EXACT || j + PF < nks)
                            ring[j % PF][m] = __builtin_nontemporal_load(wp + (size_t)(j + PF) * STEP + m * soff);
                    }
                } else {
#pragma unroll
                    for (int m = 0; m < NMAT; ++m) {
                        ring[j % PF][m] = zero8;
                        if (wp_next != nullptr && (EXACT || j + PF - KSW < nks_next))
                            ring[j % PF][m] = __builtin_nontemporal_load(wp_next + (size_t)(j + PF - KSW) * STEP + m * soff);
                    }
                }
#pragma unroll
                for (int m = 0; m < NMAT; ++m) acc[m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[m], xr[j], acc[m], 0, 0, 0);
                if (SECOND) {
                    // second tile: the same weight tiles against tokens 16..31.  Its operand ring refills from the
                    // same rows: later steps of this unit, then the first steps again for the next unit (a change
                    // of group or K-split reloads them above).
                    const bf16x8 b1 = ring1[j % PF1];
                    const int jn = (j + PF1 < KSW) ? j + PF1 : j + PF1 - KSW;
                    u32x4 packed = {0u, 0u, 0u, 0u};
                    if (brow1 != nullptr && (EXACT || jn < nks)) packed = load_global_16(brow1 + jn * 32);
                    ring1[j % PF1] = __builtin_bit_cast(bf16x8, packed);
#pragma unroll
                    for (int m = 0; m < NMAT; ++m) acc1[m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[m], b1, acc1[m], 0, 0, 0);
                }
            }
        };
        if (NTOK == 2 && two) k_steps(std::true_type{});
        else k_steps(std::false_type{});
        wp = wp_next;
        nks = nks_next;

        // ---- cross-wave reduction through LDS (buffer `buf`), summed in wave order
        float* red = s_red + buf * (p.waves * NMAT * NTOK * 256);
#pragma unroll
        for (int m = 0; m < NMAT; ++m) {
            *reinterpret_cast<f32x4*>(red + (((wave * NMAT + m) * NTOK) * 64 + lane) * 4) = acc[m];
            if (NTOK == 2 && two) *reinterpret_cast<f32x4*>(red + (((wave * NMAT + m) * NTOK + 1) * 64 + lane) * 4) = acc1[m];
        }
        if (tid == 0) s_next[it & 1] = succ;
        // LDS writes done, then workgroup barrier; outstanding weight loads keep flying across it
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        cur = nxt;
        nxt = s_next[it & 1];
        // o -> (sub-tile or token tile, token on, feature fi), consecutive threads on consecutive features; small
        // workgroups take several outputs per thread.  The kw partial sums of a sub-tile are added in wave order.
        // (NTOK = 2 launches have one N sub-tile; `sub` then is the token tile.)
        for (int o = tid; o < 256 * (NTOK == 2 ? (two ? 2 : 1) : p.nw); o += blockDim.x) {
            const int sub = o >> 8, fi = o & 15, on = (o & 255) >> 4;
            const int tok = (NTOK == 2) ? sub * 16 + on : on;        // position in the group
            if (tok >= cnt) continue;
            const int a_o = (o == tid) ? a_out : s_perm[beg + tok];
            const int src = (((fi >> 2) * 16 + on) * 4) + (fi & 3);
            float s0 = 0.f, s1 = 0.f;
            if (NTOK == 2) {
                for (int w = 0; w < p.kw; ++w) {
                    s0 += red[((w * NMAT) * NTOK + sub) * 256 + src];
                    s1 += red[((w * NMAT + 1) * NTOK + sub) * 256 + src];
                }
            } else {
                for (int w = sub * p.kw; w < (sub + 1) * p.kw; ++w) {
                    s0 += red[(w * NMAT) * 256 + src];
                    s1 += red[(w * NMAT + 1) * 256 + src];
                }
            }
            const int st = (NTOK == 2) ? nt : nt * p.nw + sub;     // sub-tile index along N
            if (MODE == MODE_GU) {
                const float hval = (s0 / (1.f + expf(-s0))) * s1;
                store_global(p.h + (size_t)a_o * N + st * 16 + fi, (uint16_t)f32_to_bf16_bits(hval));
            } else {
                float* y = p.ypart + ((size_t)s * p.A_tot + a_o) * N + st * 32 + fi;
                store_global(y, s0);
                store_global(y + 16, s1);
            }
        }
        buf ^= 1;
    }
}

// ---------------------------------------------------------------------------------------------
// fp32-weight variant on the vector ALU (small configurations).  Blob = W_gate[f][d], W_up[f][d],
// W_down[d][f] row-major.  One wave per output row; tokens of the expert in chunks of 8.
// h is fp32 [A_tot][f] here.
// ---------------------------------------------------------------------------------------------
template <int MODE>
__global__ __launch_bounds__(256) void expert_gemm_f32_kernel(const SpmoeExpertList list, const GemmParams p,
                                                              float* __restrict__ h32) {
    __shared__ unsigned s_tokens;                  // bit t: token t chose this block's expert
    __shared__ int s_asg[SPMOE_MAX_TOKENS];        // the expert's assignments, ascending
    const int li = blockIdx.y;
    const int e = list.id[li];
    const int routed = p.T * p.k;
    // the assignments of this block's expert, straight from the routing result
    if (threadIdx.x == 0) s_tokens = 0u;
    __syncthreads();
    if (e < p.E)
        for (int a = threadIdx.x; a < routed; a += blockDim.x)
            if (min(max(p.idx[a], 0), p.E - 1) == e) atomicOr(&s_tokens, 1u << (a / p.k));
    __syncthreads();
    const unsigned tokens = (e < p.E) ? s_tokens : (p.T >= 32 ? ~0u : ((1u << p.T) - 1u));
    if (e < p.E) {
        for (int a = threadIdx.x; a < routed; a += blockDim.x)
            if (min(max(p.idx[a], 0), p.E - 1) == e) s_asg[__builtin_popcount(tokens & ((1u << (a / p.k)) - 1u))] = a;
    } else if ((int)threadIdx.x < p.T) {
        s_asg[threadIdx.x] = routed + (e - p.E) * p.T + threadIdx.x;
    }
    __syncthreads();
    const int beg = 0, end = __builtin_popcount(tokens);
    if (end <= beg) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int K = (MODE == MODE_GU) ? p.d : p.f;
    const int N = (MODE == MODE_GU) ? p.f : p.d;
    const int row = blockIdx.x * 4 + wave;
    if (row >= N) return;
    const float* blob = static_cast<const float*>(list.blob[li]);
    const float* w0 = (MODE == MODE_GU) ? blob + (size_t)row * K : blob + (size_t)2 * p.d * p.f + (size_t)row * K;
    const float* w1 = blob + (size_t)p.d * p.f + (size_t)row * K;   // W_up row (MODE_GU only)

    for (int c = beg; c < end; c += 8) {
        float a0[8], a1[8];
        const float* xin[8];
        int asg[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            a0[i] = 0.f; a1[i] = 0.f;
            asg[i] = (c + i < end) ? s_asg[c + i] : -1;
            const int a = max(asg[i], 0);
            if (MODE == MODE_GU) {
                const int tok = a < routed ? a / p.k : (a - routed) % p.T;
                xin[i] = p.x + (size_t)tok * K;
            } else {
                xin[i] = h32 + (size_t)a * K;
            }
        }
        for (int j = lane * 4; j < K; j += 256) {
            const float4 wa = *reinterpret_cast<const float4*>(w0 + j);
            float4 wb = {0.f, 0.f, 0.f, 0.f};
            if (MODE == MODE_GU) wb = *reinterpret_cast<const float4*>(w1 + j);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                if (asg[i] < 0) continue;
                const float4 xv = *reinterpret_cast<const float4*>(xin[i] + j);
                a0[i] = fmaf(xv.x, wa.x, a0[i]); a0[i] = fmaf(xv.y, wa.y, a0[i]);
                a0[i] = fmaf(xv.z, wa.z, a0[i]); a0[i] = fmaf(xv.w, wa.w, a0[i]);
                if (MODE == MODE_GU) {
                    a1[i] = fmaf(xv.x, wb.x, a1[i]); a1[i] = fmaf(xv.y, wb.y, a1[i]);
                    a1[i] = fmaf(xv.z, wb.z, a1[i]); a1[i] = fmaf(xv.w, wb.w, a1[i]);
                }
            }
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (asg[i] < 0) continue;                    // uniform over the wave
            const float g = wave_sum(a0[i]);
            if (MODE == MODE_GU) {
                const float u = wave_sum(a1[i]);
                if (lane == 0) h32[(size_t)asg[i] * N + row] = (g / (1.f + expf(-g))) * u;
            } else {
                if (lane == 0) p.ypart[(size_t)asg[i] * N + row] = g;
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// K4: weighted combination (Eq. 1).  out[t][j] = sum_r w[t][r] * y[t*k + r][j] + sum_s y[shared s, t][j]
// where y[a] = sum over K-splits of ypart[split][a], every sum in ascending index order.
// Grid = (ceil(d / 1024), T), block = 256, four columns per thread.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void combine_kernel(const float* __restrict__ ypart, const float* __restrict__ w,
                                                      int T, int k, int n_shared, int d, int splits,
                                                      float* __restrict__ out) {
    const int t = blockIdx.y;
    const int j = (blockIdx.x * 256 + threadIdx.x) * 4;
    if (j >= d) return;
    const int A_tot = T * k + n_shared * T;
    float4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int r = 0; r < k + n_shared; ++r) {
        const int a = (r < k) ? t * k + r : T * k + (r - k) * T + t;
        float4 y = {0.f, 0.f, 0.f, 0.f};
        for (int s = 0; s < splits; ++s) {
            const float4 v = *reinterpret_cast<const float4*>(ypart + ((size_t)s * A_tot + a) * d + j);
            y.x += v.x; y.y += v.y; y.z += v.z; y.w += v.w;
        }
        const float g = (r < k) ? w[t * k + r] : 1.f;
        acc.x += g * y.x; acc.y += g * y.y; acc.z += g * y.z; acc.w += g * y.w;
    }
    *reinterpret_cast<float4*>(out + (size_t)t * d + j) = acc;
}

// ---------------------------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------------------------
// Experts per wave and pass (EPW) and waves per workgroup are chosen so that, where the shape allows, a lane has
// all its loads of the token in flight at once (one round: 16 / EPW chunks of 8 bf16 weights per lane and expert,
// 8 / EPW for fp32) and every expert is scored in one pass.  The choice depends on E and d only, so a token's
// logits do not depend on the batch it arrives in.
template <typename WT, int EPW>
static void launch_gate_topk_waves(hipStream_t stream, int waves, const float* x, const WT* wg, int T, int E, int d, int k,
                                   int renorm, int32_t* idx, float* w, float* logits, int32_t* steal, uint16_t* xb) {
    if (waves <= 4)
        hipLaunchKernelGGL((gate_topk_kernel<WT, EPW, 4>), dim3(T), dim3(256), 0, stream, x, wg, T, E, d, k, renorm, idx, w,
                           logits, steal, xb);
    else   // more experts than 8 waves score in one pass take further passes (16 waves would leave 128 registers: spills)
        hipLaunchKernelGGL((gate_topk_kernel<WT, EPW, 8>), dim3(T), dim3(512), 0, stream, x, wg, T, E, d, k, renorm, idx, w,
                           logits, steal, xb);
}

template <typename WT>
static void launch_gate_topk_typed(hipStream_t stream, const float* x, const WT* wg, int T, int E, int d, int k, int renorm,
                                   int32_t* idx, float* w, float* logits, int32_t* steal, uint16_t* xb) {
    const int chunks = (d / 8 + 63) / 64;                       // 8-element chunks per lane
    const int ki_max = sizeof(WT) == 2 ? 16 : 8;
    const int epw = (ki_max / 4 >= chunks) ? 4 : ((ki_max / 2 >= chunks) ? 2 : 1);
    const int waves = (E + epw - 1) / epw;
    if (epw == 4) launch_gate_topk_waves<WT, 4>(stream, waves, x, wg, T, E, d, k, renorm, idx, w, logits, steal, xb);
    else if (epw == 2) launch_gate_topk_waves<WT, 2>(stream, waves, x, wg, T, E, d, k, renorm, idx, w, logits, steal, xb);
    else launch_gate_topk_waves<WT, 1>(stream, waves, x, wg, T, E, d, k, renorm, idx, w, logits, steal, xb);
}

hipError_t spmoe_launch_gate_topk(hipStream_t stream, int dtype, const float* x, const void* wg, int T, int E, int d,
                                  int k, int renorm, int32_t* idx, float* w, float* logits, int32_t* steal, void* xb) {
    if (dtype == SPMOE_BF16)
        launch_gate_topk_typed<uint16_t>(stream, x, static_cast<const uint16_t*>(wg), T, E, d, k, renorm, idx, w, logits,
                                         steal, static_cast<uint16_t*>(xb));
    else
        launch_gate_topk_typed<float>(stream, x, static_cast<const float*>(wg), T, E, d, k, renorm, idx, w, logits, steal,
                                      nullptr);
    return hipGetLastError();
}

hipError_t spmoe_launch_permute(hipStream_t stream, const int32_t* idx, int T, int k, int E, int32_t* counts,
                                int32_t* offsets, int32_t* perm) {
    hipLaunchKernelGGL(permute_kernel, dim3(1), dim3(256), 0, stream, idx, T, k, E, counts, offsets, perm);
    return hipGetLastError();
}

// Factorisation of a GEMM: K-splits x kw waves along K x ksw k-steps per wave, and nw N sub-tiles side by side.
struct GemmPlan {
    int splits, kw, ksw, nw;
    bool exact;
    int ntok = 1;     // token tiles of an expert taken per pass over its weights: 1 (16 tokens) or 2 (32 tokens)
    int waves() const { return kw * nw; }
};

static const int kExactKsw[] = {32, 28, 24, 16, 14, 12, 11, 10, 8, 4};

static bool is_exact_ksw(int ksw) {
    for (int v : kExactKsw)
        if (v == ksw) return true;
    return false;
}

// Workgroups of more than 8 waves leave 128 VGPRs per lane, enough for 14 k-steps of token tile.
static bool plan_ok(int waves, int ksw) { return waves >= 1 && waves <= 16 && (ksw <= 14 || waves <= 8); }

// ks_total: k-steps of the contraction; n_units: N-tiles (GU) or N-tile pairs (DOWN); env: optional override
// "splits,kw,ksw,nw" (tuning aid).  two_tiles: plan for the instances that take up to 32 tokens of an expert in
// one pass over its weights (batches of more than 16 tokens): at most 8 waves, one N sub-tile.
// k-steps per wave the two-tile instances can hold in registers (256 VGPRs at 8 waves per workgroup): the second
// tile's ring and accumulators come on top of the first tile's KSW * 4 registers.
constexpr int two_tile_max_ksw(int mode) { return mode == MODE_GU ? 28 : 32; }

static GemmPlan plan_gemm(int ks_total, int n_units, int max_splits, const char* env, bool two_tiles, int mode) {
    const char* force = getenv(env);
    if (force) {
        int s = 0, kw = 0, ksw = 0, nw = 0;
        if (sscanf(force, "%d,%d,%d,%d", &s, &kw, &ksw, &nw) == 4 && s >= 1 && s <= max_splits && nw >= 1 &&
            s * kw * ksw == ks_total && n_units % nw == 0 && is_exact_ksw(ksw) && plan_ok(kw * nw, ksw) &&
            (!two_tiles || (kw <= 8 && nw == 1 && ksw <= two_tile_max_ksw(mode)))) {
            GemmPlan fp{s, kw, ksw, nw, true};
            fp.ntok = two_tiles ? 2 : 1;
            return fp;
        }
    }
    if (two_tiles) {
        // 8 waves first (most bytes in flight), then anything exact with at least 4 waves; never more K-splits than
        // the one-tile plan of the shape uses (shorter units pay the per-unit barrier more often: measured 7 % on the
        // down projection at d = 6144, f = 16384).  Shapes without such a plan keep the one-tile plan, and an expert
        // with more than 16 tokens then streams its weights once per tile in that projection.
        const GemmPlan one = plan_gemm(ks_total, n_units, max_splits, env, false, mode);
        static const int kKswTwo[] = {16, 24, 28, 32, 12, 14, 8, 11, 10, 4};
        for (int min_kw : {8, 4}) {
            for (int splits = 1; splits <= one.splits; splits *= 2) {
                if (ks_total % splits) break;
                const int per = ks_total / splits;
                for (int ksw : kKswTwo) {
                    if (per % ksw || ksw > two_tile_max_ksw(mode)) continue;
                    const int kw = per / ksw;
                    if (kw >= min_kw && kw <= 8) { GemmPlan tp{splits, kw, ksw, 1, true}; tp.ntok = 2; return tp; }
                }
            }
        }
        if (!one.exact && one.waves() <= 8) { GemmPlan tp = one; tp.ntok = 2; return tp; }   // the generic instance has a two-tile form
        return one;
    }
    // gate/up: 8 waves of at most 16 k-steps where the contraction divides that way.  Measured against the 16-wave
    // plans: 3 % faster at d = 4096 (8 x 16, with the dynamic tail of the unit schedule, which 8-wave launches use),
    // 2 % at d = 2048 (8 x 8, two workgroups per CU); 8 x 24 at d = 6144 is 0.5 % slower than 16 x 12 and is not taken.
    if (mode == MODE_GU) {
        for (int ksw : {16, 8, 12, 14})
            if (ks_total == 8 * ksw) return GemmPlan{1, 8, ksw, 1, true};
    }
    // otherwise (measured, the differences are small): as few K-splits as possible, one N sub-tile, 9..16 waves
    static const int kKswPreference[] = {12, 8, 11, 14, 16, 4, 10, 24, 28, 32};
    for (int splits = 1; splits <= max_splits; splits *= 2) {
        if (ks_total % splits) break;
        const int per = ks_total / splits;
        for (int nw : {1, 2, 4}) {
            if (n_units % nw) continue;
            for (int ksw : kKswPreference) {
                if (per % ksw) continue;
                const int kw = per / ksw, waves = kw * nw;
                if (!plan_ok(waves, ksw)) continue;
                if (waves > 8 || (waves == 8 && ksw > 14)) return GemmPlan{splits, kw, ksw, nw, true};
            }
        }
    }
    for (int splits = 1; splits <= max_splits; splits *= 2) {       // any exact plan with at least 4 waves
        if (ks_total % splits) break;
        const int per = ks_total / splits;
        for (int ksw : kKswPreference) {
            if (per % ksw) continue;
            const int kw = per / ksw;
            if (kw >= 4 && plan_ok(kw, ksw)) return GemmPlan{splits, kw, ksw, 1, true};
        }
    }
    for (int ksw : kExactKsw) {                                      // tiny contractions: any exact plan
        if (ks_total % ksw) continue;
        if (plan_ok(ks_total / ksw, ksw)) return GemmPlan{1, ks_total / ksw, ksw, 1, true};
    }
    // generic instance: up to 8 waves of at most 32 k-steps each, more K-splits for longer contractions
    int splits = 1;
    while ((ks_total + splits - 1) / splits > 8 * 32) ++splits;
    const int per = (ks_total + splits - 1) / splits;
    return GemmPlan{splits, (per + 31) / 32, 32, 1, false};
}

static GemmPlan plan_gate_up(int d, int f, bool two) { return plan_gemm(d / 32, f / 16, 1, "SPMOE_PLAN_GATE_UP", two, MODE_GU); }
static GemmPlan plan_down(int d, int f, bool two) { return plan_gemm(f / 32, d / 32, 4, "SPMOE_PLAN_DOWN", two, MODE_DOWN); }

int spmoe_down_splits(int dtype, int d, int f, int T) {
    if (dtype != SPMOE_BF16) return 1;
    return plan_down(d, f, T > 16).splits;
}

static size_t gemm_lds_bytes(int waves, int ntok) {
    return (size_t)2 * waves * 2 * ntok * 256 * sizeof(float) +
           (GEMM_MAX_GROUPS + 1 + 2 * SPMOE_MAX_ETOT + SPMOE_MAX_EXPERTS + GROUP_MAX_A + GEMM_MAX_ASSIGN + 2 + SPMOE_MAX_ETOT) *
               sizeof(int) +
           SPMOE_MAX_ETOT * sizeof(void*);
}

void spmoe_describe_plan(int projection, int d, int f, int T, int32_t out[6]) {
    const GemmPlan p = projection == 0 ? plan_gate_up(d, f, T > 16) : plan_down(d, f, T > 16);
    out[0] = p.splits; out[1] = p.kw; out[2] = p.ksw; out[3] = p.nw; out[4] = (p.exact ? 1 : 0) | (p.ntok == 2 ? 2 : 0);
    out[5] = (int32_t)gemm_lds_bytes(p.waves(), p.ntok);
}

// Persistent grid size: as many workgroups as fit on the chip at once for this instance.
template <typename Kernel>
static int resident_blocks(Kernel kernel, int threads, size_t lds) {
    int dev = 0, cus = 0, per_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 256;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) cus = 256;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, threads, lds) != hipSuccess || per_cu <= 0) {
        (void)hipGetLastError();
        per_cu = 1;
    }
    return cus * per_cu;
}

template <int MODE, int NTOK>
static hipError_t launch_gemm_bf16(hipStream_t stream, const GemmPlan& plan, const SpmoeExpertList& list,
                                   const GemmParams& p) {
    const int threads = plan.waves() * 64;
    const size_t lds = gemm_lds_bytes(plan.waves(), NTOK);
    // cache of grid sizes per (instance, waves): [exact ksw index or generic][waves]
    static int grid_cache[16][17];
    // (two-tile instances exist only up to the k-step count their registers hold; the plans never ask for others)
#define SPMOE_GEMM_CASE(SLOT_, KSW_, EXACT_)                                                                          \
    if constexpr (NTOK == 1 || !(EXACT_) || KSW_ <= two_tile_max_ksw(MODE)) {                                         \
        int& g = grid_cache[SLOT_][plan.waves()];                                                                     \
        if (g == 0) g = resident_blocks(expert_gemm_kernel<MODE, KSW_, EXACT_, NTOK>, threads, lds);                  \
        hipLaunchKernelGGL((expert_gemm_kernel<MODE, KSW_, EXACT_, NTOK>), dim3(g), dim3(threads), lds, stream, list, p); \
    } else {                                                                                                          \
        return hipErrorInvalidValue;                                                                                  \
    }
    if (plan.exact) {
        switch (plan.ksw) {
            case 32: SPMOE_GEMM_CASE(0, 32, true) break;
            case 28: SPMOE_GEMM_CASE(1, 28, true) break;
            case 24: SPMOE_GEMM_CASE(2, 24, true) break;
            case 16: SPMOE_GEMM_CASE(3, 16, true) break;
            case 14: SPMOE_GEMM_CASE(4, 14, true) break;
            case 12: SPMOE_GEMM_CASE(5, 12, true) break;
            case 11: SPMOE_GEMM_CASE(6, 11, true) break;
            case 8: SPMOE_GEMM_CASE(7, 8, true) break;
            case 4: SPMOE_GEMM_CASE(8, 4, true) break;
            case 10: SPMOE_GEMM_CASE(10, 10, true) break;
            default: return hipErrorInvalidValue;
        }
    } else {
        SPMOE_GEMM_CASE(9, 32, false)
    }
#undef SPMOE_GEMM_CASE
    return hipGetLastError();
}

static GemmParams make_params(const SpmoeShape& s, const SpmoeRouting& r) {
    GemmParams p;
    p.idx = r.idx;
    p.xb = static_cast<const uint16_t*>(r.xb);
    p.x = nullptr;
    p.h = nullptr;
    p.ypart = nullptr;
    p.T = s.T; p.k = s.k; p.d = s.d; p.f = s.f;
    p.A_tot = s.T * s.k + s.n_shared * s.T;
    p.E = s.E;
    p.E_tot = s.E + s.n_shared;
    p.ks_total = 0; p.ks_split = 0; p.splits = 1; p.n_tiles = 0;
    p.waves = 4; p.kw = 4; p.nw = 1;
    p.steal = nullptr;
    // SPMOE_DYN_DIV (testing and tuning): 0 = static schedule only, v > 0 = last 1/v of the units dynamic where
    // the kernel's own rule allows it, v < 0 = last 1/|v| dynamic in every launch that has a counter
    p.dyn_div = 8;
    p.dyn_force = 0;
    if (const char* e = getenv("SPMOE_DYN_DIV")) {
        const int v = atoi(e);
        if (v >= -64 && v <= 64) { p.dyn_div = v < 0 ? -v : v; p.dyn_force = v < 0; }
    }
    return p;
}

hipError_t spmoe_launch_gate_up(hipStream_t stream, int dtype, const SpmoeShape& s, const SpmoeExpertList& list,
                                const SpmoeRouting& r, const float* x, void* h, int32_t* steal) {
    if (list.n <= 0) return hipSuccess;
    GemmParams p = make_params(s, r);
    p.steal = p.dyn_div > 0 ? steal : nullptr;   // SPMOE_DYN_DIV=0: static schedule only
    p.x = x;
    p.h = static_cast<uint16_t*>(h);
    if (dtype == SPMOE_BF16) {
        // more than 16 tokens: an expert may get up to 32, taken in one pass where the shape has a plan for it
        const GemmPlan plan = plan_gate_up(s.d, s.f, s.T > 16);
        const bool two = plan.ntok == 2;
        p.ks_total = s.d / 32;
        p.ks_split = (p.ks_total + plan.splits - 1) / plan.splits;
        p.splits = plan.splits;
        p.n_tiles = s.f / 16 / plan.nw;
        p.waves = plan.waves(); p.kw = plan.kw; p.nw = plan.nw;
        return two ? launch_gemm_bf16<MODE_GU, 2>(stream, plan, list, p) : launch_gemm_bf16<MODE_GU, 1>(stream, plan, list, p);
    }
    hipLaunchKernelGGL(expert_gemm_f32_kernel<MODE_GU>, dim3((s.f + 3) / 4, list.n), dim3(256), 0, stream, list, p,
                       static_cast<float*>(h));
    return hipGetLastError();
}

hipError_t spmoe_launch_down(hipStream_t stream, int dtype, const SpmoeShape& s, const SpmoeExpertList& list,
                             const SpmoeRouting& r, const void* h, float* ypart, int splits, int32_t* steal) {
    if (list.n <= 0) return hipSuccess;
    GemmParams p = make_params(s, r);
    p.steal = p.dyn_div > 0 ? steal : nullptr;   // SPMOE_DYN_DIV=0: static schedule only
    p.h = static_cast<uint16_t*>(const_cast<void*>(h));
    p.ypart = ypart;
    if (dtype == SPMOE_BF16) {
        const GemmPlan plan = plan_down(s.d, s.f, s.T > 16);
        const bool two = plan.ntok == 2;
        if (plan.splits != splits) return hipErrorInvalidValue;
        p.ks_total = s.f / 32;
        p.ks_split = (p.ks_total + plan.splits - 1) / plan.splits;
        p.splits = plan.splits;
        p.n_tiles = s.d / 32 / plan.nw;
        p.waves = plan.waves(); p.kw = plan.kw; p.nw = plan.nw;
        return two ? launch_gemm_bf16<MODE_DOWN, 2>(stream, plan, list, p) : launch_gemm_bf16<MODE_DOWN, 1>(stream, plan, list, p);
    }
    hipLaunchKernelGGL(expert_gemm_f32_kernel<MODE_DOWN>, dim3((s.d + 3) / 4, list.n), dim3(256), 0, stream, list, p,
                       static_cast<float*>(const_cast<void*>(h)));
    return hipGetLastError();
}

hipError_t spmoe_launch_combine(hipStream_t stream, const SpmoeShape& s, const SpmoeRouting& r, const float* ypart,
                                int splits, float* out) {
    hipLaunchKernelGGL(combine_kernel, dim3((s.d + 1023) / 1024, s.T), dim3(256), 0, stream, ypart, r.w, s.T, s.k,
                       s.n_shared, s.d, splits, out);
    return hipGetLastError();
}
