/* Seeded synthetic-input generator shared by the CPU oracle tests, the GPU parity tests and
 * the benchmark.  It holds none of the MoE method's arithmetic: it only fills buffers with
 * reproducible pseudo-random normal values (fp32, or bf16 bit patterns rounded to nearest-even).
 *
 * Design: counter based.  Element i of the tensor named by (seed, stream) depends only on
 * (seed, stream, i), so any slice can be produced without materialising the rest, by any number
 * of threads, with the same bits.  Pair p = i/2 yields two normals through the Box-Muller
 * transform of two uniforms obtained from a 64-bit integer mixing function.  ln, sin and cos are
 * evaluated by the polynomial routines below, which use only IEEE-754 +,-,*,/ in double (built
 * with -ffp-contract=off), so the bit patterns do not depend on the host's libm or CPU model.
 */
#include <stdint.h>
#include <stddef.h>
#include <string.h>
#include <math.h>   /* sqrt only: correctly rounded by IEEE-754 */

static inline uint64_t mix64(uint64_t z) {
    z += 0x9E3779B97F4A7C15ULL;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

/* ln(u) for u in (0,1]: u = m * 2^e with m in [sqrt(1/2), sqrt(2)); ln m = 2 atanh((m-1)/(m+1)). */
static double det_log(double u) {
    uint64_t bits;
    memcpy(&bits, &u, 8);
    int e = (int)((bits >> 52) & 0x7FF) - 1023;
    bits = (bits & 0x000FFFFFFFFFFFFFULL) | 0x3FF0000000000000ULL;
    double m;
    memcpy(&m, &bits, 8);                 /* m in [1,2) */
    if (m > 1.4142135623730951) { m = m * 0.5; e += 1; }
    double s = (m - 1.0) / (m + 1.0);     /* |s| <= 0.1716 */
    double s2 = s * s;
    double poly = 1.0 / 15.0;
    poly = poly * s2 + 1.0 / 13.0;
    poly = poly * s2 + 1.0 / 11.0;
    poly = poly * s2 + 1.0 / 9.0;
    poly = poly * s2 + 1.0 / 7.0;
    poly = poly * s2 + 1.0 / 5.0;
    poly = poly * s2 + 1.0 / 3.0;
    poly = poly * s2 + 1.0;
    return (double)e * 0.6931471805599453 + 2.0 * s * poly;
}

/* sin and cos of 2*pi*v for v in [0,1): reduce to an octant, Taylor series on [0, pi/4]. */
static void det_sincos2pi(double v, double* sn, double* cs) {
    double t = v * 8.0;
    int oct = (int)t;                     /* 0..7 */
    double fr = t - (double)oct;          /* [0,1) */
    if (oct & 1) fr = 1.0 - fr;           /* odd octants are mirrored */
    double a = fr * 0.7853981633974483;   /* [0, pi/4] */
    double a2 = a * a;
    double sp = -1.0 / 6227020800.0;      /* -1/13! */
    sp = sp * a2 + 1.0 / 39916800.0;
    sp = sp * a2 - 1.0 / 362880.0;
    sp = sp * a2 + 1.0 / 5040.0;
    sp = sp * a2 - 1.0 / 120.0;
    sp = sp * a2 + 1.0 / 6.0;
    double s = a - a * a2 * sp;
    double cp = 1.0 / 479001600.0;        /* 1/12! */
    cp = cp * a2 - 1.0 / 3628800.0;
    cp = cp * a2 + 1.0 / 40320.0;
    cp = cp * a2 - 1.0 / 720.0;
    cp = cp * a2 + 1.0 / 24.0;
    cp = cp * a2 - 0.5;
    double c = 1.0 + a2 * cp;
    double S, C;
    switch (oct) {
        case 0: S = s;  C = c;  break;
        case 1: S = c;  C = s;  break;
        case 2: S = c;  C = -s; break;
        case 3: S = s;  C = -c; break;
        case 4: S = -s; C = -c; break;
        case 5: S = -c; C = -s; break;
        case 6: S = -c; C = s;  break;
        default: S = -s; C = c; break;
    }
    *sn = S; *cs = C;
}

static inline void normal_pair(uint64_t key, uint64_t pair, double* z0, double* z1) {
    uint64_t h1 = mix64(key ^ (pair * 2ULL));
    uint64_t h2 = mix64(key ^ (pair * 2ULL + 1ULL));
    double u1 = (double)((h1 >> 11) + 1ULL) * (1.0 / 9007199254740992.0);   /* (0,1] */
    double u2 = (double)(h2 >> 11) * (1.0 / 9007199254740992.0);            /* [0,1) */
    double r = sqrt(-2.0 * det_log(u1));
    double s, c;
    det_sincos2pi(u2, &s, &c);
    *z0 = r * c;
    *z1 = r * s;
}

static inline uint64_t tensor_key(uint64_t seed, uint64_t stream) {
    return mix64(mix64(seed) ^ (stream * 0xD6E8FEB86659FD93ULL + 0x2545F4914F6CDD1DULL));
}

/* fp32 -> bf16 bit pattern, round to nearest even (inputs here are finite). */
static inline uint16_t f32_to_bf16_rne(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    uint32_t rounding = 0x7FFFU + ((u >> 16) & 1U);
    return (uint16_t)((u + rounding) >> 16);
}

/* out[j] = mean + std * z_{offset+j}, j in [0,n): elements offset..offset+n-1 of tensor (seed, stream). */
void spmoe_gen_normal_f32(uint64_t seed, uint64_t stream, uint64_t offset, uint64_t n,
                          float mean, float std, float* out) {
    const uint64_t key = tensor_key(seed, stream);
    const uint64_t first_pair = offset / 2, last_pair = (offset + n + 1) / 2;   /* [first,last) */
    #pragma omp parallel for schedule(static)
    for (uint64_t p = first_pair; p < last_pair; ++p) {
        double z0, z1;
        normal_pair(key, p, &z0, &z1);
        uint64_t i0 = 2 * p, i1 = 2 * p + 1;
        if (i0 >= offset && i0 < offset + n) out[i0 - offset] = (float)((double)mean + (double)std * z0);
        if (i1 >= offset && i1 < offset + n) out[i1 - offset] = (float)((double)mean + (double)std * z1);
    }
}

/* Same values as spmoe_gen_normal_f32 with mean 0, each rounded (nearest-even) to a bf16 bit pattern. */
void spmoe_gen_normal_bf16(uint64_t seed, uint64_t stream, uint64_t offset, uint64_t n,
                           float std, uint16_t* out) {
    const uint64_t key = tensor_key(seed, stream);
    const uint64_t first_pair = offset / 2, last_pair = (offset + n + 1) / 2;
    #pragma omp parallel for schedule(static)
    for (uint64_t p = first_pair; p < last_pair; ++p) {
        double z0, z1;
        normal_pair(key, p, &z0, &z1);
        uint64_t i0 = 2 * p, i1 = 2 * p + 1;
        if (i0 >= offset && i0 < offset + n) out[i0 - offset] = f32_to_bf16_rne((float)((double)std * z0));
        if (i1 >= offset && i1 < offset + n) out[i1 - offset] = f32_to_bf16_rne((float)((double)std * z1));
    }
}

/* Round an fp32 buffer to bf16 bit patterns (nearest-even); used to build bf16 tensors from fp32 ones. */
void spmoe_gen_round_bf16(const float* in, uint64_t n, uint16_t* out) {
    #pragma omp parallel for schedule(static)
    for (uint64_t i = 0; i < n; ++i) out[i] = f32_to_bf16_rne(in[i]);
}
