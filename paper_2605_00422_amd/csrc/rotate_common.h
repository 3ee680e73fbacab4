// Shared by the rotation kernels: the per-token quantizer plan
// (symmetric or min-max affine codes), launch constants, LDS shapes of the fp32 path, fast division.
#pragma once
#include "bwla_internal.h"

namespace {


// How a token is quantized, from its largest and smallest rotated value (hi >= 0 >= lo: the
// reductions start at zero, which also covers the zero padding).
//   symmetric:   codes rint(x * qmax / amax) in [-qmax, qmax], scale = amax / qmax
//   asymmetric:  L = 2 qmax + 1 steps over [lo, hi], scale = (hi - lo) / L, zero point
//                z = rint(-lo / scale); the code q = rint(x / scale) + z in [0, L] is stored as
//                q - (qmax + 1), so zc = z - (qmax + 1) is what the stored code has to lose
struct QuantPlan {
    float inv, zc, cmin, cmax;
};
__device__ __forceinline__ QuantPlan quant_plan(float hi, float lo, float qmax, bool asym) {
    QuantPlan p;
    if (asym) {
        const float L = 2.0f * qmax + 1.0f, span = hi - lo;
        p.inv = span > 0.0f ? L / span : 0.0f;
        p.zc = rintf(-lo * p.inv) - (qmax + 1.0f);
        if (!(span > 0.0f)) p.zc = -(qmax + 1.0f);      // all-zero token: q = z = 0
        p.cmin = -(qmax + 1.0f);
        p.cmax = qmax;
    } else {
        const float amax = fmaxf(hi, -lo);
        p.inv = amax > 0.0f ? qmax / amax : 0.0f;
        p.zc = 0.0f;
        p.cmin = -qmax;
        p.cmax = qmax;
    }
    return p;
}
// the token's step (only the thread that writes it out needs it)
__device__ __forceinline__ float quant_scale(float hi, float lo, float qmax, bool asym) {
    return asym ? (hi - lo) / (2.0f * qmax + 1.0f) : fmaxf(hi, -lo) / qmax;
}
__device__ __forceinline__ int quant_code(float x, const QuantPlan& p) {
    return (int)fminf(fmaxf(rintf(x * p.inv) + p.zc, p.cmin), p.cmax);
}
// The entries of T that the layer's mode adds for token t (tmode points at the first of them in
// row 0, or is NULL): asymmetric codes: -scale * zc, twice; row shift: scale * sum_k (q - z).
__device__ __forceinline__ void quant_extras(float* tmode, int tp, int64_t t, bool asym, bool shift,
                                             const QuantPlan& p, float scale, int tot, int64_t K) {
    if (!tmode) return;
    float* row = tmode + t * tp;
    int c = 0;
    if (asym) { row[0] = row[1] = -(scale * p.zc); c = 2; }
    if (shift) row[c] = scale * ((float)tot - (float)K * p.zc);
}

constexpr int RQ_THREADS = 512;
constexpr int RQ_WAVES = RQ_THREADS / 64;
constexpr int RQ_MAXT = 16;          // 16x16 output tiles per wavefront
constexpr int RQ_CK = 16;            // contraction indices per streamed factor chunk
constexpr int RQ_CLD = RQ_CK + 4;    // LDS pitch of a streamed chunk row
constexpr int RQ_RING = 3;           // streamed chunks in flight (registers)
constexpr int PP_SLICE = 512;        // columns of K per projection workgroup
constexpr int PP_MAXJT = BWLA_MAX_RANK / 16;
constexpr int PP_GROUPJT = 2;        // 16-column tiles of the rank per projection workgroup when they are dealt out
constexpr size_t RQ_LDS_LIMIT = 160 * 1024 - 256;   // leaves room for the few static bytes

__host__ __device__ inline int rq_pad16(int n) { return (n + 15) & ~15; }

// LDS layout of a rotation workgroup (floats).  Every matrix is stored so that the MFMA
// contraction index runs along a row with a pitch of (multiple of 16) + 4: a lane then fetches
// four consecutive contraction values of its operand row with one 128-bit read, and the 16 rows
// of a lane group fall into disjoint banks.
//   region  V  [a][b]  pitch ldv   (token, stage-1 A)   later  ZT [d][a]  pitch ldzt (stage-2 A)
//   R2T [d][b] pitch ld2t (stage-1 B),  R1T [c][a] pitch ld1t (stage-2 B)      -- resident mode
//   two chunk buffers [row][16] pitch RQ_CLD                                   -- streaming mode
struct RqShape {
    int n1, n2, n1p, n2p, ldv, ldzt, ld2t, ld1t, region, nmaxp;
    bool resident;
    size_t lds_bytes;
};

__host__ __device__ inline RqShape rq_shape(int n1, int n2) {
    RqShape s;
    s.n1 = n1; s.n2 = n2;
    s.n1p = rq_pad16(n1); s.n2p = rq_pad16(n2);
    s.ldv = s.n2p + 4; s.ldzt = s.n1p + 4; s.ld2t = s.n2p + 4; s.ld1t = s.n1p + 4;
    const int rv = s.n1p * s.ldv, rz = s.n2p * s.ldzt;
    s.region = rv > rz ? rv : rz;
    s.nmaxp = s.n1p > s.n2p ? s.n1p : s.n2p;
    const size_t res = ((size_t)s.region + (size_t)s.n2p * s.ld2t + (size_t)s.n1p * s.ld1t + 64) * sizeof(float);
    const size_t str = ((size_t)s.region + (size_t)2 * s.nmaxp * RQ_CLD + 64) * sizeof(float);
    s.resident = res <= RQ_LDS_LIMIT;
    s.lds_bytes = s.resident ? res : str;
    return s;
}

__host__ __device__ inline size_t pp_lds_bytes(int r, int waves = RQ_WAVES) {
    const int rp = ((r + 15) >> 4) * 16;
    return (size_t)waves * (rp / 16) * 64 * 16 + 16;                   // cross-wave reduction
}

// Exact n / d for n * d < 2^32 with one multiply-high; index arithmetic on run-time factor
// sizes would otherwise cost a ~30-instruction division sequence per use.
struct FastDiv {
    uint32_t d, m;
    __device__ explicit FastDiv(uint32_t dd) : d(dd), m(dd > 1 ? 0xFFFFFFFFu / dd + 1u : 0u) {}
    __device__ __forceinline__ int div(int n) const { return d > 1 ? (int)__umulhi((uint32_t)n, m) : n; }
};

}  // namespace
