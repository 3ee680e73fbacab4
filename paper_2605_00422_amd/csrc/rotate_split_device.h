// Rotation of a token split over several workgroups (few tokens and a large n1: R1 too large for
// LDS, or a long stage 2), the launch that quantizes afterwards, and where the in-workgroup
// rotation leaves its results.
#pragma once
#include "rotate_bf16_device.h"
#include "gemm_decode_bs_device.h"
#include "psp_block_device.h"

namespace {

// ================================================================== few tokens, many tiles along n1
// One workgroup per token has to do all of stage 2 on one CU's four MFMA pipes, and, when R1 does
// not fit LDS, to stream all of its terms through that CU, chunk by chunk, with a memory round
// trip per chunk.  With only a few tokens most of the chip is idle meanwhile, so the rotation of
// a token is split over G = n1/16 workgroups, one per 16-row tile c of the result, and the
// product is taken in the other order, (R1^T V) R2, in which such a slice needs nothing that
// another slice computes:
//   A:  P[c, b] = sum_a R1[a, c] V[a, b]    for the 16 rows c of the slice  (the R1 slice: 16 rows)
//   B:  x~[c, d] = sum_b P[c, b] R2[b, d]   wavefront w: columns d of strip w
// The first contraction runs over a, and V is stored with b contiguous: a lane gathers the eight
// values of its operand from eight rows of the token in LDS (2-byte reads, in the order in which
// the packed R1 terms hold a).  Each wavefront computes the 16 x 16 tile of P for its own strip of
// b, splits it into three bf16 terms and leaves it in LDS for the others.  The token's maximum is not known
// inside the launch: the workgroups write the rotated values (fp32, in k order) and, per
// wavefront, their extremes to scratch, and a second, small launch quantizes.
struct RsShape {
    int G, E;                        // workgroups per token; (largest, smallest) pairs per token
    int spitch, ppitch;              // bytes of one row of the R1 slice, of P
    int vtbytes, slbytes;
    size_t lds_bytes;
    bool ok;
};
__host__ __device__ inline RsShape rs_shape(const R3Shape& s3) {
    RsShape r;
    r.G = s3.at;
    r.E = s3.at * s3.strips;
    r.spitch = s3.ch2 * 64 + 16;
    r.ppitch = s3.k1 * 64 + 16;
    r.vtbytes = s3.vbytes;
    r.slbytes = 3 * 16 * r.spitch;
    r.lds_bytes = (size_t)r.vtbytes + (size_t)r.slbytes + (size_t)3 * 16 * r.ppitch;
    r.ok = s3.at <= R3_MAXA && s3.k1 <= R3_MAXK1 && s3.strips <= R3_MAXW && r.lds_bytes <= RQ_LDS_LIMIT;
    return r;
}

__device__ __forceinline__ void rotate_slice_block(char* lds, const uint16_t* __restrict__ X, int64_t t, int j,
                                                   int64_t K, int n1, int n2, const uint16_t* __restrict__ R1p,
                                                   const uint16_t* __restrict__ R2p, float* __restrict__ xs,
                                                   float* __restrict__ pmax, int32_t* __restrict__ qsum) {
    const R3Shape sh = r3_shape(n1, n2);
    const RsShape rs = rs_shape(sh);
    const int tid = threadIdx.x, lane = tid & 63, li = lane & 15, lg = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);         // = strip
    // all wavefronts of the workgroup fetch; those beyond the strips end behind the first barrier
    const bool worker = wave < sh.strips;
    const int nthreads = (int)blockDim.x;
    const int n1p16 = sh.at * 16, n1p32 = sh.ch2 * 32, n2p32 = sh.k1 * 32;
    char* vt = lds;                                                    // token rows V[a][b]
    char* sl = lds + rs.vtbytes;                                       // R1 slice [term][c in slice][a]
    char* pl = sl + rs.slbytes;                                        // P terms [term][c in slice][b]

    // R2 terms of my strip (operand B of the second product)
    v4i bfr[R3_MAXK1][3];
#pragma unroll
    for (int kb = 0; kb < R3_MAXK1; ++kb)
#pragma unroll
        for (int p = 0; p < 3; ++p) {
            bfr[kb][p] = v4i{0, 0, 0, 0};
            if (kb < sh.k1 && worker)
                bfr[kb][p] = *reinterpret_cast<const v4i*>(R2p + ((int64_t)(p * sh.strips * 16 + wave * 16 + li)) * n2p32 +
                                                           kb * 32 + 8 * lg);
        }
    // the slice of the R1 terms: rows 16 j .. 16 j + 15 of each term, at most three pieces a thread
    // (3 * 16 * 32 pieces at most, 512 threads at least)
    const int row_items = sh.ch2 * 4, slice_items = 3 * 16 * row_items;
    const FastDiv dri(row_items);
    v4i rp[3];
#pragma unroll
    for (int e = 0; e < 3; ++e) {
        const int g = tid + e * nthreads;
        const int gc = g < slice_items ? g : slice_items - 1;
        const int row = dri.div(gc), piece = gc - row * row_items;     // row = term * 16 + c in slice
        rp[e] = *reinterpret_cast<const v4i*>(R1p + ((int64_t)((row >> 4) * n1p16 + j * 16 + (row & 15))) * n1p32 +
                                              piece * 8);
    }
    // token rows into LDS (bf16 as stored; zero padding), eight loads in flight per thread
    {
        const int per_row = n2p32 >> 3, items = n1p16 * per_row;
        const uint16_t* xrow = X + t * K;
        const FastDiv dpr(per_row);
        if ((n2 & 7) == 0) {
            for (int base = 0; base < items; base += 8 * nthreads) {
                v4i tmp[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int it = base + e * nthreads + tid;
                    const int a = dpr.div(it), b0 = (it - a * per_row) << 3;
                    const bool in = it < items && a < n1 && b0 < n2;
                    const v4i v = *reinterpret_cast<const v4i*>(xrow + (in ? (int64_t)a * n2 + b0 : 0));
                    tmp[e] = in ? v : v4i{0, 0, 0, 0};
                }
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int it = base + e * nthreads + tid;
                    if (it < items) {
                        const int a = dpr.div(it), b0 = (it - a * per_row) << 3;
                        *reinterpret_cast<v4i*>(vt + a * sh.vpitch + b0 * 2) = tmp[e];
                    }
                }
            }
        } else if ((n2 & 1) == 0) {
            // rows start on 4-byte boundaries only: four 4-byte loads per item, eight items in flight
            const uint32_t* x32 = reinterpret_cast<const uint32_t*>(xrow);
            for (int base = 0; base < items; base += 8 * nthreads) {
                uint32_t tmp[8][4];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int it = base + e * nthreads + tid;
                    const int a = dpr.div(it), b0 = (it - a * per_row) << 3;
#pragma unroll
                    for (int p = 0; p < 4; ++p) {
                        const bool in = it < items && a < n1 && b0 + 2 * p < n2;
                        const uint32_t v = x32[in ? ((a * n2 + b0) >> 1) + p : 0];
                        tmp[e][p] = in ? v : 0u;
                    }
                }
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int it = base + e * nthreads + tid;
                    if (it < items) {
                        const int a = dpr.div(it), b0 = (it - a * per_row) << 3;
                        *reinterpret_cast<v4i*>(vt + a * sh.vpitch + b0 * 2) =
                            v4i{(int)tmp[e][0], (int)tmp[e][1], (int)tmp[e][2], (int)tmp[e][3]};
                    }
                }
            }
        } else {
            for (int it = tid; it < items; it += nthreads) {
                const int a = dpr.div(it), b0 = (it - a * per_row) << 3;
                uint32_t w[4] = {0u, 0u, 0u, 0u};
                if (a < n1) {
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        if (b0 + e < n2) w[e >> 1] |= (uint32_t)xrow[(int64_t)a * n2 + b0 + e] << (16 * (e & 1));
                }
                *reinterpret_cast<v4i*>(vt + a * sh.vpitch + b0 * 2) = v4i{(int)w[0], (int)w[1], (int)w[2], (int)w[3]};
            }
        }
    }
    // the slice into LDS; columns of P past the last strip (a 32-deep step half filled) are zeros
#pragma unroll
    for (int e = 0; e < 3; ++e) {
        const int g = tid + e * nthreads;
        if (g < slice_items) {
            const int row = dri.div(g), piece = g - row * row_items;
            *reinterpret_cast<v4i*>(sl + row * rs.spitch + piece * 16) = rp[e];
        }
    }
    if ((sh.strips & 1) != 0)
        for (int i = tid; i < 3 * 16 * 2; i += nthreads)
            *reinterpret_cast<v4i*>(pl + (i >> 1) * rs.ppitch + sh.strips * 32 + (i & 1) * 16) = v4i{0, 0, 0, 0};
    bwla_lds_barrier();
    if (!worker) return;

    // ---- A: tile of P for my strip of b: rows of the tile are b = 16 w + 4 lg + v, columns c = li
    {
        v4f pa = v4f{0.f, 0.f, 0.f, 0.f};
        // lane (li, lg): b = 16 w + li; position e of step ch is row a = 32 ch + 4 lg + e (e < 4),
        // 32 ch + 16 + 4 lg + e - 4 (e >= 4); rows past the padded n1 (their R1 terms are zero)
        // read the last row instead
        const char* ap = vt + (wave * 16 + li) * 2;
        const char* bp = sl + li * rs.spitch + lg * 16;
#pragma unroll
        for (int ch = 0; ch < R3_MAXA / 2; ++ch) {
            if (ch < sh.ch2) {
                uint32_t w[4];
#pragma unroll
                for (int e = 0; e < 8; e += 2) {
                    int a = 32 * ch + 4 * lg + (e < 4 ? e : 12 + e);
                    const int a0 = a < n1p16 ? a : n1p16 - 1, a1 = a + 1 < n1p16 ? a + 1 : n1p16 - 1;
                    const uint32_t lo = *reinterpret_cast<const uint16_t*>(ap + a0 * sh.vpitch);
                    const uint32_t hi = *reinterpret_cast<const uint16_t*>(ap + a1 * sh.vpitch);
                    w[e >> 1] = lo | (hi << 16);
                }
                const v8bf va = __builtin_bit_cast(v8bf, v4i{(int)w[0], (int)w[1], (int)w[2], (int)w[3]});
#pragma unroll
                for (int p = 2; p >= 0; --p) {
                    const v8bf vb = __builtin_bit_cast(v8bf, *reinterpret_cast<const v4i*>(bp + p * 16 * rs.spitch + ch * 64));
                    pa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, vb, pa, 0, 0, 0);
                }
            }
        }
        // three bf16 terms of the four values, to P[term][c = li][b = 16 w + 4 lg ..]
        uint32_t w1[2], w2[2], w3[2];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const __bf16 h1 = (__bf16)pa[v];
            const float r1 = pa[v] - (float)h1;
            const __bf16 h2 = (__bf16)r1;
            const __bf16 h3 = (__bf16)(r1 - (float)h2);
            const uint32_t sft = 16 * (v & 1);
            if ((v & 1) == 0) { w1[v >> 1] = 0u; w2[v >> 1] = 0u; w3[v >> 1] = 0u; }
            w1[v >> 1] |= (uint32_t)__builtin_bit_cast(uint16_t, h1) << sft;
            w2[v >> 1] |= (uint32_t)__builtin_bit_cast(uint16_t, h2) << sft;
            w3[v >> 1] |= (uint32_t)__builtin_bit_cast(uint16_t, h3) << sft;
        }
        char* pd = pl + li * rs.ppitch + (wave * 16 + 4 * lg) * 2;
        *reinterpret_cast<uint2*>(pd) = uint2{w1[0], w1[1]};
        *reinterpret_cast<uint2*>(pd + 16 * rs.ppitch) = uint2{w2[0], w2[1]};
        *reinterpret_cast<uint2*>(pd + 32 * rs.ppitch) = uint2{w3[0], w3[1]};
    }
    bwla_lds_barrier();

    // ---- B: my strip of the result: rows c = 16 j + 4 lg + v, column d = 16 w + li
    v4f y = v4f{0.f, 0.f, 0.f, 0.f};
    {
        const char* ap = pl + li * rs.ppitch + lg * 16;
#pragma unroll
        for (int kb = 0; kb < R3_MAXK1; ++kb) {
            if (kb < sh.k1) {
                const v8bf a1 = __builtin_bit_cast(v8bf, *reinterpret_cast<const v4i*>(ap + kb * 64));
                const v8bf a2 = __builtin_bit_cast(v8bf, *reinterpret_cast<const v4i*>(ap + 16 * rs.ppitch + kb * 64));
                const v8bf a3 = __builtin_bit_cast(v8bf, *reinterpret_cast<const v4i*>(ap + 32 * rs.ppitch + kb * 64));
                const v8bf b0 = __builtin_bit_cast(v8bf, bfr[kb][0]);
                const v8bf b1 = __builtin_bit_cast(v8bf, bfr[kb][1]);
                const v8bf b2 = __builtin_bit_cast(v8bf, bfr[kb][2]);
                y = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a3, b0, y, 0, 0, 0);
                y = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, b2, y, 0, 0, 0);
                y = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a2, b1, y, 0, 0, 0);
                y = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a2, b0, y, 0, 0, 0);
                y = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, b1, y, 0, 0, 0);
                y = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, b0, y, 0, 0, 0);
            }
        }
    }

    // ---- rotated values out, and the extremes of my tile (0 included)
    float mx = 0.0f, mn = 0.0f;
    const int d = wave * 16 + li;
    float* xt = xs + t * K;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        const int c = j * 16 + 4 * lg + v;
        if (c < n1 && d < n2) {
            xt[(int64_t)c * n2 + d] = y[v];
            mx = fmaxf(mx, y[v]);
            mn = fminf(mn, y[v]);
        }
    }
    mx = bwla_wave_max(mx);
    mn = -bwla_wave_max(-mn);
    if (lane == 0) {
        float* pm = pmax + ((t * rs.G + j) * sh.strips + wave) * 2;
        pm[0] = mx;
        pm[1] = mn;
        if (j == 0 && wave == 0) qsum[t] = 0;          // the quantizing launch adds its sums up here
    }
}

// second launch of the split rotation: RS_QB workgroups per token quantize the rotated values, each
// its share of k, every load in flight at once; the code sum is added up in qsum[t], which the
// first launch has set to zero (integer adds: the order does not matter).  Workgroups from
// `first` on (one per tile of 16 tokens, none if S == 1) add up the projection's partial tiles.
struct PspSum {
    const float* partials;
    float* T;
    int64_t M, first;
    int r, S;
};
constexpr int RS_QB = 8;
constexpr int RS_QI = 4;             // float4 per thread: K <= RS_QB * 512 * RS_QI * 4
__global__ __launch_bounds__(512) void quantize_rows_kernel(const float* __restrict__ xs, const float* __restrict__ pmax,
                                                            int E, int64_t K, int8_t* __restrict__ q,
                                                            float* __restrict__ scale, int32_t* __restrict__ qsum,
                                                            float qmax, int asym, float* __restrict__ tmode, int tp,
                                                            float* __restrict__ zcs, PspSum ps) {
    __shared__ int redi[8];
    __shared__ float redf[16];
    if ((int64_t)blockIdx.x >= ps.first) {              // behind the quantizing workgroups: T from its partial tiles
        psp_sum_partials(ps.partials, ps.T, ps.M, ps.r, ps.S, (int)(blockIdx.x - ps.first), tp);
        return;
    }
    const int64_t t = blockIdx.x / RS_QB;
    const int part = (int)(blockIdx.x - t * RS_QB);
    const int tid = threadIdx.x;
    const int n4 = (int)(K >> 2);
    const float4* src = reinterpret_cast<const float4*>(xs + t * K);
    float4 x[RS_QI];
#pragma unroll
    for (int e = 0; e < RS_QI; ++e) {
        const int i = (e * RS_QB + part) * 512 + tid;
        x[e] = src[i < n4 ? i : n4 - 1];
    }
    // the token's extremes: one (largest, smallest) pair per thread, then over the workgroup
    float hi = 0.0f, lo = 0.0f;
    if (tid < E) {
        const float2 pr = *reinterpret_cast<const float2*>(pmax + (t * E + tid) * 2);
        hi = pr.x; lo = pr.y;
    }
    hi = bwla_wave_max(hi);
    lo = -bwla_wave_max(-lo);
    if ((tid & 63) == 0) { redf[tid >> 6] = hi; redf[8 + (tid >> 6)] = lo; }
    __syncthreads();
    hi = redf[0]; lo = redf[8];
#pragma unroll
    for (int w = 1; w < 8; ++w) { hi = fmaxf(hi, redf[w]); lo = fminf(lo, redf[8 + w]); }
    const QuantPlan qp = quant_plan(hi, lo, qmax, asym != 0);
    int* dst = reinterpret_cast<int*>(q + t * K);
    int lsum = 0;
#pragma unroll
    for (int e = 0; e < RS_QI; ++e) {
        const int i = (e * RS_QB + part) * 512 + tid;
        if (i < n4) {
            const float f[4] = {x[e].x, x[e].y, x[e].z, x[e].w};
            int code[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                code[v] = quant_code(f[v], qp);
                lsum += code[v];
            }
            dst[i] = (code[0] & 0xff) | ((code[1] & 0xff) << 8) | ((code[2] & 0xff) << 16) | (code[3] << 24);
        }
    }
    lsum = bwla_wave_sum_i32(lsum);
    if ((tid & 63) == 0) redi[tid >> 6] = lsum;
    __syncthreads();
    if (tid == 0) {
        int tot = 0;
        for (int w = 0; w < 8; ++w) tot += redi[w];
        atomicAdd(qsum + t, tot);
        if (part == 0) {
            const float sc = quant_scale(hi, lo, qmax, asym != 0);
            scale[t] = sc;
            zcs[t] = qp.zc;
            if (asym && tmode) tmode[t * tp] = tmode[t * tp + 1] = -(sc * qp.zc);
        }
    }
}

// layers with row shifts, after the split rotation (the code sum is complete only now):
// T[t, last] = scale_t * sum_k (q - z) = scale_t * (qsum_t - K zc_t)
__global__ void shift_column_kernel(const float* __restrict__ scale, const int32_t* __restrict__ qsum,
                                    const float* __restrict__ zcs, int64_t M, int64_t K,
                                    float* __restrict__ tshift, int tp) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < M) tshift[t * tp] = scale[t] * ((float)qsum[t] - (float)K * zcs[t]);
}

}  // namespace
