// Rotation of a token split over several workgroups (few tokens and a large n1: R1 too large for
// LDS, or a long stage 2), the launch that quantizes afterwards, and where the in-workgroup
// rotation leaves its results.
#pragma once
#include "rotate_bf16_device.h"
#include "gemm_decode_bs_device.h"

namespace {

// ================================================================== few tokens, many tiles along n1
// One workgroup per token has to do all of stage 2 on one CU's four MFMA pipes, and, when R1 does
// not fit LDS, to stream all of its terms through that CU, chunk by chunk, with a memory round
// trip per chunk.  With only a few tokens most of the chip is idle meanwhile, so
// the rotation of a token is split over G workgroups: each does stage 1 for the whole token (it
// is cheap) and stage 2 for RS_CT tiles along n1, for which its slice of the R1 terms fits LDS
// whole and is requested at once.  The token's maximum is then not known inside the launch:
// the workgroups write the rotated values (fp32, in k order) and their own maxima to scratch,
// and a second, small launch quantizes.  Same products in the same order as rotate3_token, so
// the codes are the same.
constexpr int RS_CT = 2;             // 16-row tiles along n1 per workgroup (stage 2)
constexpr int RS_FILL = 6;           // 16-byte pieces of the R1 slice a thread keeps in flight

struct RsShape {
    int G, spitch;                   // workgroups per token; bytes of one R1 row in LDS
    size_t lds_bytes;
    bool ok;
};
__host__ __device__ inline RsShape rs_shape(const R3Shape& s3) {
    RsShape r;
    r.G = (s3.at + RS_CT - 1) / RS_CT;
    r.spitch = s3.ch2 * 64 + 16;
    r.lds_bytes = (size_t)s3.vbytes + (size_t)3 * RS_CT * 16 * r.spitch + 256;
    // one wavefront per strip in a 512-thread workgroup; the slice in RS_FILL pieces per thread
    r.ok = s3.at <= R3_MAXA && s3.k1 <= R3_MAXK1 && s3.strips <= 8 && r.lds_bytes <= RQ_LDS_LIMIT &&
           3 * RS_CT * 16 * s3.ch2 * 4 <= RS_FILL * 64 * s3.strips;
    return r;
}

template <int ATM>
__device__ __forceinline__ void rotate_split_block(char* lds, const uint16_t* __restrict__ X, int64_t t, int j,
                                                   int64_t K, int n1, int n2, const uint16_t* __restrict__ R1p,
                                                   const uint16_t* __restrict__ R2p, float* __restrict__ xs,
                                                   float* __restrict__ pmax, int32_t* __restrict__ qsum) {
    const R3Shape sh = r3_shape(n1, n2);
    const RsShape rs = rs_shape(sh);
    const int tid = threadIdx.x, lane = tid & 63, li = lane & 15, lg = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);         // = strip
    if (wave >= sh.strips) return;
    const int nthreads = 64 * sh.strips;
    const int n1p16 = sh.at * 16, n1p32 = sh.ch2 * 32, n2p32 = sh.k1 * 32;
    char* vt = lds;                                                    // token rows
    char* sl = lds + sh.vbytes;                                        // R1 slice [term][c in slice][a]
    float* red = reinterpret_cast<float*>(sl + 3 * RS_CT * 16 * rs.spitch);
    const int c_base = j * RS_CT * 16;                                 // first row c of the slice

    // R2 terms of my strip
    v4i bfr[R3_MAXK1][3];
#pragma unroll
    for (int kb = 0; kb < R3_MAXK1; ++kb)
#pragma unroll
        for (int p = 0; p < 3; ++p) {
            bfr[kb][p] = v4i{0, 0, 0, 0};
            if (kb < sh.k1)
                bfr[kb][p] = *reinterpret_cast<const v4i*>(R2p + ((int64_t)(p * sh.strips * 16 + wave * 16 + li)) * n2p32 +
                                                           kb * 32 + 8 * lg);
        }
    // the slice of the R1 terms: rows c_base .. c_base + 31 of each term (rows past the padded n1
    // repeat the last one and are never used), all requested now and stored after stage 1
    const int row_items = sh.ch2 * 4, slice_items = 3 * RS_CT * 16 * row_items;
    const FastDiv dri(row_items);
    v4i rp[RS_FILL];
    auto slice_issue = [&]() {
#pragma unroll
        for (int e = 0; e < RS_FILL; ++e) {
            const int g = tid + e * nthreads;
            const int gc = g < slice_items ? g : slice_items - 1;
            const int row = dri.div(gc), piece = gc - row * row_items;  // row = term * 32 + c in slice
            const int term = row / (RS_CT * 16), cs = row - term * (RS_CT * 16);
            const int c = c_base + cs < n1p16 ? c_base + cs : n1p16 - 1;
            rp[e] = *reinterpret_cast<const v4i*>(R1p + ((int64_t)(term * n1p16 + c)) * n1p32 + piece * 8);
        }
    };
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
                if (base == 0) slice_issue();          // behind the first token loads
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
                if (base == 0) slice_issue();          // behind the first token loads
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
            slice_issue();
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
    bwla_lds_barrier();

    // ---- stage 1 (as in rotate3_token): Z[a, d] for the whole token, my strip of d
    v4f z[ATM];
#pragma unroll
    for (int ta = 0; ta < ATM; ++ta) z[ta] = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int g = 0; g < ATM / 2; ++g) {
        if (2 * g < sh.at) {
            const int t0 = 2 * g, t1 = 2 * g + 1 < sh.at ? 2 * g + 1 : 2 * g;
            const char* a0p = vt + (t0 * 16 + li) * sh.vpitch + lg * 16;
            const char* a1p = vt + (t1 * 16 + li) * sh.vpitch + lg * 16;
#pragma unroll
            for (int kb = 0; kb < R3_MAXK1; ++kb) {
                if (kb < sh.k1) {
                    const v8bf a0 = __builtin_bit_cast(v8bf, *reinterpret_cast<const v4i*>(a0p + kb * 64));
                    const v8bf a1 = __builtin_bit_cast(v8bf, *reinterpret_cast<const v4i*>(a1p + kb * 64));
#pragma unroll
                    for (int p = 2; p >= 0; --p) {
                        const v8bf b = __builtin_bit_cast(v8bf, bfr[kb][p]);
                        z[2 * g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, b, z[2 * g], 0, 0, 0);
                        z[2 * g + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, b, z[2 * g + 1], 0, 0, 0);
                    }
                }
            }
        }
    }
    if ((sh.at & 1) != 0) {
#pragma unroll
        for (int ta = 1; ta < ATM; ta += 2)
            if (ta == sh.at) z[ta] = v4f{0.f, 0.f, 0.f, 0.f};
    }

    // ---- the slice into LDS
#pragma unroll
    for (int e = 0; e < RS_FILL; ++e) {
        const int g = tid + e * nthreads;
        if (g < slice_items) {
            const int row = dri.div(g), piece = g - row * row_items;
            *reinterpret_cast<v4i*>(sl + row * rs.spitch + piece * 16) = rp[e];
        }
    }
    bwla_lds_barrier();

    // ---- stage 2 for tiles c0 = RS_CT * j, c0 + 1 (products and their order as in rotate3_token)
    v4f y0 = v4f{0.f, 0.f, 0.f, 0.f}, y1 = v4f{0.f, 0.f, 0.f, 0.f};
    const bool two = RS_CT * j + 1 < sh.at;            // an odd last tile is done twice; the copy is dropped
    const char* s0 = sl + li * rs.spitch + lg * 16;
    const char* s1 = sl + ((two ? 16 : 0) + li) * rs.spitch + lg * 16;
#pragma unroll
    for (int ch = 0; ch < ATM / 2; ++ch) {
        if (ch < sh.ch2) {
            const float f[8] = {z[2 * ch][0], z[2 * ch][1], z[2 * ch][2], z[2 * ch][3],
                                z[2 * ch + 1][0], z[2 * ch + 1][1], z[2 * ch + 1][2], z[2 * ch + 1][3]};
            v8bf a1, a2, a3;
            r3_split3(f, a1, a2, a3);
            v8bf b0[3], b1[3];
#pragma unroll
            for (int p = 0; p < 3; ++p) {
                b0[p] = __builtin_bit_cast(v8bf, *reinterpret_cast<const v4i*>(s0 + p * RS_CT * 16 * rs.spitch + ch * 64));
                b1[p] = __builtin_bit_cast(v8bf, *reinterpret_cast<const v4i*>(s1 + p * RS_CT * 16 * rs.spitch + ch * 64));
            }
            y0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a3, b0[0], y0, 0, 0, 0);
            y1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a3, b1[0], y1, 0, 0, 0);
            y0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, b0[2], y0, 0, 0, 0);
            y1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, b1[2], y1, 0, 0, 0);
            y0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a2, b0[1], y0, 0, 0, 0);
            y1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a2, b1[1], y1, 0, 0, 0);
            y0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a2, b0[0], y0, 0, 0, 0);
            y1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a2, b1[0], y1, 0, 0, 0);
            y0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, b0[1], y0, 0, 0, 0);
            y1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, b1[1], y1, 0, 0, 0);
            y0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, b0[0], y0, 0, 0, 0);
            y1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, b1[0], y1, 0, 0, 0);
        }
    }

    // ---- rotated values out (lane: d = 16*strip + 4*lg + v, c = 16*tile + li), and my extremes
    float mx = 0.0f, mn = 0.0f;
    const int d0 = wave * 16 + 4 * lg;
    float* xt = xs + t * K;
#pragma unroll
    for (int u = 0; u < RS_CT; ++u) {
        const v4f y = u == 0 ? y0 : y1;
        const int c = (RS_CT * j + u) * 16 + li;
        if ((u == 0 || two) && c < n1) {
#pragma unroll
            for (int v = 0; v < 4; ++v)
                if (d0 + v < n2) {
                    xt[(int64_t)c * n2 + d0 + v] = y[v];
                    mx = fmaxf(mx, y[v]);
                    mn = fminf(mn, y[v]);
                }
        }
    }
    mx = bwla_wave_max(mx);
    mn = -bwla_wave_max(-mn);
    if (lane == 0) { red[wave] = mx; red[32 + wave] = mn; }
    bwla_lds_barrier();
    if (tid == 0) {
        float hi = red[0], lo = red[32];
        for (int w = 1; w < sh.strips; ++w) { hi = fmaxf(hi, red[w]); lo = fminf(lo, red[32 + w]); }
        pmax[(t * rs.G + j) * 2] = hi;                 // largest and smallest value of my slice (0 included)
        pmax[(t * rs.G + j) * 2 + 1] = lo;
        if (j == 0) qsum[t] = 0;                       // the quantizing launch adds its sums up here
    }
}

// second launch of the split rotation: RS_QB workgroups per token quantize the rotated values, each
// its share of k, every load in flight at once; the code sum is added up in qsum[t], which the
// first launch has set to zero (integer adds: the order does not matter)
constexpr int RS_QB = 8;
constexpr int RS_QI = 4;             // float4 per thread: K <= RS_QB * 512 * RS_QI * 4
__global__ __launch_bounds__(512) void quantize_rows_kernel(const float* __restrict__ xs, const float* __restrict__ pmax,
                                                            int G, int64_t K, int8_t* __restrict__ q,
                                                            float* __restrict__ scale, int32_t* __restrict__ qsum,
                                                            float qmax, int asym, float* __restrict__ tmode, int tp,
                                                            float* __restrict__ zcs) {
    __shared__ int redi[8];
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
    float hi = pmax[t * G * 2], lo = pmax[t * G * 2 + 1];
    for (int j = 1; j < G; ++j) { hi = fmaxf(hi, pmax[(t * G + j) * 2]); lo = fminf(lo, pmax[(t * G + j) * 2 + 1]); }
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

// where rotate3_token<.., LOCAL> leaves its results (resident shapes only)
__device__ __forceinline__ FusedLocal r3_local(const char* lds, const R3Shape& sh) {
    // words [0, 16) largest values, [16, 32) code sums, [32, 48) smallest values (of the 64 words
    // behind the chunk buffers)
    const float* red = reinterpret_cast<const float*>(lds + sh.r0bytes + (size_t)sh.nbuf * sh.cbytes);
    return FusedLocal{lds, red, reinterpret_cast<const int*>(red) + 16, sh.strips};
}

}  // namespace
