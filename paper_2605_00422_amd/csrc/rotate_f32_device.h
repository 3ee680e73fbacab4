// Rotation + quantization of one token per workgroup on fp32 MFMA (fp32 activations, and shapes
// the bf16 form does not take); see rotate_quant.hip for the method.
#pragma once
#include "rotate_common.h"

namespace {

// ================================================================== rotation of one token
template <bool BF16>
__device__ __forceinline__ void store_token_vec(float* d, const uint4& v) {
    // d is 16-byte aligned (pitches and column offsets are multiples of four floats)
    float4* d4 = reinterpret_cast<float4*>(d);
    if (BF16) {
        d4[0] = make_float4(__uint_as_float(v.x << 16), __uint_as_float(v.x & 0xffff0000u),
                            __uint_as_float(v.y << 16), __uint_as_float(v.y & 0xffff0000u));
        d4[1] = make_float4(__uint_as_float(v.z << 16), __uint_as_float(v.z & 0xffff0000u),
                            __uint_as_float(v.w << 16), __uint_as_float(v.w & 0xffff0000u));
    } else {
        d4[0] = make_float4(__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w));
    }
}

// Token (and, in resident mode, R2 and R1 transposed) into LDS.  Every global load of a batch is
// issued before the first use, so that a decode token pays one memory round trip.  Items are
// 16-byte vectors [token | R2 | R1] when the shapes allow it; odd shapes take scalar loops.
template <bool BF16>
__device__ __forceinline__ void fill_lds(const void* __restrict__ X, int64_t row_off, int n1, int n2,
                                         const float* __restrict__ R1, const float* __restrict__ R2,
                                         const RqShape& sh, float* V, float* r2t, float* r1t) {
    constexpr int VEC = BF16 ? 8 : 4;
    const bool with_factors = sh.resident;
    // zero the padding first (disjoint from everything written below)
    if (n2 != sh.n2p || n1 != sh.n1p) {
        for (int idx = threadIdx.x; idx < sh.n1p * sh.n2p; idx += RQ_THREADS) {
            const int a = idx / sh.n2p, b = idx - a * sh.n2p;
            if (a >= n1 || b >= n2) V[a * sh.ldv + b] = 0.0f;
        }
        if (with_factors) {
            for (int idx = threadIdx.x; idx < sh.n2p * sh.n2p; idx += RQ_THREADS) {
                const int d = idx / sh.n2p, b = idx - d * sh.n2p;
                if (d >= n2 || b >= n2) r2t[d * sh.ld2t + b] = 0.0f;
            }
            for (int idx = threadIdx.x; idx < sh.n1p * sh.n1p; idx += RQ_THREADS) {
                const int c = idx / sh.n1p, a = idx - c * sh.n1p;
                if (c >= n1 || a >= n1) r1t[c * sh.ld1t + a] = 0.0f;
            }
        }
    }
    if ((n2 % VEC) == 0 && (n1 & 3) == 0 && (n2 & 3) == 0) {
        const int vpr = n2 / VEC, nx = n1 * vpr;
        // A factor is cut into blocks of 16 rows k x 4 vectors (16 columns x): lane l of an item
        // group takes row (l & 15), vector (l >> 4).  A wave then loads 64-byte row pieces and its
        // four transposed scalar stores each hit 64 distinct LDS banks.
        const int q2 = n2 >> 2, kg2 = (n2 + 15) >> 4, nr2 = with_factors ? 64 * kg2 * ((q2 + 3) >> 2) : 0;
        const int q1 = n1 >> 2, kg1 = (n1 + 15) >> 4, nr1 = with_factors ? 64 * kg1 * ((q1 + 3) >> 2) : 0;
        const int total = nx + nr2 + nr1;
        const FastDiv dvpr(vpr), dkg1(kg1), dkg2(kg2);
        auto factor_item = [&](int it, bool& second, int& k, int& x4) -> bool {
            second = it >= nx + nr2;
            const int j = second ? it - nx - nr2 : it - nx;
            const int l = j & 63, blk = j >> 6;
            const int kg = second ? kg1 : kg2;
            const int xgi = (second ? dkg1 : dkg2).div(blk), kgi = blk - xgi * kg;
            k = 16 * kgi + (l & 15);
            x4 = 4 * xgi + (l >> 4);
            return k < (second ? n1 : n2) && x4 < (second ? q1 : q2);
        };
        for (int base = 0; base < total; base += 8 * RQ_THREADS) {
            uint4 v[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int it = base + e * RQ_THREADS + threadIdx.x;
                v[e] = make_uint4(0, 0, 0, 0);
                if (it < nx) {
                    const int a = dvpr.div(it), b0 = (it - a * vpr) * VEC;
                    const int64_t off = row_off + (int64_t)a * n2 + b0;
                    v[e] = BF16 ? *reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(X) + off)
                                : *reinterpret_cast<const uint4*>(reinterpret_cast<const float*>(X) + off);
                } else if (it < total) {
                    bool second; int k, x4;
                    if (factor_item(it, second, k, x4))
                        v[e] = *reinterpret_cast<const uint4*>((second ? R1 : R2) + (int64_t)k * (second ? n1 : n2) + 4 * x4);
                }
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int it = base + e * RQ_THREADS + threadIdx.x;
                if (it < nx) {
                    const int a = dvpr.div(it), b0 = (it - a * vpr) * VEC;
                    store_token_vec<BF16>(V + a * sh.ldv + b0, v[e]);
                } else if (it < total) {
                    // R[k][x0..x0+3] -> transposed rows x0..x0+3, column k
                    bool second; int k, x4;
                    if (factor_item(it, second, k, x4)) {
                        const int ld = second ? sh.ld1t : sh.ld2t;
                        float* d = (second ? r1t : r2t) + 4 * x4 * ld + k;
                        d[0] = __uint_as_float(v[e].x); d[ld] = __uint_as_float(v[e].y);
                        d[2 * ld] = __uint_as_float(v[e].z); d[3 * ld] = __uint_as_float(v[e].w);
                    }
                }
            }
        }
    } else {
        for (int idx = threadIdx.x; idx < n1 * n2; idx += RQ_THREADS) {
            const int a = idx / n2, b = idx - a * n2;
            const int64_t i = row_off + idx;
            V[a * sh.ldv + b] = BF16 ? bwla_bf16_to_f32(reinterpret_cast<const uint16_t*>(X)[i])
                                     : reinterpret_cast<const float*>(X)[i];
        }
        if (with_factors) {
            for (int idx = threadIdx.x; idx < n2 * n2; idx += RQ_THREADS) {
                const int b = idx / n2, d = idx - b * n2;
                r2t[d * sh.ld2t + b] = R2[idx];
            }
            for (int idx = threadIdx.x; idx < n1 * n1; idx += RQ_THREADS) {
                const int a = idx / n1, c = idx - a * n1;
                r1t[c * sh.ld1t + a] = R1[idx];
            }
        }
    }
}

// one 16-wide contraction group: four MFMA steps fed by one 128-bit LDS read per operand
__device__ __forceinline__ v4f mfma16(const float* ap, const float* bp, v4f acc) {
    const float4 a4 = *reinterpret_cast<const float4*>(ap);
    const float4 b4 = *reinterpret_cast<const float4*>(bp);
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a4.x, b4.x, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a4.y, b4.y, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a4.z, b4.z, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a4.w, b4.w, acc, 0, 0, 0);
    return acc;
}

// Streamed factor chunks (n % 4 == 0): chunk c holds R[16c .. 16c+15][all x]; a thread carries
// two 16-byte vectors of it (slot e: local row kk[e], columns x0[e]..x0[e]+3).  They are stored
// transposed, [x][k_local] with pitch RQ_CLD.
struct ChunkRegs { float4 v[2]; };
struct ChunkSlots { int kk[2], x0[2]; };
// lane l of a 64-item group takes local row (l & 15) and vector (l >> 4) of the group's 16
// columns: 64-byte row pieces from global memory, conflict-free transposed stores (pitch 20
// floats puts the four column groups 16 banks apart)
__device__ __forceinline__ ChunkSlots chunk_slots(int n) {
    ChunkSlots cs;
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const int idx = threadIdx.x + e * RQ_THREADS;
        const int l = idx & 63, grp = idx >> 6;
        cs.x0[e] = (4 * grp + (l >> 4)) << 2;
        cs.kk[e] = cs.x0[e] < n ? (l & 15) : RQ_CK;      // RQ_CK marks an unused slot
    }
    return cs;
}
__device__ __forceinline__ ChunkRegs chunk_fetch(const float* __restrict__ R, int n, int c, const ChunkSlots& cs) {
    ChunkRegs cr;
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const int k = c * RQ_CK + cs.kk[e];
        cr.v[e] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (cs.kk[e] < RQ_CK && k < n) cr.v[e] = *reinterpret_cast<const float4*>(R + (int64_t)k * n + cs.x0[e]);
    }
    return cr;
}
__device__ __forceinline__ void chunk_store(float* dst, const ChunkSlots& cs, const ChunkRegs& cr) {
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        if (cs.kk[e] < RQ_CK) {
            float* d = dst + cs.x0[e] * RQ_CLD + cs.kk[e];
            d[0] = cr.v[e].x; d[RQ_CLD] = cr.v[e].y; d[2 * RQ_CLD] = cr.v[e].z; d[3 * RQ_CLD] = cr.v[e].w;
        }
    }
}

template <bool BF16>
__device__ __forceinline__ void rotate_token(float* lds, const void* __restrict__ X, int64_t t, int64_t K, int n1,
                                             int n2, const float* __restrict__ R1, const float* __restrict__ R2,
                                             int8_t* __restrict__ q, float* __restrict__ scale,
                                             int32_t* __restrict__ qsum, float* __restrict__ tmode, int tp,
                                             float qmax, bool asym, bool shift) {
    const RqShape sh = rq_shape(n1, n2);
    float* reg = lds;                                              // V, later ZT
    float* fac = lds + sh.region;                                  // R2T | R1T (resident) or two chunk buffers
    float* red = fac + (sh.resident ? sh.n2p * sh.ld2t + sh.n1p * sh.ld1t : 2 * sh.nmaxp * RQ_CLD);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // wave-uniform: tile indices stay scalar
    const int li = lane & 15, lg = lane >> 4;
    const int tiles1 = sh.n1p >> 4, tiles2 = sh.n2p >> 4;         // 16-row tiles along a/c and along b/d
    const int tiles = tiles1 * tiles2;
    const int my_tiles = (tiles - wave + RQ_WAVES - 1) / RQ_WAVES;      // tiles wave, wave+8, ...
    const FastDiv dt1(tiles1), dt2(tiles2);
    // Tiles are processed in pairs so that two independent read->MFMA chains overlap; an odd
    // last tile is paired with a copy of itself whose result is never used.
#define RQ_PAIR_SLOTS(g) const int s0 = 2 * (g), s1 = (2 * (g) + 1 < my_tiles) ? 2 * (g) + 1 : 2 * (g)

    v4f acc[RQ_MAXT];
#pragma unroll
    for (int s = 0; s < RQ_MAXT; ++s) acc[s] = v4f{0.f, 0.f, 0.f, 0.f};

    fill_lds<BF16>(X, t * K, n1, n2, R1, R2, sh, reg, fac, fac + sh.n2p * sh.ld2t);

    if (sh.resident) {
        const float* r2t = fac;
        const float* r1t = fac + sh.n2p * sh.ld2t;
        __syncthreads();
        // stage 1: Z[a][d] = sum_b V[a][b] R2[b][d];   tile (ti over a, tj over d)
#pragma unroll
        for (int g = 0; g < RQ_MAXT / 2; ++g) {
            if (2 * g < my_tiles) {
                RQ_PAIR_SLOTS(g);
                const int tau0 = wave + s0 * RQ_WAVES, tau1 = wave + s1 * RQ_WAVES;
                const int ti0 = dt2.div(tau0), tj0 = tau0 - ti0 * tiles2;
                const int ti1 = dt2.div(tau1), tj1 = tau1 - ti1 * tiles2;
                const float* ap0 = reg + (ti0 * 16 + li) * sh.ldv + 4 * lg;
                const float* bp0 = r2t + (tj0 * 16 + li) * sh.ld2t + 4 * lg;
                const float* ap1 = reg + (ti1 * 16 + li) * sh.ldv + 4 * lg;
                const float* bp1 = r2t + (tj1 * 16 + li) * sh.ld2t + 4 * lg;
#pragma unroll 2
                for (int k = 0; k < sh.n2p; k += 16) {
                    acc[2 * g] = mfma16(ap0 + k, bp0 + k, acc[2 * g]);
                    acc[2 * g + 1] = mfma16(ap1 + k, bp1 + k, acc[2 * g + 1]);
                }
            }
        }
        bwla_lds_barrier();                                        // every wave is done reading V
        // lane holds Z[a = ti*16 + 4*lg + v][d = tj*16 + li]: one 128-bit store into ZT[d][a..a+3]
#pragma unroll
        for (int s = 0; s < RQ_MAXT; ++s) {
            if (s < my_tiles) {
                const int tau = wave + s * RQ_WAVES;
                const int ti = dt2.div(tau), tj = tau - ti * tiles2;
                *reinterpret_cast<float4*>(reg + (tj * 16 + li) * sh.ldzt + ti * 16 + 4 * lg) =
                    make_float4(acc[s][0], acc[s][1], acc[s][2], acc[s][3]);
                acc[s] = v4f{0.f, 0.f, 0.f, 0.f};
            }
        }
        bwla_lds_barrier();                                        // ZT is published
        // stage 2: Yt[d][c] = sum_a ZT[d][a] R1[a][c];   tile (ti over d, tj over c)
#pragma unroll
        for (int g = 0; g < RQ_MAXT / 2; ++g) {
            if (2 * g < my_tiles) {
                RQ_PAIR_SLOTS(g);
                const int tau0 = wave + s0 * RQ_WAVES, tau1 = wave + s1 * RQ_WAVES;
                const int ti0 = dt1.div(tau0), tj0 = tau0 - ti0 * tiles1;
                const int ti1 = dt1.div(tau1), tj1 = tau1 - ti1 * tiles1;
                const float* ap0 = reg + (ti0 * 16 + li) * sh.ldzt + 4 * lg;
                const float* bp0 = r1t + (tj0 * 16 + li) * sh.ld1t + 4 * lg;
                const float* ap1 = reg + (ti1 * 16 + li) * sh.ldzt + 4 * lg;
                const float* bp1 = r1t + (tj1 * 16 + li) * sh.ld1t + 4 * lg;
#pragma unroll 2
                for (int k = 0; k < sh.n1p; k += 16) {
                    acc[2 * g] = mfma16(ap0 + k, bp0 + k, acc[2 * g]);
                    acc[2 * g + 1] = mfma16(ap1 + k, bp1 + k, acc[2 * g + 1]);
                }
            }
        }
    } else {
        // ---------------- factors streamed in 16-index chunks: RQ_RING chunks in flight in
        // registers, two chunk buffers in LDS, one LDS-only barrier per chunk
        float* cb = fac;
        const int cbs = sh.nmaxp * RQ_CLD;                         // floats per chunk buffer
        for (int idx = tid; idx < 2 * cbs; idx += RQ_THREADS) cb[idx] = 0.0f;    // padded rows stay zero
        __syncthreads();
        for (int stage = 0; stage < 2; ++stage) {
            const float* R = stage == 0 ? R2 : R1;
            const int n = stage == 0 ? n2 : n1;
            const int nchunks = (n + RQ_CK - 1) / RQ_CK;
            const int lda = stage == 0 ? sh.ldv : sh.ldzt;
            const int tdiv = stage == 0 ? tiles2 : tiles1;         // tiles along the operand-B rows
            const FastDiv dtd = stage == 0 ? dt2 : dt1;
            const ChunkSlots cs = chunk_slots(n);
            ChunkRegs ring[RQ_RING];
#pragma unroll
            for (int d = 0; d < RQ_RING; ++d) ring[d] = chunk_fetch(R, n, d, cs);
            chunk_store(cb, cs, ring[0]);
            bwla_lds_barrier();                                    // chunk 0 (and V / ZT) published
            for (int c0 = 0; c0 < nchunks; c0 += RQ_RING) {
#pragma unroll
                for (int d = 0; d < RQ_RING; ++d) {
                    const int c = c0 + d;
                    if (c < nchunks) {
                        const float* cur = cb + (c & 1) * cbs;
#pragma unroll
                        for (int g = 0; g < RQ_MAXT / 2; ++g) {
                            if (2 * g < my_tiles) {
                                RQ_PAIR_SLOTS(g);
                                const int tau0 = wave + s0 * RQ_WAVES, tau1 = wave + s1 * RQ_WAVES;
                                const int ti0 = dtd.div(tau0), tj0 = tau0 - ti0 * tdiv;
                                const int ti1 = dtd.div(tau1), tj1 = tau1 - ti1 * tdiv;
                                acc[2 * g] = mfma16(reg + (ti0 * 16 + li) * lda + c * RQ_CK + 4 * lg,
                                                    cur + (tj0 * 16 + li) * RQ_CLD + 4 * lg, acc[2 * g]);
                                acc[2 * g + 1] = mfma16(reg + (ti1 * 16 + li) * lda + c * RQ_CK + 4 * lg,
                                                        cur + (tj1 * 16 + li) * RQ_CLD + 4 * lg, acc[2 * g + 1]);
                            }
                        }
                    }
                    // chunk c+1 (requested RQ_RING - 1 chunks ago) into the other buffer, whose last
                    // readers passed the previous barrier; then refill this ring slot
                    chunk_store(cb + ((c + 1) & 1) * cbs, cs, ring[(d + 1) % RQ_RING]);
                    ring[d] = chunk_fetch(R, n, c + RQ_RING, cs);
                    bwla_lds_barrier();
                }
            }
            if (stage == 0) {
                // lane holds Z[a = ti*16 + 4*lg + v][d = tj*16 + li] -> ZT[d][a..a+3]; V is dead
                // (every wave passed the last barrier of the loop)
#pragma unroll
                for (int s = 0; s < RQ_MAXT; ++s) {
                    if (s < my_tiles) {
                        const int tau = wave + s * RQ_WAVES;
                        const int ti = dt2.div(tau), tj = tau - ti * tiles2;
                        *reinterpret_cast<float4*>(reg + (tj * 16 + li) * sh.ldzt + ti * 16 + 4 * lg) =
                            make_float4(acc[s][0], acc[s][1], acc[s][2], acc[s][3]);
                        acc[s] = v4f{0.f, 0.f, 0.f, 0.f};
                    }
                }
            }
        }
    }

    // ================= per-token max magnitude
    float mx = 0.0f, mn = 0.0f;
#pragma unroll
    for (int s = 0; s < RQ_MAXT; ++s)
        if (s < my_tiles) {
#pragma unroll
            for (int v = 0; v < 4; ++v) { mx = fmaxf(mx, acc[s][v]); mn = fminf(mn, acc[s][v]); }
        }
    mx = bwla_wave_max(mx);
    mn = -bwla_wave_max(-mn);
    if (lane == 0) { red[wave] = mx; red[32 + wave] = mn; }
    bwla_lds_barrier();                                // also: every wave is done reading ZT
    float hi = red[0], lo = red[32];
#pragma unroll
    for (int w = 1; w < RQ_WAVES; ++w) { hi = fmaxf(hi, red[w]); lo = fminf(lo, red[32 + w]); }
    const QuantPlan qp = quant_plan(hi, lo, qmax, asym);

    // ================= quantize from registers into an LDS byte image of the token's codes:
    // lane holds Yt[d = ti*16 + 4*lg + v][c = tj*16 + li], i.e. four consecutive d of one c
    int8_t* codes = reinterpret_cast<int8_t*>(reg);
    int lsum = 0;
#pragma unroll
    for (int s = 0; s < RQ_MAXT; ++s) {
        if (s < my_tiles) {
            const int tau = wave + s * RQ_WAVES;
            const int ti = dt1.div(tau), tj = tau - ti * tiles1;
            const int c = tj * 16 + li, d0 = ti * 16 + 4 * lg;
            int code[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) code[v] = quant_code(acc[s][v], qp);
            if (c < n1) {
                if ((n2 & 3) == 0) {
                    if (d0 < n2) {
                        *reinterpret_cast<int*>(codes + c * n2 + d0) = (code[0] & 0xff) | ((code[1] & 0xff) << 8) |
                                                                        ((code[2] & 0xff) << 16) | (code[3] << 24);
                        lsum += code[0] + code[1] + code[2] + code[3];
                    }
                } else {
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        if (d0 + v < n2) {
                            codes[c * n2 + d0 + v] = (int8_t)code[v];
                            lsum += code[v];
                        }
                }
            }
        }
    }
    lsum = bwla_wave_sum_i32(lsum);
    int* redi = reinterpret_cast<int*>(red) + 16;
    if (lane == 0) redi[wave] = lsum;
    bwla_lds_barrier();
    // coalesced 16-byte stores of the code row (K % 16 == 0)
    {
        const uint4* src = reinterpret_cast<const uint4*>(codes);
        uint4* dst = reinterpret_cast<uint4*>(q + t * K);
        const int n16 = (int)(K >> 4);
        for (int idx = tid; idx < n16; idx += RQ_THREADS) dst[idx] = src[idx];
    }
    if (tid == 0) {
        int tot = 0;
#pragma unroll
        for (int w = 0; w < RQ_WAVES; ++w) tot += redi[w];
        qsum[t] = tot;
        const float sc = quant_scale(hi, lo, qmax, asym);
        scale[t] = sc;
        quant_extras(tmode, tp, t, asym, shift, qp, sc, tot, K);
    }
#undef RQ_PAIR_SLOTS
}

}  // namespace
