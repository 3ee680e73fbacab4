// bwla_rotate_quant in one launch: workgroups [0, M) rotate and quantize one token each,
// the workgroups behind them compute the PSP projection T = X U.
//
// Rotation (paper Sec. 3.1; App. A.2.2), per token on the row-major n1 x n2 reshape V:
//   X~[t, c*n2 + d] = sum_{a,b} X[t, a*n2 + b] R1[a,c] R2[b,d]   =   (R1^T (V R2))[c,d]
//   stage 1  Z = V R2      stage 2  Y = R1^T Z          (fp32 MFMA 16x16x4)
// The token tile lives in LDS, Z replaces V in place (through the accumulators), and Y never
// leaves registers before it is quantized:
//   amax = max |Y|, scale = amax / 31, q = clamp(rint(Y * 31 / amax)), qsum = sum q.
// When both factors fit into LDS next to the token they are loaded once, together with the
// token ("resident" mode: one global round trip, four barriers in total -- the decode case);
// otherwise they are streamed in 8-row chunks through a double buffer.
//
// PSP projection (paper Sec. 3.2), T = X U from the un-rotated, un-quantized activations:
// a workgroup takes 16 tokens x 512 columns of K, stages its slice of U (fp16) in LDS with
// 16-byte loads and multiplies on fp32 MFMA.  With several slices, every workgroup writes its
// partial tile to scratch and the one that arrives last adds them in slice order.
#include "bwla_internal.h"

namespace {

#ifdef BWLA_TRACE
__device__ long long bwla_rq_trace_buf[16 * 8 * 16];
#define RQTRACE(slot) do { if ((threadIdx.x & 63) == 0 && blockIdx.x < 16) bwla_rq_trace_buf[(blockIdx.x * 8 + (threadIdx.x >> 6)) * 16 + (slot)] = __builtin_readcyclecounter(); } while (0)
#else
#define RQTRACE(slot) do { } while (0)
#endif

constexpr int RQ_THREADS = 512;
constexpr int RQ_WAVES = RQ_THREADS / 64;
constexpr int RQ_MAXT = 16;          // 16x16 output tiles per wavefront
constexpr int RQ_KC = 8;             // factor rows per chunk in streaming mode
constexpr int PP_SLICE = 512;        // columns of K per projection workgroup
constexpr int PP_MAXJT = BWLA_MAX_RANK / 16;
constexpr size_t RQ_LDS_LIMIT = 160 * 1024 - 256;   // leaves room for the few static bytes

__host__ __device__ inline int rq_pad16(int n) { return (n + 15) & ~15; }
// leading dimension with ld % 32 == 17: both the "16 rows x 4 columns" and the
// "4 rows x 16 columns" access patterns of the two stages then spread over the LDS banks
__host__ __device__ inline int rq_ld(int np16) { return np16 + ((np16 & 31) == 16 ? 1 : 17); }

struct RqShape {
    int n1, n2, n1p, n2p, ldz, ldr, ld1, ld2;
    bool resident;
    size_t lds_bytes;      // rotation workgroups
};

__host__ __device__ inline RqShape rq_shape(int n1, int n2) {
    RqShape s;
    s.n1 = n1; s.n2 = n2;
    s.n1p = rq_pad16(n1); s.n2p = rq_pad16(n2);
    s.ldz = rq_ld(s.n2p);
    const int nmax = s.n1p > s.n2p ? s.n1p : s.n2p;
    s.ldr = rq_ld(nmax);                 // streaming mode: one pitch for both factors
    s.ld2 = rq_ld(s.n2p);                // resident mode: R2 is n2p rows x ld2, R1 is n1p rows x ld1
    s.ld1 = rq_ld(s.n1p);
    const size_t res = ((size_t)s.n1p * s.ldz + (size_t)s.n2p * s.ld2 + (size_t)s.n1p * s.ld1 + 64) * sizeof(float);
    const size_t str = ((size_t)s.n1p * s.ldz + 2 * RQ_KC * s.ldr + 64) * sizeof(float);
    s.resident = res <= RQ_LDS_LIMIT;
    s.lds_bytes = s.resident ? res : str;
    return s;
}

__host__ __device__ inline size_t pp_lds_bytes(int r) {
    const int rp = ((r + 15) >> 4) * 16;
    const size_t us = (size_t)PP_SLICE * (rp + 8) * 2;                 // U slice, fp16, padded pitch
    const size_t red = (size_t)RQ_WAVES * (rp / 16) * 64 * 16;         // cross-wave reduction (reuses the slice)
    return (us > red ? us : red) + 16;
}

// ================================================================== rotation of one token
// Stage a chunk of RQ_KC rows of an n x n factor (rows k0.., all columns) into registers.
__device__ __forceinline__ void chunk_fetch(const float* __restrict__ R, int n, int np, int k0, float (&reg)[4]) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int idx = threadIdx.x + e * RQ_THREADS;
        const int rr = idx / np, cc = idx - rr * np;
        const int k = k0 + rr;
        reg[e] = (rr < RQ_KC && k < n && cc < n) ? R[(int64_t)k * n + cc] : 0.0f;
    }
}
__device__ __forceinline__ void chunk_store(float* __restrict__ dst, int np, int ldr, const float (&reg)[4]) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int idx = threadIdx.x + e * RQ_THREADS;
        const int rr = idx / np, cc = idx - rr * np;
        if (rr < RQ_KC) dst[rr * ldr + cc] = reg[e];
    }
}

// whole factor -> LDS, zero padded to np rows x np columns (pitch ld)
__device__ __forceinline__ void factor_to_lds(const float* __restrict__ R, int n, int np, int ld, float* dst) {
    if ((n & 3) == 0) {
        const int q4 = np >> 2;                                    // float4 per padded row
        for (int idx = threadIdx.x; idx < np * q4; idx += RQ_THREADS) {
            const int rr = idx / q4, c4 = (idx - rr * q4) << 2;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (rr < n && c4 < n) v = *reinterpret_cast<const float4*>(R + (int64_t)rr * n + c4);
            float* d = dst + rr * ld + c4;
            d[0] = v.x; d[1] = v.y; d[2] = v.z; d[3] = v.w;
        }
    } else {
        for (int idx = threadIdx.x; idx < np * np; idx += RQ_THREADS) {
            const int rr = idx / np, cc = idx - rr * np;
            dst[rr * ld + cc] = (rr < n && cc < n) ? R[(int64_t)rr * n + cc] : 0.0f;
        }
    }
}

template <bool BF16>
__device__ __forceinline__ void token_to_lds(const void* __restrict__ X, int64_t row_off, int n1, int n2,
                                             const RqShape& sh, float* buf) {
    constexpr int VEC = BF16 ? 8 : 4;                              // elements per 16-byte load
    if (n2 % VEC == 0) {
        const int vpr = n2 / VEC;
        for (int idx = threadIdx.x; idx < n1 * vpr; idx += RQ_THREADS) {
            const int a = idx / vpr, b0 = (idx - a * vpr) * VEC;
            float* d = buf + a * sh.ldz + b0;
            if (BF16) {
                const uint4 raw = *reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(X) + row_off +
                                                                  (int64_t)a * n2 + b0);
                d[0] = __uint_as_float(raw.x << 16); d[1] = __uint_as_float(raw.x & 0xffff0000u);
                d[2] = __uint_as_float(raw.y << 16); d[3] = __uint_as_float(raw.y & 0xffff0000u);
                d[4] = __uint_as_float(raw.z << 16); d[5] = __uint_as_float(raw.z & 0xffff0000u);
                d[6] = __uint_as_float(raw.w << 16); d[7] = __uint_as_float(raw.w & 0xffff0000u);
            } else {
                const float4 raw = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(X) + row_off +
                                                                    (int64_t)a * n2 + b0);
                d[0] = raw.x; d[1] = raw.y; d[2] = raw.z; d[3] = raw.w;
            }
        }
        // zero padding: columns [n2, n2p) of the real rows, then the rows [n1, n1p)
        const int padc = sh.n2p - n2;
        for (int idx = threadIdx.x; idx < n1 * padc; idx += RQ_THREADS) {
            const int a = idx / padc, b = n2 + (idx - a * padc);
            buf[a * sh.ldz + b] = 0.0f;
        }
        for (int idx = threadIdx.x; idx < (sh.n1p - n1) * sh.n2p; idx += RQ_THREADS) {
            const int a = n1 + idx / sh.n2p, b = idx % sh.n2p;
            buf[a * sh.ldz + b] = 0.0f;
        }
    } else {
        for (int idx = threadIdx.x; idx < sh.n1p * sh.n2p; idx += RQ_THREADS) {
            const int a = idx / sh.n2p, b = idx - a * sh.n2p;
            float v = 0.0f;
            if (a < n1 && b < n2) {
                const int64_t i = row_off + (int64_t)a * n2 + b;
                v = BF16 ? bwla_bf16_to_f32(reinterpret_cast<const uint16_t*>(X)[i])
                         : reinterpret_cast<const float*>(X)[i];
            }
            buf[a * sh.ldz + b] = v;
        }
    }
}

// Token, R2 and R1 into LDS with every global load of a batch issued before the first use, so
// that a decode token pays one memory round trip instead of one per array.  Items are 16-byte
// vectors: [token | R2 | R1]; a thread takes items tid, tid + 512, ... in batches of 8.
template <bool BF16>
__device__ __forceinline__ void resident_fill(const void* __restrict__ X, int64_t row_off, int n1, int n2,
                                              const float* __restrict__ R1, const float* __restrict__ R2,
                                              const RqShape& sh, float* buf, float* r2s, float* r1s) {
    constexpr int VEC = BF16 ? 8 : 4;
    if ((n2 % VEC) != 0 || (n1 & 3) != 0 || (n2 & 3) != 0) {       // odd shapes: plain loops
        token_to_lds<BF16>(X, row_off, n1, n2, sh, buf);
        factor_to_lds(R2, n2, sh.n2p, sh.ld2, r2s);
        factor_to_lds(R1, n1, sh.n1p, sh.ld1, r1s);
        return;
    }
    const int vpr = n2 / VEC;                      // token vectors per row
    const int nx = n1 * vpr;
    const int q2 = n2 >> 2, nr2 = n2 * q2;         // float4 per R2 row, R2 vectors
    const int q1 = n1 >> 2, nr1 = n1 * q1;
    const int total = nx + nr2 + nr1;
    for (int base = 0; base < total; base += 8 * RQ_THREADS) {
        uint4 v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int it = base + e * RQ_THREADS + threadIdx.x;
            v[e] = make_uint4(0, 0, 0, 0);
            if (it < nx) {
                const int a = it / vpr, b0 = (it - a * vpr) * VEC;
                const int64_t off = row_off + (int64_t)a * n2 + b0;
                v[e] = BF16 ? *reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(X) + off)
                            : *reinterpret_cast<const uint4*>(reinterpret_cast<const float*>(X) + off);
            } else if (it < nx + nr2) {
                v[e] = *reinterpret_cast<const uint4*>(R2 + (int64_t)(it - nx) * 4);
            } else if (it < total) {
                v[e] = *reinterpret_cast<const uint4*>(R1 + (int64_t)(it - nx - nr2) * 4);
            }
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int it = base + e * RQ_THREADS + threadIdx.x;
            if (it < nx) {
                const int a = it / vpr, b0 = (it - a * vpr) * VEC;
                float* d = buf + a * sh.ldz + b0;
                if (BF16) {
                    d[0] = __uint_as_float(v[e].x << 16); d[1] = __uint_as_float(v[e].x & 0xffff0000u);
                    d[2] = __uint_as_float(v[e].y << 16); d[3] = __uint_as_float(v[e].y & 0xffff0000u);
                    d[4] = __uint_as_float(v[e].z << 16); d[5] = __uint_as_float(v[e].z & 0xffff0000u);
                    d[6] = __uint_as_float(v[e].w << 16); d[7] = __uint_as_float(v[e].w & 0xffff0000u);
                } else {
                    d[0] = __uint_as_float(v[e].x); d[1] = __uint_as_float(v[e].y);
                    d[2] = __uint_as_float(v[e].z); d[3] = __uint_as_float(v[e].w);
                }
            } else if (it < total) {
                const bool second = it >= nx + nr2;
                const int j = second ? it - nx - nr2 : it - nx;
                const int q = second ? q1 : q2;
                const int rr = j / q, c4 = (j - rr * q) << 2;
                float* d = (second ? r1s + rr * sh.ld1 : r2s + rr * sh.ld2) + c4;
                d[0] = __uint_as_float(v[e].x); d[1] = __uint_as_float(v[e].y);
                d[2] = __uint_as_float(v[e].z); d[3] = __uint_as_float(v[e].w);
            }
        }
    }
    // zero padding of the token tile and of the factors (rows and columns up to the next 16)
    if (n1 == sh.n1p && n2 == sh.n2p) return;
    const int padc = sh.n2p - n2;
    for (int idx = threadIdx.x; idx < n1 * padc; idx += RQ_THREADS) {
        const int a = idx / padc, b = n2 + (idx - a * padc);
        buf[a * sh.ldz + b] = 0.0f;
    }
    for (int idx = threadIdx.x; idx < (sh.n1p - n1) * sh.n2p; idx += RQ_THREADS)
        buf[(n1 + idx / sh.n2p) * sh.ldz + idx % sh.n2p] = 0.0f;
    for (int idx = threadIdx.x; idx < sh.n2p * sh.n2p; idx += RQ_THREADS) {
        const int rr = idx / sh.n2p, cc = idx - rr * sh.n2p;
        if (rr >= n2 || cc >= n2) r2s[rr * sh.ld2 + cc] = 0.0f;
    }
    for (int idx = threadIdx.x; idx < sh.n1p * sh.n1p; idx += RQ_THREADS) {
        const int rr = idx / sh.n1p, cc = idx - rr * sh.n1p;
        if (rr >= n1 || cc >= n1) r1s[rr * sh.ld1 + cc] = 0.0f;
    }
}

template <bool BF16>
__device__ __forceinline__ void rotate_token(float* lds, const void* __restrict__ X, int64_t t, int64_t K, int n1,
                                             int n2, const float* __restrict__ R1, const float* __restrict__ R2,
                                             int8_t* __restrict__ q, float* __restrict__ scale,
                                             int32_t* __restrict__ qsum) {
    const RqShape sh = rq_shape(n1, n2);
    float* buf = lds;                                              // n1p x ldz
    float* fac = lds + (size_t)sh.n1p * sh.ldz;                    // factors (resident) or chunk ring (streaming)
    float* red = fac + (sh.resident ? (size_t)sh.n2p * sh.ld2 + (size_t)sh.n1p * sh.ld1 : (size_t)2 * RQ_KC * sh.ldr);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 15, lg = lane >> 4;
    const int tilesN = sh.n2p >> 4;
    const int tiles = (sh.n1p >> 4) * tilesN;
    const int my_tiles = (tiles - wave + RQ_WAVES - 1) / RQ_WAVES;      // tiles wave, wave+8, ...

    v4f acc[RQ_MAXT];
#pragma unroll
    for (int s = 0; s < RQ_MAXT; ++s) acc[s] = v4f{0.f, 0.f, 0.f, 0.f};

    if (sh.resident) {
        // ---------------- everything the token needs in one round trip
        float* r2s = fac;
        float* r1s = fac + (size_t)sh.n2p * sh.ld2;
        RQTRACE(0);
        resident_fill<BF16>(X, t * K, n1, n2, R1, R2, sh, buf, r2s, r1s);
        RQTRACE(1);
        __syncthreads();
        RQTRACE(2);
        // stage 1: Z = V R2 (contraction over b)
#pragma unroll
        for (int s = 0; s < RQ_MAXT; ++s) {
            if (s < my_tiles) {
                const int tau = wave + s * RQ_WAVES;
                const int ti = tau / tilesN, tj = tau - ti * tilesN;
                const float* ap = buf + (ti * 16 + li) * sh.ldz + lg;
                const float* bp = r2s + lg * sh.ld2 + tj * 16 + li;
#pragma unroll 4
                for (int k = 0; k < sh.n2p; k += 4)
                    acc[s] = __builtin_amdgcn_mfma_f32_16x16x4f32(ap[k], bp[k * sh.ld2], acc[s], 0, 0, 0);
            }
        }
        RQTRACE(3);
        bwla_lds_barrier();                                        // every wave is done reading V
#pragma unroll
        for (int s = 0; s < RQ_MAXT; ++s) {
            if (s < my_tiles) {
                const int tau = wave + s * RQ_WAVES;
                const int ti = tau / tilesN, tj = tau - ti * tilesN;
#pragma unroll
                for (int v = 0; v < 4; ++v) buf[(ti * 16 + 4 * lg + v) * sh.ldz + tj * 16 + li] = acc[s][v];
                acc[s] = v4f{0.f, 0.f, 0.f, 0.f};
            }
        }
        bwla_lds_barrier();                                        // Z is published
        RQTRACE(4);
        // stage 2: Y = R1^T Z (contraction over a):  A[c][a] = R1[a][c],  B[a][d] = Z[a][d]
#pragma unroll
        for (int s = 0; s < RQ_MAXT; ++s) {
            if (s < my_tiles) {
                const int tau = wave + s * RQ_WAVES;
                const int ti = tau / tilesN, tj = tau - ti * tilesN;
                const float* ap = r1s + lg * sh.ld1 + ti * 16 + li;
                const float* bp = buf + lg * sh.ldz + tj * 16 + li;
#pragma unroll 4
                for (int k = 0; k < sh.n1p; k += 4)
                    acc[s] = __builtin_amdgcn_mfma_f32_16x16x4f32(ap[k * sh.ld1], bp[k * sh.ldz], acc[s], 0, 0, 0);
            }
        }
    } else {
        // ---------------- factors streamed in RQ_KC-row chunks through a double buffer
        float* rch = fac;
        float creg[4];
        token_to_lds<BF16>(X, t * K, n1, n2, sh, buf);
        {
            const int nchunks = (n2 + RQ_KC - 1) / RQ_KC;
            chunk_fetch(R2, n2, sh.n2p, 0, creg);
            chunk_store(rch, sh.n2p, sh.ldr, creg);
            __syncthreads();
            for (int c = 0; c < nchunks; ++c) {
                const float* cur = rch + (c & 1) * RQ_KC * sh.ldr;
                if (c + 1 < nchunks) chunk_fetch(R2, n2, sh.n2p, (c + 1) * RQ_KC, creg);
#pragma unroll
                for (int s = 0; s < RQ_MAXT; ++s) {
                    if (s < my_tiles) {
                        const int tau = wave + s * RQ_WAVES;
                        const int ti = tau / tilesN, tj = tau - ti * tilesN;
#pragma unroll
                        for (int ks = 0; ks < RQ_KC; ks += 4) {
                            const float a = buf[(ti * 16 + li) * sh.ldz + c * RQ_KC + ks + lg];
                            const float b = cur[(ks + lg) * sh.ldr + tj * 16 + li];
                            acc[s] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc[s], 0, 0, 0);
                        }
                    }
                }
                if (c + 1 < nchunks) chunk_store(rch + ((c + 1) & 1) * RQ_KC * sh.ldr, sh.n2p, sh.ldr, creg);
                __syncthreads();
            }
        }
        // Z replaces V (every wave is past its last read of V after the loop's final barrier)
#pragma unroll
        for (int s = 0; s < RQ_MAXT; ++s) {
            if (s < my_tiles) {
                const int tau = wave + s * RQ_WAVES;
                const int ti = tau / tilesN, tj = tau - ti * tilesN;
#pragma unroll
                for (int v = 0; v < 4; ++v) buf[(ti * 16 + 4 * lg + v) * sh.ldz + tj * 16 + li] = acc[s][v];
                acc[s] = v4f{0.f, 0.f, 0.f, 0.f};
            }
        }
        {
            const int nchunks = (n1 + RQ_KC - 1) / RQ_KC;
            chunk_fetch(R1, n1, sh.n1p, 0, creg);
            chunk_store(rch, sh.n1p, sh.ldr, creg);       // last stage-1 reads of rch ended at its final barrier
            __syncthreads();                              // also publishes Z
            for (int c = 0; c < nchunks; ++c) {
                const float* cur = rch + (c & 1) * RQ_KC * sh.ldr;
                if (c + 1 < nchunks) chunk_fetch(R1, n1, sh.n1p, (c + 1) * RQ_KC, creg);
#pragma unroll
                for (int s = 0; s < RQ_MAXT; ++s) {
                    if (s < my_tiles) {
                        const int tau = wave + s * RQ_WAVES;
                        const int ti = tau / tilesN, tj = tau - ti * tilesN;
#pragma unroll
                        for (int ks = 0; ks < RQ_KC; ks += 4) {
                            const float a = cur[(ks + lg) * sh.ldr + ti * 16 + li];
                            const float b = buf[(c * RQ_KC + ks + lg) * sh.ldz + tj * 16 + li];
                            acc[s] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc[s], 0, 0, 0);
                        }
                    }
                }
                if (c + 1 < nchunks) chunk_store(rch + ((c + 1) & 1) * RQ_KC * sh.ldr, sh.n1p, sh.ldr, creg);
                __syncthreads();
            }
        }
    }

    RQTRACE(5);
    // ================= per-token max magnitude
    float m = 0.0f;
#pragma unroll
    for (int s = 0; s < RQ_MAXT; ++s)
        if (s < my_tiles) {
#pragma unroll
            for (int v = 0; v < 4; ++v) m = fmaxf(m, fabsf(acc[s][v]));
        }
    m = bwla_wave_max(m);
    if (lane == 0) red[wave] = m;
    bwla_lds_barrier();                                // also: every wave is done reading Z
    float amax = red[0];
#pragma unroll
    for (int w = 1; w < RQ_WAVES; ++w) amax = fmaxf(amax, red[w]);
    const float inv = amax > 0.0f ? 31.0f / amax : 0.0f;
    RQTRACE(6);

    // ================= quantize from registers into an LDS byte image of the token's codes
    int8_t* codes = reinterpret_cast<int8_t*>(buf);
    int lsum = 0;
#pragma unroll
    for (int s = 0; s < RQ_MAXT; ++s) {
        if (s < my_tiles) {
            const int tau = wave + s * RQ_WAVES;
            const int ti = tau / tilesN, tj = tau - ti * tilesN;
            const int d = tj * 16 + li;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int c = ti * 16 + 4 * lg + v;
                float r = rintf(acc[s][v] * inv);
                r = fminf(fmaxf(r, -31.0f), 31.0f);
                const int code = (int)r;
                if (c < n1 && d < n2) {
                    codes[c * n2 + d] = (int8_t)code;
                    lsum += code;
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
    RQTRACE(7);
    if (tid == 0) {
        int tot = 0;
#pragma unroll
        for (int w = 0; w < RQ_WAVES; ++w) tot += redi[w];
        qsum[t] = tot;
        scale[t] = amax / 31.0f;
    }
    RQTRACE(8);
}

// ================================================================== PSP projection T = X U
template <bool BF16>
__device__ __forceinline__ void psp_block(char* smem, const void* __restrict__ X, int64_t M, int64_t K, int r,
                                          const __half* __restrict__ U, float* __restrict__ T,
                                          int* __restrict__ counters, float* __restrict__ partials, int S, int tt,
                                          int s) {
    __shared__ int is_last;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 15, lg = lane >> 4;
    const int JT = (r + 15) >> 4, rp = JT * 16, pitch = rp + 8;
    __half* Us = reinterpret_cast<__half*>(smem);
    const int64_t kbase = (int64_t)s * PP_SLICE;

    // activations of my 64 columns first (they do not depend on LDS): 4 groups of 16 columns,
    // lane (li, lg) owns columns 16*g + 4*lg + e, e = 0..3, of token li in MFMA step e
    int64_t trow = (int64_t)tt * 16 + li;
    if (trow > M - 1) trow = M - 1;                    // padded token rows are never stored
    float x[4][4];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const int64_t kx = kbase + wave * 64 + g * 16 + 4 * lg;
        if (kx < K) {
            if (BF16) {
                const uint2 raw = *reinterpret_cast<const uint2*>(reinterpret_cast<const uint16_t*>(X) + trow * K + kx);
                x[g][0] = __uint_as_float(raw.x << 16); x[g][1] = __uint_as_float(raw.x & 0xffff0000u);
                x[g][2] = __uint_as_float(raw.y << 16); x[g][3] = __uint_as_float(raw.y & 0xffff0000u);
            } else {
                const float4 raw = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(X) + trow * K + kx);
                x[g][0] = raw.x; x[g][1] = raw.y; x[g][2] = raw.z; x[g][3] = raw.w;
            }
        } else {
            x[g][0] = x[g][1] = x[g][2] = x[g][3] = 0.0f;
        }
    }
    // U slice -> LDS with 16-byte loads (rows past K are zero)
    {
        const int gpr = rp >> 3;                           // 16-byte granules per row
        for (int idx = tid; idx < PP_SLICE * gpr; idx += RQ_THREADS) {
            const int row = idx / gpr, g = idx - row * gpr;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (kbase + row < K) v = *reinterpret_cast<const uint4*>(U + (kbase + row) * rp + g * 8);
            *reinterpret_cast<uint4*>(Us + row * pitch + g * 8) = v;
        }
    }
    __syncthreads();

    v4f acc[PP_MAXJT];
#pragma unroll
    for (int jt = 0; jt < PP_MAXJT; ++jt) acc[jt] = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll 1
    for (int g = 0; g < 4; ++g) {
        const __half* up = Us + (wave * 64 + g * 16 + 4 * lg) * pitch + li;
        const float xg[4] = {g == 0 ? x[0][0] : g == 1 ? x[1][0] : g == 2 ? x[2][0] : x[3][0],
                             g == 0 ? x[0][1] : g == 1 ? x[1][1] : g == 2 ? x[2][1] : x[3][1],
                             g == 0 ? x[0][2] : g == 1 ? x[1][2] : g == 2 ? x[2][2] : x[3][2],
                             g == 0 ? x[0][3] : g == 1 ? x[1][3] : g == 2 ? x[2][3] : x[3][3]};
#pragma unroll
        for (int jt = 0; jt < PP_MAXJT; ++jt) {
            if (jt < JT) {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    acc[jt] = __builtin_amdgcn_mfma_f32_16x16x4f32(xg[e], __half2float(up[e * pitch + jt * 16]),
                                                                  acc[jt], 0, 0, 0);
            }
        }
    }
    __syncthreads();                                   // the U slice is dead: reuse it for the reduction
    v4f* red = reinterpret_cast<v4f*>(smem);           // [wave][jt][lane]
#pragma unroll
    for (int jt = 0; jt < PP_MAXJT; ++jt)
        if (jt < JT) red[(wave * JT + jt) * 64 + lane] = acc[jt];
    __syncthreads();
    // waves share the column tiles; lane holds tokens 4*lg + v, column jt*16 + li
    for (int jt = wave; jt < JT; jt += RQ_WAVES) {
        v4f sum = red[jt * 64 + lane];
        for (int w = 1; w < RQ_WAVES; ++w) sum += red[(w * JT + jt) * 64 + lane];
        const int col = jt * 16 + li;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int row = 4 * lg + v;
            const int64_t tok = (int64_t)tt * 16 + row;
            if (S == 1) {
                if (tok < M && col < r) T[tok * r + col] = sum[v];
            } else {
                partials[(((int64_t)tt * S + s) * 16 + row) * rp + col] = sum[v];
            }
        }
    }
    if (S == 1) return;

    __threadfence();
    __syncthreads();
    if (tid == 0) {
        const int old = atomicAdd(&counters[tt], 1);
        is_last = (old == S - 1);
    }
    __syncthreads();
    if (!is_last) return;
    __threadfence();
    // last workgroup of this token tile: add the S partial tiles in slice order
    for (int idx = tid; idx < 16 * rp; idx += RQ_THREADS) {
        const int row = idx / rp, col = idx - row * rp;
        const int64_t tok = (int64_t)tt * 16 + row;
        if (tok < M && col < r) {
            float sum = 0.0f;
            for (int ss = 0; ss < S; ++ss)
                sum += __builtin_nontemporal_load(&partials[(((int64_t)tt * S + ss) * 16 + row) * rp + col]);
            T[tok * r + col] = sum;
        }
    }
    if (tid == 0) counters[tt] = 0;                    // leave the scratch as it was found
}

struct RqArgs {
    const void* X; int64_t M, K; int n1, n2, r;
    const float* R1; const float* R2; const __half* U;
    int8_t* q; float* scale; int32_t* qsum; float* T;
    int* counters; float* partials; int S;
};

template <bool BF16>
__global__ __launch_bounds__(RQ_THREADS) void rotate_quant_kernel(RqArgs a) {
    extern __shared__ float lds[];
    if ((int64_t)blockIdx.x < a.M) {
        rotate_token<BF16>(lds, a.X, blockIdx.x, a.K, a.n1, a.n2, a.R1, a.R2, a.q, a.scale, a.qsum);
    } else {
        const int pb = (int)(blockIdx.x - a.M);
        psp_block<BF16>(reinterpret_cast<char*>(lds), a.X, a.M, a.K, a.r, a.U, a.T, a.counters, a.partials, a.S,
                        pb / a.S, pb % a.S);
    }
}

__global__ __launch_bounds__(256) void code_sums_kernel(const int8_t* __restrict__ q, int64_t K,
                                                        int32_t* __restrict__ qsum) {
    __shared__ int red[4];
    const int64_t t = blockIdx.x;
    const int* row = reinterpret_cast<const int*>(q + t * K);
    int s = 0;
    for (int i = threadIdx.x; i < (int)(K >> 2); i += 256) {
        const int w = row[i];
        s += (int)(int8_t)(w & 0xff) + (int)(int8_t)((w >> 8) & 0xff) + (int)(int8_t)((w >> 16) & 0xff) + (w >> 24);
    }
    s = bwla_wave_sum_i32(s);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) qsum[t] = red[0] + red[1] + red[2] + red[3];
}

}  // namespace

#ifdef BWLA_TRACE
extern "C" int bwla_rq_trace_dump(long long* host, int n) {
    return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(bwla_rq_trace_buf), (size_t)n * sizeof(long long));
}
#endif

size_t bwla_rotate_lds_bytes(int n1, int n2) { return rq_shape(n1, n2).lds_bytes; }
int bwla_rotate_tiles(int n1, int n2) { return (rq_pad16(n1) / 16) * (rq_pad16(n2) / 16); }
int bwla_rotate_max_tiles() { return RQ_MAXT * RQ_WAVES; }

bwla_psp_plan bwla_make_psp_plan(int64_t M, int64_t K, int r) {
    bwla_psp_plan p;
    p.token_tiles = (int)((M + 15) / 16);
    p.k_per_split = PP_SLICE;
    p.splits = r > 0 ? (int)((K + PP_SLICE - 1) / PP_SLICE) : 1;
    return p;
}

hipError_t bwla_launch_rotate_quant(const bwla_layer_t* L, const void* dX, int xdtype, int64_t M, int8_t* dq,
                                    float* dscale, int32_t* dqsum, float* dT, void* dws, const bwla_psp_plan& plan,
                                    hipStream_t st) {
    const char* blob = (const char*)L->d_blob;
    const RqShape sh = rq_shape(L->n1, L->n2);
    size_t lds = sh.lds_bytes;
    int64_t blocks = M;
    if (L->r > 0) {
        const size_t pl = pp_lds_bytes(L->r);
        if (pl > lds) lds = pl;
        blocks += (int64_t)plan.token_tiles * plan.splits;
    }
    RqArgs a;
    a.X = dX; a.M = M; a.K = L->K; a.n1 = L->n1; a.n2 = L->n2; a.r = L->r;
    a.R1 = (const float*)(blob + L->off_R1); a.R2 = (const float*)(blob + L->off_R2);
    a.U = (const __half*)(blob + L->off_U);
    a.q = dq; a.scale = dscale; a.qsum = dqsum; a.T = dT;
    a.counters = (int*)dws;
    a.partials = dws ? (float*)((char*)dws + bwla_align256((uint64_t)plan.token_tiles * sizeof(int))) : nullptr;
    a.S = plan.splits;
    hipError_t e;
    if (xdtype == BWLA_X_BF16) {
        static bwla_lds_attr attr;
        e = attr.ensure((const void*)rotate_quant_kernel<true>, lds);
        if (e != hipSuccess) return e;
        rotate_quant_kernel<true><<<dim3((unsigned)blocks), dim3(RQ_THREADS), lds, st>>>(a);
    } else {
        static bwla_lds_attr attr;
        e = attr.ensure((const void*)rotate_quant_kernel<false>, lds);
        if (e != hipSuccess) return e;
        rotate_quant_kernel<false><<<dim3((unsigned)blocks), dim3(RQ_THREADS), lds, st>>>(a);
    }
    return hipGetLastError();
}

hipError_t bwla_launch_code_sums(const int8_t* dq, int64_t M, int64_t K, int32_t* dqsum, hipStream_t st) {
    code_sums_kernel<<<dim3((unsigned)M), dim3(256), 0, st>>>(dq, K, dqsum);
    return hipGetLastError();
}
