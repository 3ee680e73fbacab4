// Online Orthogonal-Kronecker rotation fused with per-token symmetric INT6 quantization.
//
//   X~[t, c*n2 + d] = sum_{a,b} X[t, a*n2 + b] R1[a,c] R2[b,d]      (paper Sec. 3.1; App. A.2.2)
//
// evaluated per token as two small products on the row-major n1 x n2 reshape V:
//   stage 1  Z = V R2      stage 2  Y = R1^T Z
// on fp32 MFMA (16x16x4), one workgroup per token.  The token tile lives in LDS, Z replaces V
// in place (through the accumulators), and Y never leaves registers before it is quantized:
//   amax = max |Y|, scale = amax / 31, q = clamp(rint(Y * 31 / amax)), qsum = sum q.
#include "bwla_internal.h"

namespace {

constexpr int RQ_THREADS = 512;
constexpr int RQ_WAVES = RQ_THREADS / 64;
constexpr int RQ_MAXT = 16;   // 16x16 output tiles per wavefront
constexpr int RQ_KC = 8;      // factor rows staged per chunk

__host__ __device__ inline int rq_pad16(int n) { return (n + 15) & ~15; }
// leading dimension with ld % 32 == 17: both the "16 rows x 4 columns" and the
// "4 rows x 16 columns" access patterns of the two stages then spread over the LDS banks
__host__ __device__ inline int rq_ld(int np16) { return np16 + ((np16 & 31) == 16 ? 1 : 17); }

struct RqShape {
    int n1, n2, n1p, n2p, ldz, ldr;
    size_t lds_bytes;
};

__host__ __device__ inline RqShape rq_shape(int n1, int n2) {
    RqShape s;
    s.n1 = n1; s.n2 = n2;
    s.n1p = rq_pad16(n1); s.n2p = rq_pad16(n2);
    s.ldz = rq_ld(s.n2p);
    const int nmax = s.n1p > s.n2p ? s.n1p : s.n2p;
    s.ldr = rq_ld(nmax);
    s.lds_bytes = ((size_t)s.n1p * s.ldz + 2 * RQ_KC * s.ldr + 64) * sizeof(float);
    return s;
}

template <bool BF16>
__device__ __forceinline__ float load_x(const void* X, int64_t idx) {
    if (BF16) return bwla_bf16_to_f32(reinterpret_cast<const uint16_t*>(X)[idx]);
    return reinterpret_cast<const float*>(X)[idx];
}

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

template <bool BF16>
__global__ __launch_bounds__(RQ_THREADS) void rotate_quant_kernel(
    const void* __restrict__ X, int64_t K, int n1, int n2, const float* __restrict__ R1,
    const float* __restrict__ R2, int8_t* __restrict__ q, float* __restrict__ scale,
    int32_t* __restrict__ qsum) {
    extern __shared__ float lds[];
    const RqShape sh = rq_shape(n1, n2);
    float* buf = lds;                                  // n1p x ldz
    float* rch = lds + (size_t)sh.n1p * sh.ldz;        // 2 x RQ_KC x ldr
    float* red = rch + 2 * RQ_KC * sh.ldr;             // 64 floats of reduction scratch

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 15, lg = lane >> 4;
    const int64_t t = blockIdx.x;
    const int tilesN = sh.n2p >> 4;
    const int tiles = (sh.n1p >> 4) * tilesN;
    const int my_tiles = (tiles - wave + RQ_WAVES - 1) / RQ_WAVES;   // tiles wave, wave+8, ...

    // ---- token row -> LDS (fp32, zero padded)
    {
        const int total = sh.n1p * sh.n2p;
        for (int idx = tid; idx < total; idx += RQ_THREADS) {
            const int a = idx / sh.n2p, b = idx - a * sh.n2p;
            float v = 0.0f;
            if (a < n1 && b < n2) v = load_x<BF16>(X, t * K + (int64_t)a * n2 + b);
            buf[a * sh.ldz + b] = v;
        }
    }

    v4f acc[RQ_MAXT];
    float creg[4];

    // ================= stage 1: Z = V R2  (contraction over b, length n2)
#pragma unroll
    for (int s = 0; s < RQ_MAXT; ++s) acc[s] = v4f{0.f, 0.f, 0.f, 0.f};
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
        }
    }

    // ================= stage 2: Y = R1^T Z  (contraction over a, length n1)
#pragma unroll
    for (int s = 0; s < RQ_MAXT; ++s) acc[s] = v4f{0.f, 0.f, 0.f, 0.f};
    {
        const int nchunks = (n1 + RQ_KC - 1) / RQ_KC;
        chunk_fetch(R1, n1, sh.n1p, 0, creg);
        chunk_store(rch, sh.n1p, sh.ldr, creg);   // last stage-1 reads of rch ended at its final barrier
        __syncthreads();                          // also publishes Z
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
                        // A[c_out][a] = R1[a][c_out];  B[a][d] = Z[a][d]
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
    __syncthreads();                                   // also: every wave is done reading Z
    float amax = red[0];
#pragma unroll
    for (int w = 1; w < RQ_WAVES; ++w) amax = fmaxf(amax, red[w]);
    const float inv = amax > 0.0f ? 31.0f / amax : 0.0f;

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
    __syncthreads();
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
        scale[t] = amax / 31.0f;
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

size_t bwla_rotate_lds_bytes(int n1, int n2) { return rq_shape(n1, n2).lds_bytes; }
int bwla_rotate_tiles(int n1, int n2) { return (rq_pad16(n1) / 16) * (rq_pad16(n2) / 16); }
int bwla_rotate_max_tiles() { return RQ_MAXT * RQ_WAVES; }

hipError_t bwla_launch_rotate_quant(const bwla_layer_t* L, const void* dX, int xdtype, int64_t M,
                                    int8_t* dq, float* dscale, int32_t* dqsum, hipStream_t st) {
    const char* blob = (const char*)L->d_blob;
    const float* R1 = (const float*)(blob + L->off_R1);
    const float* R2 = (const float*)(blob + L->off_R2);
    const RqShape sh = rq_shape(L->n1, L->n2);
    hipError_t e;
    if (xdtype == BWLA_X_BF16) {
        static bwla_lds_attr attr;
        e = attr.ensure((const void*)rotate_quant_kernel<true>, sh.lds_bytes);
        if (e != hipSuccess) return e;
        rotate_quant_kernel<true><<<dim3((unsigned)M), dim3(RQ_THREADS), sh.lds_bytes, st>>>(
            dX, L->K, L->n1, L->n2, R1, R2, dq, dscale, dqsum);
    } else {
        static bwla_lds_attr attr;
        e = attr.ensure((const void*)rotate_quant_kernel<false>, sh.lds_bytes);
        if (e != hipSuccess) return e;
        rotate_quant_kernel<false><<<dim3((unsigned)M), dim3(RQ_THREADS), sh.lds_bytes, st>>>(
            dX, L->K, L->n1, L->n2, R1, R2, dq, dscale, dqsum);
    }
    return hipGetLastError();
}

hipError_t bwla_launch_code_sums(const int8_t* dq, int64_t M, int64_t K, int32_t* dqsum, hipStream_t st) {
    code_sums_kernel<<<dim3((unsigned)M), dim3(256), 0, st>>>(dq, K, dqsum);
    return hipGetLastError();
}
