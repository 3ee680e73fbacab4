// Offline packing of one layer: sign bits into the tiled layout, per-row scale, fp16 PSP
// factors, fp32 Kronecker factors.  (Paper Algorithm 2 "Final binarization" restricted to sign
// and scale; Sign(x) = +1 iff x > 0, paper Eq. 3; alpha = mean |w|, paper App. A.2.4.)
#include "bwla_internal.h"

namespace {

// One wavefront builds one 1 KiB unit (16 rows x 512 columns).
__global__ __launch_bounds__(64) void pack_bits_kernel(const float* __restrict__ W, int64_t N, int64_t K,
                                                       int64_t chunks, uint32_t* __restrict__ bits) {
    const int64_t unit = blockIdx.x;
    const int64_t rt = unit / chunks, kc = unit % chunks;
    const int lane = threadIdx.x;
    const int i = lane & 15, g = lane >> 4;
    const int64_t n = rt * BWLA_TILE_ROWS + i;
    const int64_t kbase = kc * BWLA_CHUNK_COLS + g * 128;
    uint32_t w[4] = {0u, 0u, 0u, 0u};
    if (n < N) {
        const float* row = W + n * K;
#pragma unroll 4
        for (int kk = 0; kk < 128; ++kk) {
            const int64_t k = kbase + kk;
            const float v = (k < K) ? row[k] : 0.0f;
            const int j = kk >> 4, d = (kk >> 2) & 3, b = kk & 3;
            if (v > 0.0f) w[d] |= 1u << (8 * b + j);
        }
    }
    uint4 out = make_uint4(w[0], w[1], w[2], w[3]);
    reinterpret_cast<uint4*>(bits)[unit * 64 + lane] = out;
}

// Exact round-to-nearest-even of a non-negative double to IEEE binary16 bits (a double ->
// float -> half chain can round twice).
__device__ uint16_t double_to_half_bits(double x) {
    if (!(x > 0.0)) return 0;
    if (x >= 65520.0) return 0x7C00;                     // rounds to infinity
    if (x < 6.103515625e-05) {                           // below 2^-14: subnormal grid 2^-24
        const double m = rint(ldexp(x, 24));             // 0..1024 (1024 encodes the least normal)
        return (uint16_t)(int)m;
    }
    int e;
    (void)frexp(x, &e);                                  // x = f * 2^e, f in [0.5, 1)
    e -= 1;                                              // x = (1.f) * 2^e
    double m = rint(ldexp(x, 10 - e));                   // in [1024, 2048]
    if (m >= 2048.0) { m = 1024.0; e += 1; }
    return (uint16_t)(((e + 15) << 10) | ((int)m - 1024));
}

// One wavefront per row: fp64 sum of magnitudes, rounded once to fp16.
__global__ __launch_bounds__(64) void row_scale_kernel(const float* __restrict__ W, int64_t N, int64_t K,
                                                       uint16_t* __restrict__ alpha) {
    const int64_t n = blockIdx.x;
    if (n >= N) return;
    const float* row = W + n * K;
    double s = 0.0;
    for (int64_t k = threadIdx.x; k < K; k += 64) s += (double)fabsf(row[k]);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
    if (threadIdx.x == 0) alpha[n] = double_to_half_bits(s / (double)K);
}

// Layers whose mode adds columns to V: one workgroup per tile of 16 rows.
// Row shift (paper Sec. 3 "Discussion", Eq. 1-2; mu_col >= 0): first the fp64 row means mu; else
// mu = 0.  Then, chunk by chunk, the bits of (w - mu > 0) in the tiled layout (padding columns
// stay 0), the fp64 sums of |w - mu| and the counts of positive signs, added up in a fixed order.
// delta goes where alpha is, mu (fp16) into column mu_col of V; for asymmetric activation codes
// (asym_col >= 0) delta_n * rowsum_n, with delta as stored and rowsum_n = sum_k Sign = 2 pos - K,
// goes into columns asym_col, asym_col + 1 as two fp16 terms.
__global__ __launch_bounds__(256) void pack_rows_mode_kernel(const float* __restrict__ W, int64_t N, int64_t K,
                                                             int64_t chunks, uint32_t* __restrict__ bits,
                                                             uint16_t* __restrict__ alpha,
                                                             uint16_t* __restrict__ V16, int rp, int mu_col,
                                                             int asym_col) {
    __shared__ double mu[16];
    __shared__ double part[4][64];
    __shared__ int pos[4][64];
    const int64_t rt = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int rr = 0; rr < 4; ++rr) {                     // wave w: rows 4w .. 4w+3 of the tile
        const int64_t n = rt * BWLA_TILE_ROWS + wave * 4 + rr;
        double s = 0.0;
        if (n < N && mu_col >= 0) {
            const float* row = W + n * K;
            for (int64_t k = lane; k < K; k += 64) s += (double)row[k];
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
        if (lane == 0) mu[wave * 4 + rr] = s / (double)K;
    }
    __syncthreads();
    const int i = lane & 15, g = lane >> 4;
    const int64_t n = rt * BWLA_TILE_ROWS + i;
    const double m = mu[i];
    double dsum = 0.0;
    int npos = 0;
    for (int64_t kc = wave; kc < chunks; kc += 4) {
        const int64_t kbase = kc * BWLA_CHUNK_COLS + g * 128;
        uint32_t w[4] = {0u, 0u, 0u, 0u};
        if (n < N) {
            const float* row = W + n * K;
#pragma unroll 4
            for (int kk = 0; kk < 128; ++kk) {
                const int64_t k = kbase + kk;
                if (k < K) {
                    const double c = (double)row[k] - m;
                    const int j = kk >> 4, d = (kk >> 2) & 3, b = kk & 3;
                    if (c > 0.0) { w[d] |= 1u << (8 * b + j); ++npos; }
                    dsum += fabs(c);
                }
            }
        }
        reinterpret_cast<uint4*>(bits)[(rt * chunks + kc) * 64 + lane] = make_uint4(w[0], w[1], w[2], w[3]);
    }
    part[wave][lane] = dsum;
    pos[wave][lane] = npos;
    __syncthreads();
    if (tid < 16 && rt * BWLA_TILE_ROWS + tid < N) {
        double s = 0.0;
        int p = 0;
        for (int w2 = 0; w2 < 4; ++w2)
            for (int g2 = 0; g2 < 4; ++g2) { s += part[w2][g2 * 16 + tid]; p += pos[w2][g2 * 16 + tid]; }
        const int64_t row = rt * BWLA_TILE_ROWS + tid;
        const uint16_t d16 = double_to_half_bits(s / (double)K);
        alpha[row] = d16;
        if (mu_col >= 0) {
            const double mm = mu[tid];
            V16[row * rp + mu_col] = (uint16_t)((mm < 0.0 ? 0x8000u : 0u) | double_to_half_bits(fabs(mm)));
        }
        if (asym_col >= 0) {
            const float c = __half2float(__ushort_as_half(d16)) * (float)(2 * p - (int)K);
            const __half hi = __float2half_rn(c);
            const __half lo = __float2half_rn(c - __half2float(hi));
            V16[row * rp + asym_col] = __half_as_ushort(hi);
            V16[row * rp + asym_col + 1] = __half_as_ushort(lo);
        }
    }
}

// rows x r fp32 -> rows x rp fp16 (rp = r rounded up to 16, zero padded)
__global__ void f32_to_f16_rows_kernel(const float* __restrict__ src, int64_t rows, int r, int rp,
                                       __half* __restrict__ dst) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= rows * rp) return;
    const int64_t row = i / rp;
    const int col = (int)(i - row * rp);
    dst[i] = col < r ? __float2half_rn(src[row * r + col]) : __float2half_rn(0.0f);
}

// K x r fp32 -> fp16 in the order in which an MFMA (16x16x32) reads its B operand: blocks
// [16-column tile jt][32-row step ks] of 1 KiB, inside a block lane (li, lg) = lg * 16 + li holds the
// eight values U[32 ks + 8 lg + e][16 jt + li], e = 0..7 (columns r..rp-1 zero).  A wavefront-wide
// 16-byte load of a block is one contiguous KiB.
__global__ void u_pack_f16_kernel(const float* __restrict__ U, int64_t K, int r, int rp, __half* __restrict__ Up) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)rp * K) return;
    const int e = (int)(i & 7), lane = (int)((i >> 3) & 63);
    const int64_t blk = i >> 9, ksteps = K >> 5;
    const int64_t jt = blk / ksteps, ks = blk - jt * ksteps;
    const int64_t k = 32 * ks + 8 * (lane >> 4) + e;
    const int j = (int)(16 * jt + (lane & 15));
    Up[i] = j < r ? __float2half_rn(U[k * r + j]) : __float2half_rn(0.0f);
}

// n x n fp32 factor R -> three bf16 term planes P[term][x][k], x < np16, k < np32, of R transposed:
// P[.][x][pos] = terms of R[k][x] (zero outside n x n), where pos = k, or -- `permute` -- inside
// every block of 32 the position 8 g + e holds k = 32 blk + (e < 4 ? 4 g + e : 16 + 4 g + e - 4):
// the order in which two stacked 16-row MFMA accumulator tiles present their rows to a lane group.
__global__ void factor_planes_kernel(const float* __restrict__ R, int n, int permute, uint16_t* __restrict__ P) {
    const int np16 = (n + 15) & ~15, np32 = (n + 31) & ~31;
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= np16 * np32) return;
    const int x = i / np32, pos = i - x * np32;
    int k = pos;
    if (permute) {
        const int blk = pos >> 5, g = (pos >> 3) & 3, e = pos & 7;
        k = 32 * blk + (e < 4 ? 4 * g + e : 16 + 4 * g + e - 4);
    }
    const float v = (x < n && k < n) ? R[(int64_t)k * n + x] : 0.0f;
    // round to nearest even on the upper 16 bits; the remainders are exact in fp32
    auto bf = [](float f) -> uint32_t {
        const uint32_t u = __float_as_uint(f);
        return (u + 0x7fffu + ((u >> 16) & 1u)) & 0xffff0000u;
    };
    const uint32_t h1 = bf(v);
    const float r1 = v - __uint_as_float(h1);
    const uint32_t h2 = bf(r1);
    const float r2 = r1 - __uint_as_float(h2);
    const uint32_t h3 = bf(r2);
    const int64_t plane = (int64_t)np16 * np32;
    P[i] = (uint16_t)(h1 >> 16);
    P[plane + i] = (uint16_t)(h2 >> 16);
    P[2 * plane + i] = (uint16_t)(h3 >> 16);
}

// Factor planes in MFMA operand order (factor pairs that are multiples of 32 up to 160), one 1 KiB
// block per MFMA operand, lane (li, lg) = lg * 16 + li holding eight 16-bit values:
//   R2d part (pairs of 32 or 64 only), blocks [strip w][step kb][term p < 3]: term p (bf16; the
//            three add up to the fp32 value) of R2[b = 32 kb + 8 lg + e][d = 16 w + li]
//   R1h part, blocks [step ch][term t < 2][tile tc]: term t (fp16; hi = nearest, lo = remainder) of
//            256 R1[a][c = 16 tc + li], a = 32 ch + (e < 4 ? 4 lg + e : 16 + 4 lg + e - 4): the order in
//            which two stacked 16-row accumulator tiles present their rows to a lane group
//   R2h part, blocks [strip w][step kb][term t < 2]: the same two fp16 terms of 256 R2[b][d]
__global__ void decode_planes_kernel(const float* __restrict__ R1, const float* __restrict__ R2, int n1, int n2,
                                     int with_r2d, uint16_t* __restrict__ out) {
    const int at = n1 / 16, k1 = n2 / 32, ch2 = n1 / 32, strips = n2 / 16;
    const int nb2 = with_r2d ? strips * k1 * 3 : 0, nb1 = ch2 * 2 * at, nb2h = strips * k1 * 2;
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (nb2 + nb1 + nb2h) * 512) return;
    const int blk = i >> 9, lane = (i >> 3) & 63, e = i & 7, li = lane & 15, lg = lane >> 4;
    if (blk < nb2) {
        const int p = blk % 3, kb = (blk / 3) % k1, w = blk / (3 * k1);
        const float v = R2[(int64_t)(32 * kb + 8 * lg + e) * n2 + 16 * w + li];
        auto bf = [](float f) -> uint32_t {
            const uint32_t u = __float_as_uint(f);
            return (u + 0x7fffu + ((u >> 16) & 1u)) & 0xffff0000u;
        };
        const uint32_t h1 = bf(v);
        const float r1 = v - __uint_as_float(h1);
        const uint32_t h2 = bf(r1);
        const uint32_t h3 = bf(r1 - __uint_as_float(h2));
        out[i] = (uint16_t)((p == 0 ? h1 : p == 1 ? h2 : h3) >> 16);
    } else if (blk < nb2 + nb1) {
        const int b1 = blk - nb2;
        const int tc = b1 % at, t = (b1 / at) % 2, ch = b1 / (2 * at);
        const int a = 32 * ch + (e < 4 ? 4 * lg + e : 16 + 4 * lg + e - 4);
        const float v = 256.0f * R1[(int64_t)a * n1 + 16 * tc + li];
        const __half hi = __float2half_rn(v);
        const __half lo = __float2half_rn(v - __half2float(hi));
        out[i] = __half_as_ushort(t == 0 ? hi : lo);
    } else {
        // R2h, blocks [strip w][step kb][term t < 2]: 256 R2[b = 32 kb + 8 lg + e][d = 16 w + li]
        const int b2 = blk - nb2 - nb1;
        const int t = b2 % 2, kb = (b2 / 2) % k1, w = b2 / (2 * k1);
        const float v = 256.0f * R2[(int64_t)(32 * kb + 8 * lg + e) * n2 + 16 * w + li];
        const __half hi = __float2half_rn(v);
        const __half lo = __float2half_rn(v - __half2float(hi));
        out[i] = __half_as_ushort(t == 0 ? hi : lo);
    }
}

__global__ void copy_f32_kernel(const float* __restrict__ src, int64_t n, float* __restrict__ dst) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = src[i];
}

__global__ void unpack_kernel(const uint32_t* __restrict__ bits, const __half* __restrict__ alpha16,
                              int64_t N, int64_t K, int64_t chunks, int8_t* __restrict__ sgn,
                              float* __restrict__ alpha) {
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx < N && alpha != nullptr) alpha[idx] = __half2float(alpha16[idx]);
    if (idx >= N * K) return;
    const int64_t n = idx / K, k = idx % K;
    const int64_t rt = n / BWLA_TILE_ROWS, kc = k / BWLA_CHUNK_COLS;
    const int i = (int)(n % BWLA_TILE_ROWS);
    const int kk = (int)(k % BWLA_CHUNK_COLS);
    const int g = kk >> 7, j = (kk >> 4) & 7, d = (kk >> 2) & 3, b = kk & 3;
    const int lane = g * 16 + i;
    const uint32_t w = bits[((rt * chunks + kc) * 64 + lane) * 4 + d];
    sgn[idx] = ((w >> (8 * b + j)) & 1u) ? 1 : -1;
}

}  // namespace

hipError_t bwla_launch_pack(const float* dW, const float* dR1, const float* dR2, const float* dU,
                            const float* dV, int64_t N, int64_t K, int n1, int n2, int r,
                            const bwla_layer_t* L, hipStream_t st) {
    // r = columns of dU and dV (the PSP rank); V has L->r columns (the layer's mode may add some)
    char* blob = (char*)L->d_blob;
    const int64_t chunks = bwla_chunks(K), rts = bwla_row_tiles(N);
    const int rpv = (L->r + 15) & ~15, rpu = (r + 15) & ~15;
    if (L->r > 0) {
        const int64_t nv = N * rpv;
        f32_to_f16_rows_kernel<<<dim3((unsigned)((nv + 255) / 256)), dim3(256), 0, st>>>(dV, N, r, rpv, (__half*)(blob + L->off_V));
    }
    if (r > 0) {
        const int64_t nu = K * rpu;
        u_pack_f16_kernel<<<dim3((unsigned)((nu + 255) / 256)), dim3(256), 0, st>>>(dU, K, r, rpu, (__half*)(blob + L->off_U));
    }
    if (L->mode != 0) {
        // columns behind the PSP ones: [asymmetric codes: 2][row shift: 1]
        const int asym_col = (L->mode & BWLA_MODE_ASYM_ACT) ? r : -1;
        const int mu_col = (L->mode & BWLA_MODE_ROW_SHIFT) ? L->r - 1 : -1;
        pack_rows_mode_kernel<<<dim3((unsigned)rts), dim3(256), 0, st>>>(
            dW, N, K, chunks, (uint32_t*)(blob + L->off_bits), (uint16_t*)(blob + L->off_alpha),
            (uint16_t*)(blob + L->off_V), rpv, mu_col, asym_col);
    } else {
        pack_bits_kernel<<<dim3((unsigned)(rts * chunks)), dim3(64), 0, st>>>(
            dW, N, K, chunks, (uint32_t*)(blob + L->off_bits));
        row_scale_kernel<<<dim3((unsigned)N), dim3(64), 0, st>>>(dW, N, K, (uint16_t*)(blob + L->off_alpha));
    }
    const int64_t e1 = (int64_t)n1 * n1, e2 = (int64_t)n2 * n2;
    copy_f32_kernel<<<dim3((unsigned)((e1 + 255) / 256)), dim3(256), 0, st>>>(dR1, e1, (float*)(blob + L->off_R1));
    copy_f32_kernel<<<dim3((unsigned)((e2 + 255) / 256)), dim3(256), 0, st>>>(dR2, e2, (float*)(blob + L->off_R2));
    const int p1 = ((n1 + 15) & ~15) * ((n1 + 31) & ~31), p2 = ((n2 + 15) & ~15) * ((n2 + 31) & ~31);
    factor_planes_kernel<<<dim3((unsigned)((p1 + 255) / 256)), dim3(256), 0, st>>>(dR1, n1, 1, (uint16_t*)(blob + L->off_R1p));
    factor_planes_kernel<<<dim3((unsigned)((p2 + 255) / 256)), dim3(256), 0, st>>>(dR2, n2, 0, (uint16_t*)(blob + L->off_R2p));
    if (L->off_Rd != 0) {
        const int nd = (int)(bwla_decode_planes_bytes(n1, n2) / 2);
        decode_planes_kernel<<<dim3((unsigned)((nd + 255) / 256)), dim3(256), 0, st>>>(
            dR1, dR2, n1, n2, bwla_decode_planes_r2_bytes(n1, n2) > 0 ? 1 : 0, (uint16_t*)(blob + L->off_Rd));
    }
    return hipGetLastError();
}

hipError_t bwla_launch_unpack(const bwla_layer_t* L, int8_t* d_sgn, float* d_alpha, hipStream_t st) {
    const char* blob = (const char*)L->d_blob;
    const int64_t total = L->N * L->K;
    unpack_kernel<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st>>>(
        (const uint32_t*)(blob + L->off_bits), (const __half*)(blob + L->off_alpha), L->N, L->K,
        bwla_chunks(L->K), d_sgn, d_alpha);
    return hipGetLastError();
}
