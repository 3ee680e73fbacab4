// Binary-weight GEMM for decode batches (M <= 16), bandwidth-bound: the sign bits stream from
// HBM exactly once, straight into registers, and are expanded there into INT8 MFMA operands.
//
//   acc[t,n] = sum_k q[t,k] Sign(W[n,k]) = 2 * sum_k q[t,k] b[n,k] - qsum_t,   b = sign bit
//   Y[t,n]   = scale_t * alpha_n * acc[t,n] + sum_j T[t,j] V[n,j]       (paper Eq. 4; Sec. 3.2)
//
// Bit expansion costs one VALU op per four weights: for the 16-byte word group w[0..3] of a
// lane, (w[d] & (0x01010101 << j)) is a run of int8 digits with value b * 2^j (j = 7 reads as
// -128).  The eight classes j accumulate in eight separate int32 tiles and are recombined by
// exact shifts once per output tile.  One 128-bit load per lane feeds eight 16x16x64 MFMAs.
#include "bwla_internal.h"

namespace {

constexpr int GD_MAX_WAVES = 8;

// q row-tile in LDS: rows x Kp bytes, 16-byte granules XOR-swizzled by row inside each 256-byte
// segment so that the 16 rows read by a wavefront fall into different banks without padding.
__device__ __forceinline__ int q_swz(int row, int kbyte, int Kp) {
    const int gran = kbyte >> 4;
    return row * Kp + (((gran & ~15) | ((gran ^ row) & 15)) << 4) + (kbyte & 15);
}

template <int NT>
__global__ __launch_bounds__(64 * GD_MAX_WAVES) void gemm_decode_kernel(
    const uint4* __restrict__ bits, int chunks, int row_tiles, const int8_t* __restrict__ q, int M, int K,
    const float* __restrict__ scale, const int32_t* __restrict__ qsum, const __half* __restrict__ alpha,
    const __half* __restrict__ V, const float* __restrict__ T, int r, float* __restrict__ Y, int N,
    int32_t* __restrict__ acc_out, int ksplit, int wn_count) {
    extern __shared__ __align__(16) char smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 15, lg = lane >> 4;
    const int Kp = chunks * BWLA_CHUNK_COLS;
    const int rows = M < 16 ? M : 16;
    const int kw = wave % ksplit, wn = wave / ksplit;

    const int tile0 = (blockIdx.x * wn_count + wn) * NT;      // first 16-row tile of this wave

    // ---- issue the first weight loads before anything else (they do not depend on LDS)
    v4i wcur[NT], wnext[NT];
    int c = kw;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        wcur[nt] = v4i{0, 0, 0, 0};
        if (c < chunks && tile0 + nt < row_tiles) {
            const uint4 u = bits[((int64_t)(tile0 + nt) * chunks + c) * 64 + lane];
            wcur[nt] = v4i{(int)u.x, (int)u.y, (int)u.z, (int)u.w};
        }
    }

    // ---- stage the code rows into LDS (zero beyond K)
    {
        const int gran_per_row = Kp >> 4;
        const int total = rows * gran_per_row;
        for (int idx = tid; idx < total; idx += blockDim.x) {
            const int row = idx / gran_per_row, gcol = idx - row * gran_per_row;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (gcol * 16 < K) v = *reinterpret_cast<const uint4*>(q + (int64_t)row * K + gcol * 16);
            *reinterpret_cast<uint4*>(smem + q_swz(row, gcol * 16, Kp)) = v;
        }
    }
    __syncthreads();

    v4i acc[NT][8];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[nt][j] = v4i{0, 0, 0, 0};

    const int brow = li < rows ? li : rows - 1;    // padded token columns repeat the last row; never stored

    for (; c < chunks; c += ksplit) {
        const int cn = c + ksplit;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            wnext[nt] = v4i{0, 0, 0, 0};
            if (cn < chunks && tile0 + nt < row_tiles) {
                const uint4 u = bits[((int64_t)(tile0 + nt) * chunks + cn) * 64 + lane];
                wnext[nt] = v4i{(int)u.x, (int)u.y, (int)u.z, (int)u.w};
            }
        }
        v4i b[8];
#pragma unroll
        for (int j = 0; j < 8; ++j)
            b[j] = *reinterpret_cast<const v4i*>(smem + q_swz(brow, c * BWLA_CHUNK_COLS + lg * 128 + j * 16, Kp));
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int m = 0x01010101 << j;
                const v4i a = v4i{wcur[nt].x & m, wcur[nt].y & m, wcur[nt].z & m, wcur[nt].w & m};
                acc[nt][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b[j], acc[nt][j], 0, 0, 0);
            }
        }
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) wcur[nt] = wnext[nt];
    }

    // ---- recombine the eight digit classes: sum_j acc_j / 2^j, class 7 carries weight -128
    v4i res[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        v4i s = v4i{0, 0, 0, 0};
#pragma unroll
        for (int j = 0; j < 7; ++j) s += acc[nt][j] << (7 - j);
        s -= acc[nt][7];
        res[nt] = s >> 7;
    }

    // ---- add the K-slices of the ksplit waves that share these output tiles
    if (ksplit > 1) {
        __syncthreads();                               // everyone is done with the code tile
        v4i* red = reinterpret_cast<v4i*>(smem);       // [wn][kw][nt][lane]
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) red[((wn * ksplit + kw) * NT + nt) * 64 + lane] = res[nt];
        __syncthreads();
        if (kw != 0) return;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
            for (int k2 = 1; k2 < ksplit; ++k2) res[nt] += red[((wn * ksplit + k2) * NT + nt) * 64 + lane];
    }

    // ---- epilogue: lane holds token li, output rows n = 16*tile + 4*lg + v
    const int t = li;
    const bool tok_ok = t < M;
    const float st = tok_ok ? scale[t] : 0.0f;
    const int qs = tok_ok ? qsum[t] : 0;
    const int JT = (r + 15) >> 4;
    const int rp = JT * 16;                            // V rows are stored padded to rp halfs
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int tile = tile0 + nt;
        if (tile >= row_tiles) continue;
        const int n0 = tile * 16;
        // low-rank term on fp32 MFMA: D[n][t] = sum_j V[n][j] T[t][j]; lane (li, lg) feeds
        // j = 16u + 4*lg + e in step e of group u for both operands
        v4f low = v4f{0.f, 0.f, 0.f, 0.f};
        for (int u = 0; u < JT; ++u) {
            const int j0 = u * 16 + 4 * lg;
            const int vrow = n0 + li;
            float vv[4] = {0.f, 0.f, 0.f, 0.f}, tv[4] = {0.f, 0.f, 0.f, 0.f};
            if (vrow < N) {
                const uint2 raw = *reinterpret_cast<const uint2*>(V + (int64_t)vrow * rp + j0);
                const __half2 h0 = *reinterpret_cast<const __half2*>(&raw.x);
                const __half2 h1 = *reinterpret_cast<const __half2*>(&raw.y);
                vv[0] = __low2float(h0); vv[1] = __high2float(h0);
                vv[2] = __low2float(h1); vv[3] = __high2float(h1);
            }
            if (tok_ok) {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (j0 + e < r) tv[e] = T[(int64_t)t * r + j0 + e];
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) low = __builtin_amdgcn_mfma_f32_16x16x4f32(vv[e], tv[e], low, 0, 0, 0);
        }
        if (!tok_ok) continue;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int n = n0 + 4 * lg + v;
            if (n < N) {
                const int a = 2 * res[nt][v] - qs;
                const float al = __half2float(alpha[n]);
                Y[(int64_t)t * N + n] = st * al * (float)a + low[v];
                if (acc_out) acc_out[(int64_t)t * N + n] = a;
            }
        }
    }
}

}  // namespace

hipError_t bwla_launch_gemm_decode(const bwla_layer_t* L, const int8_t* dq, const float* dscale,
                                   const int32_t* dqsum, const float* dT, int64_t M, float* dY,
                                   int32_t* dacc, hipStream_t st) {
    const char* blob = (const char*)L->d_blob;
    const int chunks = (int)bwla_chunks(L->K), row_tiles = (int)bwla_row_tiles(L->N);
    const int rows = M < 16 ? (int)M : 16;
    // waves of a workgroup: ksplit along K x wn along N
    int ksplit = 1;
    while (ksplit * 2 <= 8 && chunks % (ksplit * 2) == 0) ksplit *= 2;
    if (chunks >= 8 && ksplit < 2) ksplit = 2;
    int wn = GD_MAX_WAVES / ksplit;
    const int NT = 1;
    // keep at least ~2 workgroups per CU when the layer is small
    while (wn > 1 && (row_tiles + wn * NT - 1) / (wn * NT) < 512) wn >>= 1;
    const int waves = ksplit * wn;
    const int groups = (row_tiles + wn * NT - 1) / (wn * NT);
    size_t lds = (size_t)rows * chunks * BWLA_CHUNK_COLS;
    const size_t red = (size_t)waves * NT * 64 * 16;
    if (lds < red) lds = red;
    hipError_t e = bwla_ensure_lds((const void*)gemm_decode_kernel<1>, lds);
    if (e != hipSuccess) return e;
    gemm_decode_kernel<1><<<dim3((unsigned)groups), dim3(64 * waves), lds, st>>>(
        (const uint4*)(blob + L->off_bits), chunks, row_tiles, dq, (int)M, (int)L->K, dscale, dqsum,
        (const __half*)(blob + L->off_alpha), (const __half*)(blob + L->off_V), dT, L->r, dY, (int)L->N, dacc,
        ksplit, wn);
    return hipGetLastError();
}

size_t bwla_gemm_decode_lds(int64_t M, int64_t K) {
    const int rows = M < 16 ? (int)M : 16;
    return (size_t)rows * bwla_chunks(K) * BWLA_CHUNK_COLS;
}
