// Binary-weight GEMM for token batches (M > 16): a dense int8 contraction on 32x32x32 INT8
// MFMA with exact int32 accumulation.
//
//   acc[t,n] = sum_k q[t,k] Sign(W[n,k]) = 2 * sum_k q[t,k] b[n,k] - qsum_t
//   Y[t,n]   = scale_t * alpha_n * acc[t,n] + sum_j T[t,j] V[n,j]       (paper Eq. 4; Sec. 3.2)
//
// The activation codes are tiled through LDS (double buffered); the 1-bit weights never touch
// LDS: each lane keeps the 128-column bit slice of its own output channel in four registers and
// expands a 16-column run with (w >> j) & 0x01010101 right before the MFMA that consumes it.
#include "bwla_internal.h"

namespace {

constexpr int GP_BK = 128;           // columns per main-loop step = one 16-byte bit slice per row
constexpr int GP_LDA = GP_BK + 16;   // LDS row pitch of the code tile (bytes)

template <int MT, int NTL, int WM, int WN>
__global__ __launch_bounds__(64 * WM * WN) void gemm_prefill_kernel(
    const uint4* __restrict__ bits, int chunks, int row_tiles, const int8_t* __restrict__ q, int M, int K,
    const float* __restrict__ scale, const int32_t* __restrict__ qsum, const __half* __restrict__ alpha,
    const __half* __restrict__ V, const float* __restrict__ T, int r, float* __restrict__ Y, int N,
    int32_t* __restrict__ acc_out, int tiles_m, int tiles_n) {
    constexpr int THREADS = 64 * WM * WN;
    constexpr int BM = WM * MT * 32;
    constexpr int BN = WN * NTL * 32;
    constexpr int PIECES = BM * (GP_BK / 16) / THREADS;     // 16-byte granules of the A tile per thread
    static_assert(BM * (GP_BK / 16) % THREADS == 0, "tile fill must divide evenly");
    extern __shared__ __align__(16) char smem[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, lg = lane >> 5;
    const int wm = wave % WM, wn = wave / WM;

    // XCD-aware tile order: workgroups are dealt round-robin to the 8 XCDs, so give each XCD a
    // contiguous run of tiles (same token rows -> the code tile is shared in that XCD's L2)
    int pid = blockIdx.x;
    const int nblocks = gridDim.x;
    if ((nblocks & 7) == 0) pid = (pid & 7) * (nblocks >> 3) + (pid >> 3);
    const int tm = pid / tiles_n, tn = pid - tm * tiles_n;
    const int m_base = tm * BM, n_base = tn * BN;

    const int nslices = (K + GP_BK - 1) / GP_BK;

    // ---- A tile fill helpers
    uint4 areg[PIECES];
    auto a_fetch = [&](int ks) {
#pragma unroll
        for (int p = 0; p < PIECES; ++p) {
            const int idx = tid + p * THREADS;
            const int row = idx >> 3, gcol = idx & 7;
            const int m = m_base + row, k = ks * GP_BK + gcol * 16;
            areg[p] = make_uint4(0, 0, 0, 0);
            if (m < M && k < K) areg[p] = *reinterpret_cast<const uint4*>(q + (int64_t)m * K + k);
        }
    };
    auto a_store = [&](int buf) {
        char* dst = smem + buf * (BM * GP_LDA);
#pragma unroll
        for (int p = 0; p < PIECES; ++p) {
            const int idx = tid + p * THREADS;
            const int row = idx >> 3, gcol = idx & 7;
            *reinterpret_cast<uint4*>(dst + row * GP_LDA + gcol * 16) = areg[p];
        }
    };
    // ---- weight slice of this lane's output channels
    v4i wcur[NTL], wnext[NTL];
    auto w_fetch = [&](int ks, v4i (&w)[NTL]) {
#pragma unroll
        for (int nt = 0; nt < NTL; ++nt) {
            const int row = n_base + (wn * NTL + nt) * 32 + l32;
            const int rt = row >> 4;
            w[nt] = v4i{0, 0, 0, 0};
            if (rt < row_tiles) {
                const uint4 u = bits[((int64_t)rt * chunks + (ks >> 2)) * 64 + (ks & 3) * 16 + (row & 15)];
                w[nt] = v4i{(int)u.x, (int)u.y, (int)u.z, (int)u.w};
            }
        }
    };

    v16i acc[MT][NTL];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NTL; ++nt)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mt][nt][v] = 0;

    a_fetch(0);
    w_fetch(0, wcur);
    a_store(0);
    __syncthreads();

    for (int ks = 0; ks < nslices; ++ks) {
        const bool more = ks + 1 < nslices;
        if (more) {
            a_fetch(ks + 1);
            w_fetch(ks + 1, wnext);
        }
        const char* As = smem + (ks & 1) * (BM * GP_LDA) + (wm * MT * 32 + l32) * GP_LDA + lg * 16;
        // lane half lg consumes 16-column group 2*s + lg in step s (both operands use this order)
        v4i ws[NTL];
#pragma unroll
        for (int nt = 0; nt < NTL; ++nt) ws[nt] = wcur[nt] >> lg;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            v4i a[MT], b[NTL];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) a[mt] = *reinterpret_cast<const v4i*>(As + mt * 32 * GP_LDA + s * 32);
#pragma unroll
            for (int nt = 0; nt < NTL; ++nt) b[nt] = (ws[nt] >> (2 * s)) & 0x01010101;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int nt = 0; nt < NTL; ++nt)
                    acc[mt][nt] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[mt], b[nt], acc[mt][nt], 0, 0, 0);
        }
        if (more) a_store((ks + 1) & 1);
        __syncthreads();
#pragma unroll
        for (int nt = 0; nt < NTL; ++nt) wcur[nt] = wnext[nt];
    }

    // ---- epilogue.  Accumulator element v of lane (l32, lg): row 8*(v/4) + 4*lg + v%4, column l32.
    const int JT = (r + 15) >> 4;
    const int rp = JT * 16;
    const int half = rp >> 1;                          // lane half lg feeds j in [lg*half, lg*half + half)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int mrow0 = m_base + (wm * MT + mt) * 32;
        if (mrow0 >= M) continue;
#pragma unroll
        for (int nt = 0; nt < NTL; ++nt) {
            const int n = n_base + (wn * NTL + nt) * 32 + l32;
            if (n_base + (wn * NTL + nt) * 32 >= N) continue;
            v16f low;
#pragma unroll
            for (int v = 0; v < 16; ++v) low[v] = 0.0f;
            // low-rank term on fp32 MFMA: D[m][n] = sum_j T[m][j] V[n][j]
            {
                const int tm_row = mrow0 + l32;
                const float* trow = T + (int64_t)tm_row * r;
                const __half* vrow = V + (int64_t)n * rp;
                for (int p = 0; p < half; ++p) {
                    const int j = lg * half + p;
                    const float tv = (tm_row < M && j < r) ? trow[j] : 0.0f;
                    const float vv = (n < N) ? __half2float(vrow[j]) : 0.0f;
                    low = __builtin_amdgcn_mfma_f32_32x32x2f32(tv, vv, low, 0, 0, 0);
                }
            }
            const float al = (n < N) ? __half2float(alpha[n]) : 0.0f;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = mrow0 + 8 * (v >> 2) + 4 * lg + (v & 3);
                if (m < M && n < N) {
                    const int a = 2 * acc[mt][nt][v] - qsum[m];
                    Y[(int64_t)m * N + n] = scale[m] * al * (float)a + low[v];
                    if (acc_out) acc_out[(int64_t)m * N + n] = a;
                }
            }
        }
    }
}

template <int MT, int NTL, int WM, int WN>
hipError_t launch_cfg(const bwla_layer_t* L, const int8_t* dq, const float* dscale, const int32_t* dqsum,
                      const float* dT, int64_t M, float* dY, int32_t* dacc, hipStream_t st) {
    constexpr int BM = WM * MT * 32, BN = WN * NTL * 32;
    const char* blob = (const char*)L->d_blob;
    const int tiles_m = (int)((M + BM - 1) / BM), tiles_n = (int)((L->N + BN - 1) / BN);
    const size_t lds = 2 * (size_t)BM * GP_LDA;
    auto kern = gemm_prefill_kernel<MT, NTL, WM, WN>;
    static bwla_lds_attr attr;
    hipError_t e = attr.ensure((const void*)kern, lds);
    if (e != hipSuccess) return e;
    kern<<<dim3((unsigned)(tiles_m * tiles_n)), dim3(64 * WM * WN), lds, st>>>(
        (const uint4*)(blob + L->off_bits), (int)bwla_chunks(L->K), (int)bwla_row_tiles(L->N), dq, (int)M,
        (int)L->K, dscale, dqsum, (const __half*)(blob + L->off_alpha), (const __half*)(blob + L->off_V), dT,
        L->r, dY, (int)L->N, dacc, tiles_m, tiles_n);
    return hipGetLastError();
}

inline int64_t tiles_for(int64_t M, int64_t N, int BM, int BN) { return ((M + BM - 1) / BM) * ((N + BN - 1) / BN); }

// fraction of the chip kept busy by `tiles` equal workgroups on 256 CUs (last round may be ragged)
inline double wave_eff(int64_t tiles) {
    const int64_t rounds = (tiles + 255) / 256;
    return (double)tiles / (double)(rounds * 256);
}

}  // namespace

hipError_t bwla_launch_gemm_prefill(const bwla_layer_t* L, const int8_t* dq, const float* dscale,
                                    const int32_t* dqsum, const float* dT, int64_t M, float* dY,
                                    int32_t* dacc, hipStream_t st) {
    const int64_t N = L->N;
    if (M <= 64) return launch_cfg<1, 2, 2, 2>(L, dq, dscale, dqsum, dT, M, dY, dacc, st);          // 64 x 128
    // pick the largest tile that still fills the chip reasonably
    const double e256 = wave_eff(tiles_for(M, N, 256, 256));
    const double e160 = wave_eff(tiles_for(M, N, 256, 160));
    const double e128 = wave_eff(tiles_for(M, N, 128, 128)) * 0.85;   // smaller tile: more LDS traffic per MFMA
    if (e256 >= e160 && e256 >= e128) return launch_cfg<4, 4, 2, 2>(L, dq, dscale, dqsum, dT, M, dY, dacc, st);
    if (e160 >= e128) return launch_cfg<2, 5, 4, 1>(L, dq, dscale, dqsum, dT, M, dY, dacc, st);      // 256 x 160
    return launch_cfg<2, 2, 2, 2>(L, dq, dscale, dqsum, dT, M, dY, dacc, st);                        // 128 x 128
}
