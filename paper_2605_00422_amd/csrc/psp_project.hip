// PSP branch, first half: T = X U (M x r), fp32 accumulation on fp32 MFMA, from the original
// (un-rotated, un-quantized) activations (paper Sec. 3.2: the low-rank residual M = A B lives in
// the un-rotated coordinates; here U = B^T).
//
// Work split: token tiles of 16 x S slices of K.  With S > 1 every block writes its partial
// tile to scratch and the block that arrives last adds the S partials in slice order, so the
// result does not depend on timing.
#include "bwla_internal.h"

namespace {

constexpr int PP_THREADS = 256;
constexpr int PP_WAVES = 4;
constexpr int PP_MAXJT = BWLA_MAX_RANK / 16;   // 8 column tiles of 16

template <bool BF16>
__global__ __launch_bounds__(PP_THREADS) void psp_project_kernel(
    const void* __restrict__ X, int64_t M, int64_t K, int r, const __half* __restrict__ U,
    float* __restrict__ T, int* __restrict__ counters, float* __restrict__ partials, int S, int kps) {
    __shared__ float red[PP_WAVES][PP_MAXJT][64][4];
    __shared__ int is_last;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 15, lg = lane >> 4;
    const int tt = blockIdx.x, s = blockIdx.y;
    const int JT = (r + 15) >> 4;
    const int rp = JT * 16;

    int64_t trow = (int64_t)tt * 16 + li;
    if (trow > M - 1) trow = M - 1;                    // clamp: padded token rows are never stored
    const int64_t kbeg = (int64_t)s * kps;
    int64_t kend = kbeg + kps;
    if (kend > K) kend = K;

    v4f acc[PP_MAXJT];
#pragma unroll
    for (int jt = 0; jt < PP_MAXJT; ++jt) acc[jt] = v4f{0.f, 0.f, 0.f, 0.f};

    // 16-column groups of K, interleaved over the four waves; lane (li, lg) owns columns
    // k0 + 4*lg + e, e = 0..3 of its token in MFMA step e (any fixed order of the contraction
    // index is valid as long as both operands use it)
    for (int64_t k0 = kbeg + wave * 16; k0 < kend; k0 += PP_WAVES * 16) {
        float x[4];
        const int64_t kx = k0 + 4 * lg;
        if (BF16) {
            const uint2 raw = *reinterpret_cast<const uint2*>(reinterpret_cast<const uint16_t*>(X) + trow * K + kx);
            x[0] = __uint_as_float(raw.x << 16);
            x[1] = __uint_as_float(raw.x & 0xffff0000u);
            x[2] = __uint_as_float(raw.y << 16);
            x[3] = __uint_as_float(raw.y & 0xffff0000u);
        } else {
            const float4 raw = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(X) + trow * K + kx);
            x[0] = raw.x; x[1] = raw.y; x[2] = raw.z; x[3] = raw.w;
        }
#pragma unroll
        for (int jt = 0; jt < PP_MAXJT; ++jt) {
            if (jt < JT) {
                const int col = jt * 16 + li;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float u = __half2float(U[(kx + e) * rp + col]);   // rows padded to rp with zeros
                    acc[jt] = __builtin_amdgcn_mfma_f32_16x16x4f32(x[e], u, acc[jt], 0, 0, 0);
                }
            }
        }
    }

#pragma unroll
    for (int jt = 0; jt < PP_MAXJT; ++jt)
        if (jt < JT) {
#pragma unroll
            for (int v = 0; v < 4; ++v) red[wave][jt][lane][v] = acc[jt][v];
        }
    __syncthreads();

    // wave 0 adds the four waves; lane holds rows 4*lg + v (tokens), column jt*16 + li
    if (wave == 0) {
#pragma unroll
        for (int jt = 0; jt < PP_MAXJT; ++jt) {
            if (jt < JT) {
                const int col = jt * 16 + li;
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const float sum = (red[0][jt][lane][v] + red[1][jt][lane][v]) +
                                      (red[2][jt][lane][v] + red[3][jt][lane][v]);
                    const int row = 4 * lg + v;
                    const int64_t tok = (int64_t)tt * 16 + row;
                    if (S == 1) {
                        if (tok < M && col < r) T[tok * r + col] = sum;
                    } else {
                        partials[(((int64_t)tt * S + s) * 16 + row) * rp + col] = sum;
                    }
                }
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
    // last block of this token tile: add the S partial tiles in slice order
    for (int idx = tid; idx < 16 * rp; idx += PP_THREADS) {
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

}  // namespace

bwla_psp_plan bwla_make_psp_plan(int64_t M, int64_t K, int r) {
    bwla_psp_plan p;
    p.token_tiles = (int)((M + 15) / 16);
    if (r <= 0) { p.splits = 1; p.k_per_split = (int)((K + 63) / 64 * 64); return p; }
    int64_t S = 512 / p.token_tiles;
    const int64_t smax = (K + 255) / 256;
    if (S > smax) S = smax;
    if (S < 1) S = 1;
    int64_t kps = ((K + S - 1) / S + 63) / 64 * 64;
    S = (K + kps - 1) / kps;
    p.splits = (int)S;
    p.k_per_split = (int)kps;
    return p;
}

hipError_t bwla_launch_psp_project(const bwla_layer_t* L, const void* dX, int xdtype, int64_t M,
                                   float* dT, void* dws, const bwla_psp_plan& plan, hipStream_t st) {
    const char* blob = (const char*)L->d_blob;
    const __half* U = (const __half*)(blob + L->off_U);
    int* counters = (int*)dws;
    float* partials = dws ? (float*)((char*)dws + bwla_align256((uint64_t)plan.token_tiles * sizeof(int))) : nullptr;
    dim3 grid((unsigned)plan.token_tiles, (unsigned)plan.splits);
    if (xdtype == BWLA_X_BF16)
        psp_project_kernel<true><<<grid, dim3(PP_THREADS), 0, st>>>(dX, M, L->K, L->r, U, dT, counters, partials,
                                                                   plan.splits, plan.k_per_split);
    else
        psp_project_kernel<false><<<grid, dim3(PP_THREADS), 0, st>>>(dX, M, L->K, L->r, U, dT, counters, partials,
                                                                    plan.splits, plan.k_per_split);
    return hipGetLastError();
}
