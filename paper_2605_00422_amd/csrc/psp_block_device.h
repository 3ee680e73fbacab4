// PSP projection T = X U for up to 16 tokens per workgroup (rides in the rotation launch).
#pragma once
#include "rotate_common.h"

namespace {

// Sum of the S partial tiles of token tile tt, in slice order, into T (all threads of the workgroup).
__device__ __forceinline__ void psp_sum_partials(const float* __restrict__ partials, float* __restrict__ T, int64_t M,
                                                 int r, int S, int tt, int tp) {
    const int rp = ((r + 15) >> 4) * 16;
    const int rows = M - (int64_t)tt * 16 < 16 ? (int)(M - (int64_t)tt * 16) : 16;
    for (int idx = threadIdx.x; idx < rows * rp; idx += (int)blockDim.x) {
        const int row = idx / rp, col = idx - row * rp;
        const int64_t tok = (int64_t)tt * 16 + row;
        if (col < r) {
            // batches of sixteen loads in flight; slices past S re-read the last one and add zero
            float sum = 0.0f;
            for (int ss = 0; ss < S; ss += 16) {
                float v[16];
#pragma unroll
                for (int u = 0; u < 16; ++u) {
                    const int sc = ss + u < S ? ss + u : S - 1;
                    v[u] = bwla_load_agent(&partials[(((int64_t)tt * S + sc) * 16 + row) * rp + col]);
                }
#pragma unroll
                for (int u = 0; u < 16; ++u) sum += ss + u < S ? v[u] : 0.0f;
            }
            T[tok * tp + col] = sum;
        }
    }
}

// ================================================================== PSP projection T = X U
// A workgroup takes 16 tokens, one 512-column slice of K and up to PP_GROUPJT 16-column tiles of
// the rank (group jg of JG): the fp32 MFMAs of a wavefront grow with the tiles it carries (six
// tiles: 96 of them, 1.3 us), so wide ranks are dealt to more workgroups.
// finish = false: with more than one slice the workgroup only leaves its partial tile; a later
// launch adds them up (psp_sum_partials) and the arrival counters are not touched.
template <bool BF16>
__device__ __forceinline__ void psp_block(char* smem, const void* __restrict__ X, int64_t M, int64_t K, int r,
                                          const __half* __restrict__ U, float* __restrict__ T,
                                          int* __restrict__ counters, float* __restrict__ partials, int S, int tt,
                                          int s, int tp, bool finish = true, int jg = 0, int JG = 1) {
    __shared__ int is_last;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nw = (int)(blockDim.x >> 6);             // the eight 64-column parts of a slice are dealt to nw waves
    const int li = lane & 15, lg = lane >> 4;
    const int JTall = (r + 15) >> 4, rp = JTall * 16;
    const int jt0 = JG > 1 ? jg * PP_GROUPJT : 0;                      // my tiles: jt0 .. jt0 + JT - 1
    const int JT = JG > 1 ? (JTall - jt0 < PP_GROUPJT ? JTall - jt0 : PP_GROUPJT) : JTall;
    const int64_t kbase = (int64_t)s * PP_SLICE;

    // wave w takes columns [64w, 64w+64) of the slice in 4 groups of 16: lane (li, lg) owns
    // k = 16*g + 4*lg + e, e = 0..3 -- of token li as MFMA operand A, of column jt*16 + li of U as
    // operand B (8 contiguous bytes of the packed U).  All loads are issued before the first use.
    int64_t trow = (int64_t)tt * 16 + li;
    if (trow > M - 1) trow = M - 1;                    // padded token rows are never stored
    v4f acc[PP_MAXJT];
#pragma unroll
    for (int jt = 0; jt < PP_MAXJT; ++jt) acc[jt] = v4f{0.f, 0.f, 0.f, 0.f};
    for (int part = wave; part < 8; part += nw) {
    float x[4][4];
    uint2 u[4][PP_MAXJT];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const int64_t kx = kbase + part * 64 + g * 16 + 4 * lg;
        const bool in = kx < K;
        const int64_t kc = in ? kx : K - 4;            // keep the address valid, zero the value
        if (BF16) {
            const uint2 raw = *reinterpret_cast<const uint2*>(reinterpret_cast<const uint16_t*>(X) + trow * K + kc);
            x[g][0] = __uint_as_float(raw.x << 16); x[g][1] = __uint_as_float(raw.x & 0xffff0000u);
            x[g][2] = __uint_as_float(raw.y << 16); x[g][3] = __uint_as_float(raw.y & 0xffff0000u);
        } else {
            const float4 raw = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(X) + trow * K + kc);
            x[g][0] = raw.x; x[g][1] = raw.y; x[g][2] = raw.z; x[g][3] = raw.w;
        }
        if (!in) x[g][0] = x[g][1] = x[g][2] = x[g][3] = 0.0f;
#pragma unroll
        for (int jt = 0; jt < PP_MAXJT; ++jt)
            // (packed U: 1 KiB blocks [column tile][step of 32 rows], lane (li, k / 8 within the step), 8 values)
            if (jt < JT)
                u[g][jt] = *reinterpret_cast<const uint2*>(U + ((int64_t)(jt0 + jt) * (K >> 5) + (kc >> 5)) * 512 +
                                                           ((((int)kc & 31) >> 3) * 16 + li) * 8 + ((int)kc & 7));
    }

#pragma unroll
    for (int g = 0; g < 4; ++g) {
#pragma unroll
        for (int jt = 0; jt < PP_MAXJT; ++jt) {
            if (jt < JT) {
                const __half2 h01 = *reinterpret_cast<const __half2*>(&u[g][jt].x);
                const __half2 h23 = *reinterpret_cast<const __half2*>(&u[g][jt].y);
                const float2 f01 = __half22float2(h01), f23 = __half22float2(h23);
                acc[jt] = __builtin_amdgcn_mfma_f32_16x16x4f32(x[g][0], f01.x, acc[jt], 0, 0, 0);
                acc[jt] = __builtin_amdgcn_mfma_f32_16x16x4f32(x[g][1], f01.y, acc[jt], 0, 0, 0);
                acc[jt] = __builtin_amdgcn_mfma_f32_16x16x4f32(x[g][2], f23.x, acc[jt], 0, 0, 0);
                acc[jt] = __builtin_amdgcn_mfma_f32_16x16x4f32(x[g][3], f23.y, acc[jt], 0, 0, 0);
            }
        }
    }
    }
    v4f* red = reinterpret_cast<v4f*>(smem);           // [wave][jt][lane]
#pragma unroll
    for (int jt = 0; jt < PP_MAXJT; ++jt)
        if (jt < JT) red[(wave * JT + jt) * 64 + lane] = acc[jt];
    __syncthreads();
    // waves share the column tiles; lane holds tokens 4*lg + v, column jt*16 + li
    for (int jt = wave; jt < JT; jt += nw) {
        v4f sum = red[jt * 64 + lane];
        for (int w = 1; w < nw; ++w) sum += red[(w * JT + jt) * 64 + lane];
        const int col = (jt0 + jt) * 16 + li;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int row = 4 * lg + v;
            const int64_t tok = (int64_t)tt * 16 + row;
            if (S == 1) {
                if (tok < M && col < r) T[tok * tp + col] = sum[v];
            } else {
                bwla_store_agent(&partials[(((int64_t)tt * S + s) * 16 + row) * rp + col], sum[v]);
            }
        }
    }
    if (S == 1 || !finish) return;

    if (!bwla_partials_arrive(&counters[tt], S * JG, &is_last)) return;
    // last workgroup of this token tile: add the S partial tiles in slice order
    psp_sum_partials(partials, T, M, r, S, tt, tp);
    if (tid == 0) counters[tt] = 0;                    // leave the scratch as it was found
}

}  // namespace
