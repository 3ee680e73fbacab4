// PSP projection T = X U for many tokens: first factor of the rank-r side branch
// (X U) V^T that carries the low-rank part of the weight (paper Sec. 3.2).
//
// The product is tall and thin (M x K times K x r with r <= 128), so it is bound by streaming X
// once.  Both MFMA operands come straight from global memory as 16-byte vectors along K:
//   A  activations, row-major [M][K]; bf16 inputs are used as they are, fp32 inputs are split
//      into three bf16 terms (8 + 8 + 8 mantissa bits, exact)
//   B  the packed U, fp16 in MFMA operand order (one contiguous KiB per 16 columns x 32 rows); a
//      fragment is split in registers into two bf16 terms whose sum is the fp16 value exactly
//      (8 + 3 mantissa bits)
// so every product is exact and only the fp32 accumulation rounds.  A workgroup owns 64 tokens
// x up to 64 columns x one slice of K; its four wavefronts split the slice, add their tiles
// through LDS and either store T (one slice) or write a partial tile to scratch, where the
// workgroup that arrives last adds the partials in slice order (deterministic).
#include "bwla_internal.h"

namespace {

constexpr int PF_THREADS = 256;
constexpr int PF_WAVES = 4;
constexpr int PF_TM = 64;                 // tokens per workgroup
constexpr int PF_MT = PF_TM / 16;
constexpr int PF_KSTEP = 32;              // K per bf16 MFMA

typedef __attribute__((ext_vector_type(8))) __bf16 v8bf;

struct PfArgs {
    const void* X; int64_t M, K; int r, rp;   // r = rank of the projection (columns of U)
    int tp;                               // row pitch of T (r, or r + 1 for a layer with row shifts)
    const __half* Ut;                     // packed U: [rp / 16][K / 32][64 lanes][8] fp16
    float* T; int* counters; float* partials;
    int S, JG, kslice;
};

template <bool BF16> struct AFrag;
template <> struct AFrag<true> { uint4 v[PF_MT]; };
template <> struct AFrag<false> { float4 v[PF_MT][2]; };
template <bool BF16, int NJT> struct Frag { AFrag<BF16> a; uint4 b[NJT]; };

template <bool BF16, int NJT>
__device__ __forceinline__ void pf_load(Frag<BF16, NJT>& f, const void* __restrict__ X, const int64_t (&xoff)[PF_MT],
                                        const __half* __restrict__ Ut, const int64_t (&uoff)[NJT], int64_t kb) {
#pragma unroll
    for (int mt = 0; mt < PF_MT; ++mt) {
        if constexpr (BF16) {
            f.a.v[mt] = *reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(X) + xoff[mt] + kb);
        } else {
            const float* p = reinterpret_cast<const float*>(X) + xoff[mt] + kb;
            f.a.v[mt][0] = *reinterpret_cast<const float4*>(p);
            f.a.v[mt][1] = *reinterpret_cast<const float4*>(p + 4);
        }
    }
#pragma unroll
    for (int jt = 0; jt < NJT; ++jt) f.b[jt] = *reinterpret_cast<const uint4*>(Ut + uoff[jt] + kb * 16);
}

// eight fp16 values -> hi + lo, both bf16: hi = bf16(u) rounded to nearest, lo = u - hi (exact)
__device__ __forceinline__ void split_u(const uint4& raw, v8bf& hi, v8bf& lo) {
    const __half2* h2 = reinterpret_cast<const __half2*>(&raw);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const float2 f = __half22float2(h2[e]);
        const __bf16 h0 = (__bf16)f.x, h1 = (__bf16)f.y;
        hi[2 * e] = h0; hi[2 * e + 1] = h1;
        lo[2 * e] = (__bf16)(f.x - (float)h0); lo[2 * e + 1] = (__bf16)(f.y - (float)h1);
    }
}

// x = h1 + h2 + h3 exactly, each term a bf16 (round to nearest, remainders are exact in fp32)
__device__ __forceinline__ void split3(float x, __bf16& h1, __bf16& h2, __bf16& h3) {
    h1 = (__bf16)x;
    const float r1 = x - (float)h1;
    h2 = (__bf16)r1;
    const float r2 = r1 - (float)h2;
    h3 = (__bf16)r2;
}

template <bool BF16, int NJT>
__device__ __forceinline__ void pf_compute(const Frag<BF16, NJT>& f, bool valid, v4f (&acc)[PF_MT][NJT]) {
    v8bf bh[NJT], bl[NJT];
#pragma unroll
    for (int jt = 0; jt < NJT; ++jt) split_u(f.b[jt], bh[jt], bl[jt]);
#pragma unroll
    for (int mt = 0; mt < PF_MT; ++mt) {
        if constexpr (BF16) {
            uint4 av = f.a.v[mt];
            if (!valid) av = make_uint4(0, 0, 0, 0);
            const v8bf a = __builtin_bit_cast(v8bf, av);
#pragma unroll
            for (int jt = 0; jt < NJT; ++jt) {
                acc[mt][jt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, bl[jt], acc[mt][jt], 0, 0, 0);
                acc[mt][jt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, bh[jt], acc[mt][jt], 0, 0, 0);
            }
        } else {
            const float x[8] = {f.a.v[mt][0].x, f.a.v[mt][0].y, f.a.v[mt][0].z, f.a.v[mt][0].w,
                                f.a.v[mt][1].x, f.a.v[mt][1].y, f.a.v[mt][1].z, f.a.v[mt][1].w};
            v8bf a1, a2, a3;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                __bf16 h1, h2, h3;
                split3(valid ? x[e] : 0.0f, h1, h2, h3);
                a1[e] = h1; a2[e] = h2; a3[e] = h3;
            }
#pragma unroll
            for (int jt = 0; jt < NJT; ++jt) {
#pragma unroll
                for (int p = 0; p < 2; ++p) {
                    const v8bf b = p == 0 ? bl[jt] : bh[jt];
                    acc[mt][jt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a3, b, acc[mt][jt], 0, 0, 0);
                    acc[mt][jt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a2, b, acc[mt][jt], 0, 0, 0);
                    acc[mt][jt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, b, acc[mt][jt], 0, 0, 0);
                }
            }
        }
    }
}

template <bool BF16, int NJT>
__global__ __launch_bounds__(PF_THREADS) void psp_prefill_kernel(PfArgs a) {
    extern __shared__ __align__(16) char smem[];
    constexpr int W = NJT * 16;                        // columns of this workgroup's tile
    constexpr int TILE_F4 = PF_TM * W / 4;             // float4 vectors per tile
    float* red = reinterpret_cast<float*>(smem);       // [wave][64][W]
    int* is_last = reinterpret_cast<int*>(smem + (size_t)PF_WAVES * PF_TM * W * sizeof(float));

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 15, lg = lane >> 4;
    // Workgroups are dealt round-robin to the 8 XCDs.  XCD x takes the slices x, x + 8, ... of every
    // tile, so the rows of U it needs (a few hundred KB) stay in its L2 while the activations
    // stream through; the grid is padded to 8 * ceil(S / 8) slices and the surplus leaves at once.
    const int sx = (a.S + 7) >> 3;
    const int xcd = (int)(blockIdx.x & 7u), j = (int)(blockIdx.x >> 3);
    const int s = xcd + 8 * (j % sx), unit = j / sx;
    if (s >= a.S) return;
    const int jg = unit % a.JG, tile = unit / a.JG;
    const int64_t K = a.K;

    // this wavefront's part of the slice, in steps of 32
    const int64_t k0 = (int64_t)s * a.kslice;
    const int64_t kend = k0 + a.kslice < K ? k0 + a.kslice : K;
    const int kw = a.kslice / PF_WAVES;                // multiple of 32
    const int64_t klo = k0 + (int64_t)wave * kw;
    const int64_t khi = klo + kw < kend ? klo + kw : kend;
    const int nsteps = khi > klo ? (int)((khi - klo) / PF_KSTEP) : 0;

    int64_t xoff[PF_MT], uoff[NJT];
#pragma unroll
    for (int mt = 0; mt < PF_MT; ++mt) {
        int64_t t = (int64_t)tile * PF_TM + mt * 16 + li;
        if (t > a.M - 1) t = a.M - 1;                  // padded token rows are never stored
        xoff[mt] = t * K + 8 * lg;
    }
#pragma unroll
    for (int jt = 0; jt < NJT; ++jt) {
        int row = jg * 64 + jt * 16 + li;
        if (row > a.rp - 1) row = a.rp - 1;            // columns past rp are never stored
        uoff[jt] = (int64_t)(row >> 4) * K * 16 + (lg * 16 + (row & 15)) * 8;   // block row of the packed U; a step of 32 is 512 values on
    }
    // every load stays inside [0, K): steps past the range re-read the last block of K and
    // are multiplied by zero
    auto kb_of = [&](int step) -> int64_t {
        const int64_t kb = klo + (int64_t)step * PF_KSTEP;
        return kb < K - PF_KSTEP ? kb : K - PF_KSTEP;
    };

    v4f acc[PF_MT][NJT];
#pragma unroll
    for (int mt = 0; mt < PF_MT; ++mt)
#pragma unroll
        for (int jt = 0; jt < NJT; ++jt) acc[mt][jt] = v4f{0.f, 0.f, 0.f, 0.f};

    // two fragments, consumed and refilled in place (the loop body is one basic block)
    Frag<BF16, NJT> f0, f1;
    // (the scheduling barriers keep f0's loads older than f1's on loop entry as on the back
    // edge, so that the first compute step waits for f0 only)
    pf_load<BF16, NJT>(f0, a.X, xoff, a.Ut, uoff, kb_of(0));
    __builtin_amdgcn_sched_barrier(0);
    pf_load<BF16, NJT>(f1, a.X, xoff, a.Ut, uoff, kb_of(1));
    __builtin_amdgcn_sched_barrier(0);
    for (int st = 0; st < nsteps; st += 2) {
        pf_compute<BF16, NJT>(f0, true, acc);
        pf_load<BF16, NJT>(f0, a.X, xoff, a.Ut, uoff, kb_of(st + 2));
        __builtin_amdgcn_sched_barrier(0);
        pf_compute<BF16, NJT>(f1, st + 1 < nsteps, acc);
        pf_load<BF16, NJT>(f1, a.X, xoff, a.Ut, uoff, kb_of(st + 3));
        __builtin_amdgcn_sched_barrier(0);
    }

    // ---- add the four wavefront tiles: lane holds rows mt*16 + 4*lg + v, column jt*16 + li
#pragma unroll
    for (int mt = 0; mt < PF_MT; ++mt)
#pragma unroll
        for (int jt = 0; jt < NJT; ++jt)
#pragma unroll
            for (int v = 0; v < 4; ++v)
                red[(wave * PF_TM + mt * 16 + 4 * lg + v) * W + jt * 16 + li] = acc[mt][jt][v];
    __syncthreads();

    const int64_t tok0 = (int64_t)tile * PF_TM;
    const int col0 = jg * 64;
    auto store_T = [&](int e4, const float4& v) {
        const int row = (e4 * 4) / W, col = (e4 * 4) % W;
        const int64_t tok = tok0 + row;
        if (tok < a.M) {
            const float vv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (col0 + col + c < a.r) a.T[tok * a.tp + col0 + col + c] = vv[c];
        }
    };
    // a partial tile is stored as four planes (one per vector component), so that the scalar
    // device-scope stores and loads of a wavefront cover whole 256-byte runs
    float* ptile = a.partials + ((int64_t)unit * a.S + s) * (TILE_F4 * 4);
#pragma unroll
    for (int i = 0; i < NJT; ++i) {
        const int e4 = tid + i * PF_THREADS;
        const float4* r4 = reinterpret_cast<const float4*>(red);
        float4 sum = r4[e4];
#pragma unroll
        for (int w = 1; w < PF_WAVES; ++w) {
            const float4 o = r4[w * TILE_F4 + e4];
            sum.x += o.x; sum.y += o.y; sum.z += o.z; sum.w += o.w;
        }
        if (a.S == 1) {
            store_T(e4, sum);
        } else {
            float* p = ptile + e4;
            bwla_store_agent(p, sum.x); bwla_store_agent(p + TILE_F4, sum.y);
            bwla_store_agent(p + 2 * TILE_F4, sum.z); bwla_store_agent(p + 3 * TILE_F4, sum.w);
        }
    }
    if (a.S == 1) return;
    if (!bwla_partials_arrive(&a.counters[unit], a.S, is_last)) return;
    // last workgroup of this tile: add the S partial tiles in slice order
    const float* pbase = a.partials + (int64_t)unit * a.S * (TILE_F4 * 4);
#pragma unroll
    for (int i = 0; i < NJT; ++i) {
        const int e4 = tid + i * PF_THREADS;
        // batches of eight loads in flight; slices past S re-read the last one and add zero
        v4f sum4 = v4f{0.f, 0.f, 0.f, 0.f};
        for (int ss = 0; ss < a.S; ss += 8) {
            v4f v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int sc = ss + u < a.S ? ss + u : a.S - 1;
                const float* p = pbase + (int64_t)sc * (TILE_F4 * 4) + e4;
                v[u] = v4f{bwla_load_agent(p), bwla_load_agent(p + TILE_F4), bwla_load_agent(p + 2 * TILE_F4),
                           bwla_load_agent(p + 3 * TILE_F4)};
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) sum4 += ss + u < a.S ? v[u] : v4f{0.f, 0.f, 0.f, 0.f};
        }
        store_T(e4, make_float4(sum4[0], sum4[1], sum4[2], sum4[3]));
    }
    if (tid == 0) a.counters[unit] = 0;                // leave the counters as they were found
}

template <bool BF16, int NJT>
hipError_t launch(const PfArgs& a, int blocks, hipStream_t st) {
    const size_t lds = (size_t)PF_WAVES * PF_TM * NJT * 16 * sizeof(float) + 16;
    hipError_t e = bwla_ensure_lds((const void*)psp_prefill_kernel<BF16, NJT>, lds);
    if (e != hipSuccess) return e;
    psp_prefill_kernel<BF16, NJT><<<dim3((unsigned)blocks), dim3(PF_THREADS), lds, st>>>(a);
    return hipGetLastError();
}

}  // namespace

// columns per workgroup tile for a padded rank rp: 16, 32 or 64
int bwla_psp_prefill_tile_cols(int rp) { return rp <= 16 ? 16 : rp <= 32 ? 32 : 64; }

hipError_t bwla_launch_psp_prefill(const bwla_layer_t* L, const void* dX, int xdtype, int64_t M, float* dT,
                                   void* dws, const bwla_psp_plan& plan, hipStream_t st) {
    const char* blob = (const char*)L->d_blob;
    PfArgs a;
    a.X = dX; a.M = M; a.K = L->K; a.r = bwla_rank_u(L); a.rp = (a.r + 15) & ~15; a.tp = L->r;
    a.Ut = (const __half*)(blob + L->off_U);
    a.T = dT;
    a.counters = (int*)dws;
    a.partials = dws ? (float*)((char*)dws + bwla_psp_counter_bytes(M)) : nullptr;
    a.S = plan.splits; a.JG = plan.col_groups; a.kslice = plan.k_per_split;
    const int blocks = plan.token_tiles * plan.col_groups * 8 * ((plan.splits + 7) / 8);
    const bool bf = xdtype == BWLA_X_BF16;
    switch (plan.tile_cols) {
        case 16: return bf ? launch<true, 1>(a, blocks, st) : launch<false, 1>(a, blocks, st);
        case 32: return bf ? launch<true, 2>(a, blocks, st) : launch<false, 2>(a, blocks, st);
        default: return bf ? launch<true, 4>(a, blocks, st) : launch<false, 4>(a, blocks, st);
    }
}
