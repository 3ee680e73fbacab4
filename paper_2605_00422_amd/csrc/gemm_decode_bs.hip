// Binary-weight GEMM for decode batches (M <= 16) with K <= 8192: "activation-stationary".
//
// A workgroup owns a stream of 16-row output tiles.  It has one compute wavefront per CPW
// 512-column chunks of K plus one epilogue wavefront.  Each compute wave loads its slice of the
// activation codes ONCE into registers as MFMA B operands (8 digit classes x 16 bytes per lane
// and chunk) and from then on only streams sign bits: per tile one 128-bit load per lane and
// chunk, one AND per four weights to expand it, eight 16x16x64 INT8 MFMAs per chunk.
//
// Digit classes: (w & (0x01010101 << j)) is a run of int8 digits b * 2^j (class 7 reads as
// -128, so its activation operand is stored negated).  The classes are chained through the
// MFMA accumulator from the high class down with exact arithmetic shifts in between (two
// independent chains, odd and even classes),
//     r_j = (r_{j+2} >> 2) + P_j,   P_j = 2^j * sum_k q b_j   (r_{j+2} is a multiple of 2^{j+2}),
// so the recombination costs four shifts per class and no separate accumulators.
//
// Everything that streams from HBM -- sign bits, and the tile's V rows and scales ("side"
// pieces, fetched by the first compute waves) -- sits in a register ring that is consumed and
// refilled in place DEPTH tiles ahead, inside a loop body that is one basic block, so each wait
// covers exactly the load it needs.  Per tile the compute waves drop their partial sums and the
// side pieces into LDS; after one LDS-only barrier the epilogue wave (which touches HBM only to
// store) applies
//     Y[t,n] = scale_t * alpha_n * (2 * sum_k q b - qsum_t) + sum_j T[t,j] V[n,j].
// The grid is persistent.
#include "bwla_internal.h"

namespace {

constexpr int BS_MAX_THREADS = 576;                  // up to 8 compute waves + 1 epilogue wave
constexpr int BS_MAXKS = BS_MAX_THREADS / 64 - 1;    // compute waves per workgroup

#ifdef BWLA_TRACE
__device__ long long bwla_trace_buf[64 * 16 * 40];
#define TRACE(slot) do { if (lane == 0 && blockIdx.x < 64) bwla_trace_buf[(blockIdx.x * 16 + wave) * 40 + (slot)] = __builtin_readcyclecounter(); } while (0)
#else
#define TRACE(slot) do { } while (0)
#endif

// byte-wise negation of four packed int8 (no value is -128 here)
__device__ __forceinline__ int neg_bytes(int x) {
    const unsigned nx = ~(unsigned)x;
    return (int)(((nx & 0x7f7f7f7fu) + 0x01010101u) ^ (nx & 0x80808080u));
}

struct BsArgs {
    const uint4* bits; int chunks, row_tiles;
    const int8_t* q; int M, K;
    const float* scale; const int32_t* qsum; const __half* alpha; const __half* V; const float* T;
    int r; float* Y; int N; int32_t* acc_out; int KS;
};

// A step of a workgroup covers NT adjacent 16-row tiles (a "unit").
// LDS map: [partial tiles 2 x NT x BS_MAXKS x 1 KiB][side 2 x side_bytes][code rows min(M,16) x (Kp + 512)]
__host__ __device__ __forceinline__ int side_pitch(int rp) { return rp + 8; }      // halfs per V row
__host__ __device__ __forceinline__ int side_bytes(int rp, int nt) { return nt * (16 * side_pitch(rp) * 2 + 32); }
__host__ __device__ __forceinline__ int red_bytes(int nt) { return 2 * nt * BS_MAXKS * 1024; }

// Asynchronous global -> LDS copies of the code rows, 1 KiB per instruction and no registers
// involved, shared out over all waves of the workgroup.  The hardware puts lane l's 16 bytes at
// block + 16*l, so the row swizzle is applied to the source: position p of a row receives
// granule (p & ~31) | ((p ^ row) & 31).  Granules past K are left to the zero fill.
__device__ __forceinline__ void stage_codes(const BsArgs& a, char* qt, int wave, int lane) {
    const int pitch = (a.chunks + 1) * BWLA_CHUNK_COLS;
    const int rows = a.M < 16 ? a.M : 16;
    const int kgran = a.K >> 4, nblk = (kgran + 63) >> 6, nw = a.KS + 1;
    // every workgroup copies the same rows: start each one at a different block so that they do
    // not all hit the same L2 channel at the same moment
    const int total = rows * nblk;
    const int rot = (int)(blockIdx.x * 13u % (unsigned)total);
    for (int i = wave; i < total; i += nw) {
        int p = i + rot;
        if (p >= total) p -= total;
        const int row = p / nblk, blk = p - row * nblk;
        const int pos = blk * 64 + lane;
        const int gc = (pos & ~31) | ((pos ^ row) & 31);
        if (gc < kgran)
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void*)(a.q + (int64_t)row * a.K + (gc << 4)),
                (__attribute__((address_space(3))) void*)(qt + row * pitch + blk * 1024), 16, 0, 0);
    }
}

// ------------------------------------------------------------------ compute wave
template <int CPW, int DEPTH, int NT, bool SIDE>
__device__ __forceinline__ void compute_wave(const BsArgs& a, char* smem, int first, int stride, int n_iter,
                                             int wave, int lane) {
    const int li = lane & 15, lg = lane >> 4;
    const int KS = a.KS, chunks = a.chunks;
    const int JT = (a.r + 15) >> 4, rp = JT * 16;
    v4i* red = reinterpret_cast<v4i*>(smem);
    char* side = smem + red_bytes(NT);
    char* qt = side + 2 * side_bytes(rp, NT);
    const int last_it = n_iter - 1;
    const int last_tile = a.row_tiles - 1;

    // Loads in the loop are unconditional (addresses clamped to valid tiles, chunks and rows).  A
    // chunk past the end of K pairs with all-zero activation operands; a unit past this
    // workgroup's last one is fetched again and dropped.
    const uint4* wp[CPW];
#pragma unroll
    for (int i = 0; i < CPW; ++i) {
        const int c = wave + i * KS;
        wp[i] = a.bits + (c < chunks ? c : 0) * 64 + lane;
    }
    auto w_load = [&](int it_ahead, int nt, int i) -> v4i {
        const int ia = it_ahead < last_it ? it_ahead : last_it;
        int tile = (first + ia * stride) * NT + nt;
        tile = tile < last_tile ? tile : last_tile;
        const uint4 x = wp[i][(int64_t)tile * chunks * 64];
        return v4i{(int)x.x, (int)x.y, (int)x.z, (int)x.w};
    };
    // side piece of this wave: piece p < PV is 1 KiB of the unit's V rows, piece PV its scales
    const int PV = (NT * rp + 31) >> 5;
    const int e0 = (wave < PV ? wave : 0) * 512 + lane * 8;      // first half of my 16 bytes in the unit
    const int vr = rp > 0 ? e0 / rp : 0, vc = rp > 0 ? e0 - vr * rp : 0;
    const bool is_alpha = wave == PV;
    const bool side_ok = is_alpha ? lane < 2 * NT : vr < 16 * NT;
    const int side_dst = is_alpha ? NT * 16 * side_pitch(rp) * 2 + lane * 16 : (vr * side_pitch(rp) + vc) * 2;
    auto s_load = [&](int it_ahead) -> v4i {
        const int ia = it_ahead < last_it ? it_ahead : last_it;
        const int n0 = (first + ia * stride) * NT * 16;
        const __half* src;
        if (is_alpha) {
            int n = n0 + (lane < 2 * NT ? lane * 8 : 0);
            if (n >= a.N) n = 0;                                  // stays inside the padded scale array
            src = a.alpha + n;
        } else {
            int n = n0 + (vr < 16 * NT ? vr : 0);
            if (n >= a.N) n = a.N - 1;
            src = a.V + (int64_t)n * rp + vc;
        }
        const uint4 x = *reinterpret_cast<const uint4*>(src);
        return v4i{(int)x.x, (int)x.y, (int)x.z, (int)x.w};
    };

    v4i wq[DEPTH][NT][CPW];
    v4i sq[DEPTH];
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) {                      // HBM streams first: the longest latency
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int i = 0; i < CPW; ++i) wq[d][nt][i] = w_load(d, nt, i);
        if (SIDE) sq[d] = s_load(d);
    }

    // activation codes of this wave's chunks, kept in registers for the whole kernel.  All waves
    // stage the code rows into LDS first; granules are XOR-swizzled by row against bank conflicts.
    const int Kp = chunks * BWLA_CHUNK_COLS;
    const int brow = li < a.M ? li : a.M - 1;             // padded token columns repeat the last row; never stored
    stage_codes(a, qt, wave, lane);
    __builtin_amdgcn_s_waitcnt(0);                         // this wave's copies (and first units) landed
    TRACE(1);
    bwla_lds_barrier();
    v4i b[CPW][8];
#pragma unroll
    for (int i = 0; i < CPW; ++i) {
        const int c = wave + i * KS < chunks ? wave + i * KS : chunks;   // chunk `chunks` is a zero patch
#pragma unroll
        for (int j = 0; j < 8; ++j)
            b[i][j] = *reinterpret_cast<const v4i*>(qt + brow * (Kp + BWLA_CHUNK_COLS) + c * BWLA_CHUNK_COLS +
                                                    (((lg * 8 + j) ^ brow) << 4));
    }
#pragma unroll
    for (int i = 0; i < CPW; ++i)
        b[i][7] = v4i{neg_bytes(b[i][7].x), neg_bytes(b[i][7].y), neg_bytes(b[i][7].z), neg_bytes(b[i][7].w)};
    TRACE(2);

    // The trip count is rounded up to a multiple of DEPTH: surplus steps redo the last unit.
    for (int it0 = 0; it0 < n_iter; it0 += DEPTH) {
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            const int it = it0 + d;
            // per tile two independent chains (odd and even classes, two bits apart):
            // e = S6+S4+S2+S0 exactly, o = 2*(S7+S5+S3+S1) exactly
            v4i acc_e[NT], acc_o[NT];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) acc_e[nt] = acc_o[nt] = v4i{0, 0, 0, 0};
#pragma unroll
            for (int jj = 3; jj >= 0; --jj) {
                const int mo = 0x01010101 << (2 * jj + 1), me = 0x01010101 << (2 * jj);
#pragma unroll
                for (int i = 0; i < CPW; ++i)
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt) {
                        const v4i w = wq[d][nt][i];
                        const v4i xo = v4i{w.x & mo, w.y & mo, w.z & mo, w.w & mo};
                        acc_o[nt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(xo, b[i][2 * jj + 1], acc_o[nt], 0, 0, 0);
                        const v4i xe = v4i{w.x & me, w.y & me, w.z & me, w.w & me};
                        acc_e[nt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(xe, b[i][2 * jj], acc_e[nt], 0, 0, 0);
                    }
                if (jj > 0) {
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt) { acc_o[nt] = acc_o[nt] >> 2; acc_e[nt] = acc_e[nt] >> 2; }
                }
            }
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                red[(((it & 1) * NT + nt) * BS_MAXKS + wave) * 64 + lane] = acc_e[nt] + (acc_o[nt] >> 1);
            if (SIDE) {
                if (side_ok) *reinterpret_cast<v4i*>(side + (it & 1) * side_bytes(rp, NT) + side_dst) = sq[d];
                sq[d] = s_load(it + DEPTH);
            }
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int i = 0; i < CPW; ++i) wq[d][nt][i] = w_load(it + DEPTH, nt, i);
            if (it < 12) TRACE(3 + 3 * it);
            bwla_lds_barrier();
            if (it < 12) TRACE(5 + 3 * it);
            __builtin_amdgcn_sched_barrier(0);             // keep the steps in program order
        }
    }
}

// ------------------------------------------------------------------ epilogue wave
template <int DEPTH, int NT, int JTT, bool FAST>
__device__ __forceinline__ void epilogue_wave(const BsArgs& a, char* smem, int first, int stride, int n_iter,
                                              int wave, int lane) {
    const int li = lane & 15, lg = lane >> 4;
    const int KS = a.KS, N = a.N;
    const int JT = (a.r + 15) >> 4, rp = JT * 16;
    v4i* red = reinterpret_cast<v4i*>(smem);
    const char* side = smem + red_bytes(NT);
    char* qt = smem + red_bytes(NT) + 2 * side_bytes(rp, NT);
    const int last_it = n_iter - 1;
    const int t = li;
    const bool tok_ok = t < a.M;
    const float st = tok_ok ? a.scale[t] : 0.0f;
    const int qs = tok_ok ? a.qsum[t] : 0;
    // this lane's slice of T (token li, rank entries 16*uu + 4*lg + e), zero past M and r
    float tv[JTT > 0 ? JTT : 1][4];
    float tmax = 0.0f;
#pragma unroll
    for (int uu = 0; uu < JTT; ++uu)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int j = uu * 16 + 4 * lg + e;
            tv[uu][e] = (tok_ok && j < a.r) ? a.T[(int64_t)t * a.r + j] : 0.0f;
            tmax = fmaxf(tmax, fabsf(tv[uu][e]));
        }

    // ---- code rows in LDS: rows x (Kp + 512) bytes; zero what no copy will fill, from the last,
    // possibly partial, chunk to the row end (the last 512 bytes are the operand of a chunk past K)
    {
        const int pitch = (a.chunks + 1) * BWLA_CHUNK_COLS;
        const int rows = a.M < 16 ? a.M : 16;
        const int zbeg = (a.K / BWLA_CHUNK_COLS) * BWLA_CHUNK_COLS;
        for (int row = 0; row < rows; ++row)
            for (int o = zbeg + lane * 16; o < pitch; o += 64 * 16)
                *reinterpret_cast<v4i*>(qt + row * pitch + o) = v4i{0, 0, 0, 0};
    }
    stage_codes(a, qt, wave, lane);
    // partial-tile slots no compute wave writes stay zero (this wave is their only reader)
    for (int s2 = 0; s2 < 2 * NT; ++s2)
        for (int k2 = KS; k2 < BS_MAXKS; ++k2) red[(s2 * BS_MAXKS + k2) * 64 + lane] = v4i{0, 0, 0, 0};
    __builtin_amdgcn_s_waitcnt(0);                         // zeros written, this wave's copies landed
    TRACE(1);
    bwla_lds_barrier();

    // fp16 operands of T for the f16 MFMA: T * 2^k = hi + lo (both fp16, error 2^-22), with the
    // power of two k chosen per token so that the largest entry sits near 2^13
    tmax = fmaxf(tmax, __shfl_xor(tmax, 16, 64));
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
    int kexp = 0;
    if (tmax > 0.0f && tmax < 3.0e38f) kexp = 13 - ilogbf(tmax);
    kexp = kexp > 100 ? 100 : (kexp < -100 ? -100 : kexp);
    const float tinv = ldexpf(1.0f, -kexp);
    typedef _Float16 v4h __attribute__((ext_vector_type(4)));
    v4h thi[JTT > 0 ? JTT : 1], tlo[JTT > 0 ? JTT : 1];
#pragma unroll
    for (int uu = 0; uu < JTT; ++uu)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float x = ldexpf(tv[uu][e], kexp);
            const _Float16 h = (_Float16)x;
            thi[uu][e] = h;
            tlo[uu][e] = (_Float16)(x - (float)h);
        }
    TRACE(2);

    const int n_steps = (n_iter + DEPTH - 1) / DEPTH * DEPTH;    // same barrier count as the compute waves
    for (int it = 0; it < n_steps; ++it) {
        if (it < 12) TRACE(3 + 3 * it);
        bwla_lds_barrier();                                // partial tiles and side pieces of `it` are in LDS
        if (it < 12) TRACE(4 + 3 * it);
        const char* sd = side + (it & 1) * side_bytes(rp, NT);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const int tile = (first + it * stride) * NT + nt;
            if (it >= n_iter || tile >= a.row_tiles) continue;      // surplus step or ragged last unit
            v4i tot = v4i{0, 0, 0, 0};
#pragma unroll
            for (int k2 = 0; k2 < BS_MAXKS; ++k2)
                tot += red[(((it & 1) * NT + nt) * BS_MAXKS + k2) * 64 + lane];

            // low-rank term on f16 MFMA (fp32 accumulate): D[n][t] = sum_j V[n][j] T[t][j]; lane
            // (li, lg) feeds j = 16*uu + 4*lg + e, e = 0..3, of group uu for both operands
            v4f low0 = v4f{0.f, 0.f, 0.f, 0.f}, low1 = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int uu = 0; uu < JTT; ++uu) {
                const int ue = uu < JT ? uu : 0;           // groups past the rank pair with zero T
                const v4h vv = *reinterpret_cast<const v4h*>(
                    sd + ((nt * 16 + li) * side_pitch(rp) + ue * 16 + 4 * lg) * 2);
                low0 = __builtin_amdgcn_mfma_f32_16x16x16f16(vv, thi[uu], low0, 0, 0, 0);
                low1 = __builtin_amdgcn_mfma_f32_16x16x16f16(vv, tlo[uu], low1, 0, 0, 0);
            }
            const uint2 av = *reinterpret_cast<const uint2*>(sd + NT * 16 * side_pitch(rp) * 2 + nt * 32 + 8 * lg);
            const __half2 a0 = *reinterpret_cast<const __half2*>(&av.x);
            const __half2 a1 = *reinterpret_cast<const __half2*>(&av.y);
            const float al[4] = {__low2float(a0), __high2float(a0), __low2float(a1), __high2float(a1)};

            int ai[4];
            float y[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                ai[v] = 2 * tot[v] - qs;
                y[v] = st * al[v] * (float)ai[v] + (low0[v] + low1[v]) * tinv;
            }
            const int nb = tile * 16 + 4 * lg;
            if (FAST) {
                if (tok_ok && nb < N)
                    *reinterpret_cast<float4*>(a.Y + (int64_t)t * N + nb) = make_float4(y[0], y[1], y[2], y[3]);
            } else if (tok_ok) {
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    if (nb + v < N) {
                        a.Y[(int64_t)t * N + nb + v] = y[v];
                        if (a.acc_out) a.acc_out[(int64_t)t * N + nb + v] = ai[v];
                    }
            }
        }
        if (it < 12) TRACE(5 + 3 * it);
    }
}

// NT: 16-row tiles per step.  JTT: compile-time number of 16-wide rank groups (>= ceil(r/16)).
// FAST: N % 4 == 0 and no accumulator dump, which allows float4 stores.
template <int CPW, int DEPTH, int NT, int JTT, bool FAST>
__global__ __launch_bounds__(BS_MAX_THREADS) void gemm_decode_bs_kernel(BsArgs a) {
    extern __shared__ __align__(16) char smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int stride = gridDim.x, first = blockIdx.x;
    const int units = (a.row_tiles + NT - 1) / NT;
    const int n_iter = (units - first + stride - 1) / stride;            // >= 1: grid <= units
    const int PV = (NT * (((a.r + 15) >> 4) * 16) + 31) >> 5;
    TRACE(0);
    if (wave == a.KS) epilogue_wave<DEPTH, NT, JTT, FAST>(a, smem, first, stride, n_iter, wave, lane);
    else if (wave <= PV) compute_wave<CPW, DEPTH, NT, true>(a, smem, first, stride, n_iter, wave, lane);
    else compute_wave<CPW, DEPTH, NT, false>(a, smem, first, stride, n_iter, wave, lane);
}


constexpr int BS_CPW = 2;   // two chunks per compute wave amortize the class recombination

size_t bs_lds_bytes(int64_t M, int chunks, int rp, int nt) {
    return (size_t)red_bytes(nt) + 2 * (size_t)side_bytes(rp, nt) +
           (size_t)(M < 16 ? M : 16) * ((size_t)chunks + 1) * BWLA_CHUNK_COLS;
}

// one compute wave per side piece (the unit's V rows in 1 KiB pieces + its scales), LDS fits
bool bs_fits(int64_t M, int chunks, int r, int nt) {
    const int KS = (chunks + BS_CPW - 1) / BS_CPW;
    const int rp = ((r + 15) >> 4) * 16;
    return KS <= BS_MAXKS && KS >= ((nt * rp + 31) >> 5) + 1 && bs_lds_bytes(M, chunks, rp, nt) <= 160 * 1024;
}

}  // namespace

#ifdef BWLA_TRACE
extern "C" int bwla_trace_dump(long long* host, int n) {
    return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(bwla_trace_buf), (size_t)n * sizeof(long long));
}
#endif

bool bwla_gemm_decode_bs_supported(int64_t M, int64_t K, int r) {
    const int chunks = (int)bwla_chunks(K);
    return M <= 16 && chunks >= 2 && bs_fits(M, chunks, r, 1);
}

// explicit launch shape: nt tiles per step (1 or 2), grid size, prefetch depth (2 or 4)
hipError_t bwla_launch_gemm_decode_bs_cfg(const bwla_layer_t* L, const int8_t* dq, const float* dscale,
                                          const int32_t* dqsum, const float* dT, int64_t M, float* dY,
                                          int32_t* dacc, hipStream_t st, int nt, int grid, int depth) {
    const char* blob = (const char*)L->d_blob;
    const int chunks = (int)bwla_chunks(L->K), row_tiles = (int)bwla_row_tiles(L->N);
    if ((nt != 1 && nt != 2) || grid < 1 || chunks < 2 || M > 16 || !bs_fits(M, chunks, L->r, nt))
        return hipErrorInvalidValue;
    const int KS = (chunks + BS_CPW - 1) / BS_CPW;
    const int JT = (L->r + 15) >> 4, rp = JT * 16;
    const int units = (row_tiles + nt - 1) / nt;
    if (grid > units) grid = units;
    const int jtt = JT == 0 ? 0 : JT == 1 ? 1 : JT == 2 ? 2 : JT <= 4 ? 4 : 8;
    const size_t lds = bs_lds_bytes(M, chunks, rp, nt);
    BsArgs a{(const uint4*)(blob + L->off_bits), chunks, row_tiles, dq, (int)M, (int)L->K, dscale, dqsum,
             (const __half*)(blob + L->off_alpha), (const __half*)(blob + L->off_V), dT, L->r, dY, (int)L->N,
             dacc, KS};
    auto launch = [&](auto kern) -> hipError_t {
        static bwla_lds_attr attr;
        hipError_t e = attr.ensure((const void*)kern, lds);
        if (e != hipSuccess) return e;
        kern<<<dim3((unsigned)grid), dim3(64 * (KS + 1)), lds, st>>>(a);
        return hipGetLastError();
    };
    const bool fast = (L->N % 4 == 0) && dacc == nullptr;
#define BS_CASE(D, T, J)                                                                                   \
    if (depth == D && nt == T && jtt == J)                                                                 \
        return fast ? launch(gemm_decode_bs_kernel<BS_CPW, D, T, J, true>)                                 \
                    : launch(gemm_decode_bs_kernel<BS_CPW, D, T, J, false>);
#define BS_CASES(J) BS_CASE(2, 1, J) BS_CASE(4, 1, J) BS_CASE(2, 2, J) BS_CASE(4, 2, J)
    BS_CASES(0) BS_CASES(1) BS_CASES(2) BS_CASES(4) BS_CASES(8)
#undef BS_CASES
#undef BS_CASE
    return hipErrorInvalidValue;
}

hipError_t bwla_launch_gemm_decode_bs(const bwla_layer_t* L, const int8_t* dq, const float* dscale,
                                      const int32_t* dqsum, const float* dT, int64_t M, float* dY,
                                      int32_t* dacc, hipStream_t st) {
    const int chunks = (int)bwla_chunks(L->K), row_tiles = (int)bwla_row_tiles(L->N);
    const int cus = bwla_device_cus();
    // Measured on MI355X: one tile per step and one workgroup per CU is the best shape for all
    // decode layers tried (two tiles per step run the steady state ~30% faster but pay more at
    // start-up, which dominates at these sizes).
    const int nt = 1;
    const int units = (row_tiles + nt - 1) / nt;
    const int grid = units < cus ? units : cus;
    (void)chunks;
    return bwla_launch_gemm_decode_bs_cfg(L, dq, dscale, dqsum, dT, M, dY, dacc, st, nt, grid, 2);
}

int bwla_device_cus() {
    static int cus = 0;
    if (cus == 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
            cus = n;
        else
            cus = 256;
    }
    return cus;
}
