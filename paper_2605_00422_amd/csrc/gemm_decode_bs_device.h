// Device code of the activation-stationary decode GEMM (see gemm_decode_bs.hip for the design):
// argument block, LDS map, the compute wavefronts and the epilogue wavefront.  Shared by the
// stand-alone kernel and by the fused single-launch decode kernel.
#pragma once
#include "bwla_internal.h"

namespace {

constexpr int BS_MAX_THREADS = 576;                  // up to 8 compute waves + 1 epilogue wave
constexpr int BS_MAXKS = BS_MAX_THREADS / 64 - 1;    // compute waves per workgroup


// byte-wise negation of four packed int8 (no value is -128 here)
__device__ __forceinline__ int neg_bytes(int x) {
    const unsigned nx = ~(unsigned)x;
    return (int)(((nx & 0x7f7f7f7fu) + 0x01010101u) ^ (nx & 0x80808080u));
}

// n / d for small non-negative n (d >= 1)
struct FastDivU {
    uint32_t d, m;
    __device__ explicit FastDivU(uint32_t dd) : d(dd), m(dd > 1 ? 0xFFFFFFFFu / dd + 1u : 0u) {}
    __device__ __forceinline__ int div(int n) const { return d > 1 ? (int)__umulhi((uint32_t)n, m) : n; }
};

struct BsArgs {
    const uint4* bits; int chunks, row_tiles;
    const int8_t* q; int M, K;
    const float* scale; const int32_t* qsum; const __half* alpha; const __half* V; const float* T;
    int r; float* Y; int N; int32_t* acc_out; int KS;
    int direct;      // stand-alone kernel: compute waves load their codes straight from global memory
                     // (else the code rows are staged in LDS first)
    int passes;      // rows longer than KS * CPW chunks are contracted in this many passes (else 1)
    uint16_t* H;     // not NULL: the rows interleave a gate and an up projection; instead of Y the
                     // kernel stores h[t, i] = silu(y[t, 2 i]) * y[t, 2 i + 1] as bf16, M x N / 2
};
// the gate of an MLP block on two neighbouring outputs (gate, up), rounded to bf16 (nearest even)
__device__ __forceinline__ uint32_t bs_swiglu_bf16(float g, float u) {
    const float h = g / (1.0f + __expf(-g)) * u;
    return (uint32_t)__builtin_bit_cast(uint16_t, (__bf16)h);
}

// zero what no copy fills in the code rows (from the last, possibly partial, chunk to the row end;
// the last 512 bytes are the operand of a chunk past K; only positions whose granule lies past K:
// the others belong to the copies, which may land at any time), and the partial-tile slots that
// no compute wave writes (the epilogue wave is their only reader)
template <int NT>
__device__ __forceinline__ void bs_zero_fill(const BsArgs& a, char* qt, v4i* red, int lane, bool code_rows = true) {
    const int pitch = (a.chunks + 1) * BWLA_CHUNK_COLS;
    const int rows = !code_rows ? 0 : (a.M < 16 ? a.M : 16);
    const int kgran = a.K >> 4;
    const int zbeg = (a.K / BWLA_CHUNK_COLS) * BWLA_CHUNK_COLS;
    for (int row = 0; row < rows; ++row)
        for (int o = zbeg + lane * 16; o < pitch; o += 64 * 16) {
            const int pos = o >> 4;
            if (((pos & ~31) | ((pos ^ row) & 31)) >= kgran)
                *reinterpret_cast<v4i*>(qt + row * pitch + o) = v4i{0, 0, 0, 0};
        }
    for (int s2 = 0; s2 < 2 * NT; ++s2)
        for (int k2 = a.KS; k2 < BS_MAXKS; ++k2) red[(s2 * BS_MAXKS + k2) * 64 + lane] = v4i{0, 0, 0, 0};
}

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
template <int CPW, int DEPTH, int NT, bool SIDE, bool MULTI = false>
__device__ __forceinline__ void compute_wave(const BsArgs& a, char* smem, int first, int stride, int n_iter,
                                             int wave, int lane) {
    const int li = lane & 15, lg = lane >> 4;
    const int KS = a.KS, chunks = a.chunks;
    const int JT = (a.r + 15) >> 4, rp = JT * 16;
    v4i* red = reinterpret_cast<v4i*>(smem);
    char* side = smem + red_bytes(NT);
    char* qt = side + 2 * side_bytes(rp, NT);
    // A row longer than KS * CPW chunks is contracted in several passes: step s of the loop is
    // unit s % n_iter in pass s / n_iter (all units of a pass, then the next pass, whose operand
    // codes are loaded when it begins); the weight prefetch runs on across the pass boundaries.
    // (MULTI is a compile-time choice: the one-pass kernels keep their precomputed addresses)
    const int H = MULTI ? a.passes : 1;
    const int last_it = n_iter * H - 1;                   // last step
    const int last_tile = a.row_tiles - 1;
    const FastDivU dni((uint32_t)n_iter);
    const uint4* wp[CPW];
#pragma unroll
    for (int i = 0; i < CPW; ++i) {
        const int c = wave + i * KS;
        wp[i] = a.bits + (c < chunks ? c : 0) * 64 + lane;
    }

    // Loads in the loop are unconditional (addresses clamped to valid tiles, chunks and rows).  A
    // chunk past the end of K pairs with all-zero activation operands; a step past this
    // workgroup's last one is fetched again and dropped.
    auto w_load = [&](int it_ahead, int nt, int i) -> v4i {
        const int sa = it_ahead < last_it ? it_ahead : last_it;
        if constexpr (MULTI) {
            const int hp = dni.div(sa), ia = sa - hp * n_iter;
            const int c = hp * KS * CPW + wave + i * KS;
            int tile = (first + ia * stride) * NT + nt;
            tile = tile < last_tile ? tile : last_tile;
            const uint4 x = a.bits[((int64_t)tile * chunks + (c < chunks ? c : 0)) * 64 + lane];
            return v4i{(int)x.x, (int)x.y, (int)x.z, (int)x.w};
        } else {
            int tile = (first + sa * stride) * NT + nt;
            tile = tile < last_tile ? tile : last_tile;
            const uint4 x = wp[i][(int64_t)tile * chunks * 64];
            return v4i{(int)x.x, (int)x.y, (int)x.z, (int)x.w};
        }
    };
    // side piece of this wave: piece p < PV is 1 KiB of the unit's V rows, piece PV its scales
    const int PV = (NT * rp + 31) >> 5;
    const int e0 = (wave < PV ? wave : 0) * 512 + lane * 8;      // first half of my 16 bytes in the unit
    const int vr = rp > 0 ? e0 / rp : 0, vc = rp > 0 ? e0 - vr * rp : 0;
    const bool is_alpha = wave == PV;
    const bool side_ok = is_alpha ? lane < 2 * NT : vr < 16 * NT;
    const int side_dst = is_alpha ? NT * 16 * side_pitch(rp) * 2 + lane * 16 : (vr * side_pitch(rp) + vc) * 2;
    auto s_load = [&](int it_ahead) -> v4i {
        const int sa = it_ahead < last_it ? it_ahead : last_it;
        const int ia = MULTI ? sa - dni.div(sa) * n_iter : sa;
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
    if (!a.direct) {
        stage_codes(a, qt, wave, lane);
        __builtin_amdgcn_s_waitcnt(0);
        bwla_lds_barrier();
    }
    v4i b[CPW][8];
    // operand codes of pass hp: chunks hp * KS * CPW + wave + i * KS
    auto load_b = [&](int hp) {
        const int cbase = hp * KS * CPW + wave;
        if (!a.direct) {
#pragma unroll
            for (int i = 0; i < CPW; ++i) {
                const int c = cbase + i * KS < chunks ? cbase + i * KS : chunks;   // chunk `chunks` is a zero patch
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    b[i][j] = *reinterpret_cast<const v4i*>(qt + brow * (Kp + BWLA_CHUNK_COLS) + c * BWLA_CHUNK_COLS +
                                                            (((lg * 8 + j) ^ brow) << 4));
            }
        } else {
            // Straight from global memory, once per workgroup and pass: lane (li, lg) takes, for
            // step j of a chunk, the 16 codes of token li at columns 128 lg + 16 j of the chunk
            // (the column order of the packed bits).  Granules past K (the last chunk may be
            // partial) and chunks this wave does not have are zero operands.  No LDS and no
            // barrier are involved, so every token count up to 16 and every row length fit; with
            // more than a few tokens it is also the faster way (16 tokens: 11.7 -> 9.7 us on the
            // 32B up projection), with one token the address arithmetic of the 16 or 32 loads
            // costs more than the staging (5.0 -> 5.1 us).
            const int kgran = a.K >> 4;
            const int8_t* qrow = a.q + (int64_t)brow * a.K;
#pragma unroll
            for (int i = 0; i < CPW; ++i)
#pragma unroll
                for (int j = 0; j < 8; ++j) b[i][j] = v4i{0, 0, 0, 0};
            // (lanes of token columns past M stay out of the loads: their operands are never used,
            // and an instruction costs the texture path as many cycles as it has active lanes)
            if (li < a.M) {
#pragma unroll
                for (int i = 0; i < CPW; ++i) {
                    const int c = cbase + i * KS;
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const int g = c * 32 + lg * 8 + j;
                        const bool ok = c < chunks && g < kgran;
                        const v4i v = *reinterpret_cast<const v4i*>(qrow + (ok ? g : 0) * 16);
                        b[i][j] = ok ? v : v4i{0, 0, 0, 0};
                    }
                }
            }
        }
#pragma unroll
        for (int i = 0; i < CPW; ++i)
            b[i][7] = v4i{neg_bytes(b[i][7].x), neg_bytes(b[i][7].y), neg_bytes(b[i][7].z), neg_bytes(b[i][7].w)};
    };
    load_b(0);
    int cur_pass = 0;

    // The trip count is rounded up to a multiple of DEPTH: surplus steps redo the last step.
    for (int it0 = 0; it0 < n_iter * H; it0 += DEPTH) {
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            const int it = it0 + d;
            if constexpr (MULTI) {                         // a new pass begins: its operand codes
                const int hp = dni.div(it < last_it ? it : last_it);
                if (hp != cur_pass) { load_b(hp); cur_pass = hp; }
            }
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
            bwla_lds_barrier();
            __builtin_amdgcn_sched_barrier(0);             // keep the steps in program order
        }
    }
}

// ------------------------------------------------------------------ epilogue wave
template <int DEPTH, int NT, int JTT, bool FAST, bool MULTI = false>
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
    float st = 0.0f;
    int qs = 0;
    // this lane's slice of T (token li, rank entries 16*uu + 4*lg + e), zero past M and r
    float tv[JTT > 0 ? JTT : 1][4];
    float tmax = 0.0f;
    if (tok_ok) {
        st = a.scale[t];
        qs = a.qsum[t];
    }
#pragma unroll
    for (int uu = 0; uu < JTT; ++uu)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int j = uu * 16 + 4 * lg + e;
            tv[uu][e] = 0.0f;
            if (tok_ok && j < a.r) tv[uu][e] = a.T[(int64_t)t * a.r + j];
            tmax = fmaxf(tmax, fabsf(tv[uu][e]));
        }
    if (a.direct) {
        bs_zero_fill<NT>(a, qt, red, lane, false);         // (the compute waves fetch their codes themselves)
    } else {
        bs_zero_fill<NT>(a, qt, red, lane);
        stage_codes(a, qt, wave, lane);
        __builtin_amdgcn_s_waitcnt(0);                     // zeros written, this wave's copies landed
        bwla_lds_barrier();
    }

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

    // Several passes over a long row (see compute_wave): step `it` is unit it % n_iter of pass
    // it / n_iter; the sums of the earlier passes wait in LDS (this wavefront alone touches them)
    // and the unit is finished in the last pass.
    const int H = MULTI ? a.passes : 1;
    const FastDivU dni((uint32_t)n_iter);
    v4i* usum = reinterpret_cast<v4i*>(qt + (a.direct ? 0 : (size_t)(a.M < 16 ? a.M : 16) * (a.chunks + 1) * BWLA_CHUNK_COLS));
    const int n_real = n_iter * H;
    const int n_steps = (n_real + DEPTH - 1) / DEPTH * DEPTH;    // same barrier count as the compute waves
    for (int it = 0; it < n_steps; ++it) {
        bwla_lds_barrier();                                // partial tiles and side pieces of `it` are in LDS
        const char* sd = side + (it & 1) * side_bytes(rp, NT);
        const int hp = MULTI ? dni.div(it < n_real ? it : 0) : 0, ui = it - hp * n_iter;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const int tile = (first + ui * stride) * NT + nt;
            if (it >= n_real || tile >= a.row_tiles) continue;      // surplus step or ragged last unit
            v4i tot = v4i{0, 0, 0, 0};
#pragma unroll
            for (int k2 = 0; k2 < BS_MAXKS; ++k2)
                tot += red[(((it & 1) * NT + nt) * BS_MAXKS + k2) * 64 + lane];
            if constexpr (MULTI) {
                v4i* us = usum + (ui * NT + nt) * 64 + lane;
                if (hp > 0) tot += *us;
                if (hp < H - 1) { *us = tot; continue; }
            }

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
            if (a.H != nullptr) {
                // (N is even; a pair never straddles the end of a row)
                if (tok_ok) {
                    uint16_t* hrow = a.H + (int64_t)t * (N >> 1) + (nb >> 1);
                    if (FAST) {
                        if (nb < N)
                            *reinterpret_cast<uint32_t*>(hrow) = bs_swiglu_bf16(y[0], y[1]) | (bs_swiglu_bf16(y[2], y[3]) << 16);
                    } else {
                        if (nb + 1 < N) hrow[0] = (uint16_t)bs_swiglu_bf16(y[0], y[1]);
                        if (nb + 3 < N) hrow[1] = (uint16_t)bs_swiglu_bf16(y[2], y[3]);
                    }
                }
            } else if (FAST) {
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
    }
}

constexpr int BS_CPW = 2;   // two chunks per compute wave amortize the class recombination
// Longer rows (K up to 7 * 4 * 512 = 14336, e.g. the 7B down projection): four chunks per compute
// wave, whose 32 operand registers per chunk then need the 256-register budget of a workgroup of
// at most eight wavefronts (seven compute waves + the epilogue wave).
constexpr int BS_CPW_LONG = 4;
constexpr int BS_MAXKS_LONG = 7;
inline int bs_cpw_for(int chunks) {
    return (chunks + BS_CPW - 1) / BS_CPW <= BS_MAXKS ? BS_CPW : BS_CPW_LONG;
}
// still longer rows: passes of BS_MAXKS_LONG * BS_CPW_LONG = 28 chunks (70B down, K = 28672: two)
inline int bs_passes_for(int chunks) {
    const int per = BS_MAXKS_LONG * BS_CPW_LONG;
    return bs_cpw_for(chunks) == BS_CPW ? 1 : (chunks + per - 1) / per;
}
inline int bs_ks_for(int chunks) {
    const int cpw = bs_cpw_for(chunks);
    const int ks = (chunks + cpw - 1) / cpw;
    return cpw == BS_CPW ? ks : (ks < BS_MAXKS_LONG ? ks : BS_MAXKS_LONG);
}

// (M: token rows staged in LDS; 0 when the compute waves load their codes themselves.  With more
// than one pass: 1 KiB per tile of the workgroup's units behind them, for the sums of earlier passes.)
inline size_t bs_lds_bytes(int64_t M, int chunks, int rp, int nt, int pass_units = 0) {
    return (size_t)red_bytes(nt) + 2 * (size_t)side_bytes(rp, nt) +
           (size_t)(M < 16 ? M : 16) * ((size_t)chunks + 1) * BWLA_CHUNK_COLS + (size_t)pass_units * nt * 1024;
}

// one compute wave per side piece (the unit's V rows in 1 KiB pieces + its scales), LDS fits
inline bool bs_fits(int64_t M, int chunks, int r, int nt, int cpw = BS_CPW, int pass_units = 0) {
    const int KS = cpw == BS_CPW ? (chunks + cpw - 1) / cpw : bs_ks_for(chunks);
    const int rp = ((r + 15) >> 4) * 16;
    return KS <= (cpw == BS_CPW ? BS_MAXKS : BS_MAXKS_LONG) && KS >= ((nt * rp + 31) >> 5) + 1 &&
           bs_lds_bytes(M, chunks, rp, nt, pass_units) <= 160 * 1024;
}

}  // namespace
