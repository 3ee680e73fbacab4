// Rotation + quantization of one token per workgroup on bf16 MFMA with exact operand splits.
#pragma once
#include "rotate_common.h"

namespace {

// ================================================================== rotation on bf16 MFMA
// bf16 activations, second form of the rotation: every product is exact (bf16 x bf16 in fp32)
// and only the fp32 accumulation rounds, because the fp32 factors are stored as three bf16
// terms (8 + 8 + 8 mantissa bits) and the intermediate Z is split the same way in registers.
//   stage 1  Z[a,d]  = sum_b V[a,b] R2[b,d]       MFMA 16x16x32: A = V rows (LDS), B = R2 terms
//   stage 2  Yt[d,c] = sum_a Z[a,d] R1[a,c]       A = Z terms, B = R1 terms (LDS)
// Wavefront w owns the 16 columns d of strip w.  The accumulator tile of stage 1 (lane (li, lg)
// holds Z[a = 4*lg + v][d = li]) already is an A operand of stage 2 (row d = li, contraction
// indices a = 4*lg + v): two stacked tiles give the eight indices of one 32-deep step, in the
// order for which the packed R1 terms were permuted.  Z therefore never leaves registers, and
// between the two stages there is neither an LDS round trip nor a barrier.  The R2 terms of a
// strip are read once, from global memory, by the one wavefront that uses them.
constexpr int R3_MAXA = 16;          // 16-row tiles along n1 (a and c); kernels are built for 4, 8, 12, 16
constexpr int R3_MAXK1 = 5;          // 32-deep steps along n2 in stage 1: n2 <= 160
constexpr int R3_MAXW = 10;          // wavefronts = 16-column strips along n2
constexpr int R3_CPITCH = 80;        // bytes of one chunk row in LDS: 32 bf16 + 16 bytes of padding
constexpr int R3_ITEMS = 6;          // 16-byte pieces of a streamed chunk per thread

typedef __attribute__((ext_vector_type(8))) __bf16 v8bf;

struct R3Shape {
    int n1, n2, at, strips, k1, ch2, vpitch, vbytes, cbytes, nbuf, r0bytes;
    bool ok, resident, alias;
    size_t lds_bytes;
};

__host__ __device__ inline R3Shape r3_shape(int n1, int n2) {
    R3Shape s;
    s.n1 = n1; s.n2 = n2;
    s.at = (n1 + 15) >> 4; s.strips = (n2 + 15) >> 4;
    s.k1 = (n2 + 31) >> 5; s.ch2 = (n1 + 31) >> 5;
    s.vpitch = s.k1 * 64 + 16;                                   // bytes per token row: n2 padded to 32, + 16
    s.vbytes = s.at * 16 * s.vpitch;
    s.cbytes = 3 * s.at * 16 * R3_CPITCH;                        // one chunk: three terms x n1p16 rows
    const size_t res = (size_t)s.vbytes + (size_t)s.ch2 * s.cbytes + 256;
    s.resident = res <= RQ_LDS_LIMIT;
    s.nbuf = s.resident ? s.ch2 : 2;
    // streaming with two chunk buffers; if they do not fit next to the token rows, the second one
    // takes the place of the token rows, which are dead once stage 1 is done
    s.alias = !s.resident && (size_t)s.vbytes + 2 * (size_t)s.cbytes + 256 > RQ_LDS_LIMIT;
    s.r0bytes = s.alias && s.cbytes > s.vbytes ? s.cbytes : s.vbytes;
    s.lds_bytes = (size_t)s.r0bytes + (size_t)(s.alias ? 1 : s.nbuf) * s.cbytes + 256;
    // streamed chunks: 12 * n1p16 pieces over 64 * strips threads, at most R3_ITEMS each
    const bool stream_ok = 12 * s.at * 16 <= R3_ITEMS * 64 * s.strips;
    // more than 12 tiles along n1 need more registers than a 10-wavefront workgroup can have
    s.ok = s.at <= R3_MAXA && s.k1 <= R3_MAXK1 && s.strips <= (s.at > 12 ? 8 : R3_MAXW) &&
           s.lds_bytes <= RQ_LDS_LIMIT && (s.resident || stream_ok);
    return s;
}

__device__ __forceinline__ void r3_split3(const float (&f)[8], v8bf& h1, v8bf& h2, v8bf& h3) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const __bf16 a = (__bf16)f[e];
        const float r1 = f[e] - (float)a;
        const __bf16 b = (__bf16)r1;
        h1[e] = a; h2[e] = b; h3[e] = (__bf16)(r1 - (float)b);
    }
}

// One token per workgroup with resident factors (!LOOP): everything the token needs is requested
// in one go -- its R2 terms, the token itself, and last the R1 terms, which stay in flight (in
// registers) through stage 1 and go to LDS just before stage 2.  Wavefronts beyond the strips, if
// the workgroup has any, carry their share of the R1 terms and end once it is in LDS.
constexpr int R3_FILLR = 12;         // 16-byte pieces of the R1 terms a thread keeps in flight
// DUAL (with LOOP): the workgroup has two sets of strip wavefronts, each with token rows and
// reduction words of its own, which work on two tokens at a time with the one copy of the R1
// terms in LDS: where LDS lets only one workgroup be resident, a SIMD then has two independent
// MFMA chains to interleave instead of one.  Both sets pass the same barriers; a set without a
// token left repeats the last one and stores nothing.
template <int ATM, bool LOOP, bool DUAL = false>
__device__ __forceinline__ void rotate3_token(char* lds, const uint16_t* __restrict__ X, int64_t t_first,
                                              int64_t t_stride, int64_t M, int64_t K, int n1, int n2,
                                              const uint16_t* __restrict__ R1p,
                                              const uint16_t* __restrict__ R2p, int8_t* __restrict__ q,
                                              float* __restrict__ scale, int32_t* __restrict__ qsum,
                                              float* __restrict__ tmode = nullptr,
                                              int tp = 0, float qmax = 31.0f, bool asym = false,
                                              bool shift = false) {
    const R3Shape sh = r3_shape(n1, n2);
    const int tid_all = threadIdx.x;
    const int wv = __builtin_amdgcn_readfirstlane(tid_all >> 6);
    const int grp = DUAL ? (wv >= sh.strips ? 1 : 0) : 0;              // which of the two tokens in flight
    const int wave = wv - grp * sh.strips;                             // = strip
    const int tid = tid_all - grp * 64 * sh.strips, lane = tid & 63;
    // the workgroup may have more wavefronts than strips (the projection workgroups of the same
    // launch use them): those only help to fetch the R1 terms, or leave at once
    // (more than 8 tiles along n1 never fit LDS whole: no code for them)
    const bool early = !LOOP && ATM <= 8 && sh.resident;
    const bool helper = wave >= sh.strips;
    if (helper && !early) return;
    const int nthreads = 64 * sh.strips;
    const int nth_all = DUAL ? 2 * nthreads : nthreads;
    const int nfill = early ? (int)blockDim.x : nthreads;
    const int li = lane & 15, lg = lane >> 4;
    const int n1p16 = sh.at * 16, n1p32 = sh.ch2 * 32, n2p32 = sh.k1 * 32;
    char* vt = lds + grp * sh.r0bytes;                                 // token rows, later the code image
    char* cb = lds + (DUAL ? 2 : 1) * sh.r0bytes;                      // chunk buffers
    float* red = reinterpret_cast<float*>(cb + (size_t)(sh.alias ? 1 : sh.nbuf) * sh.cbytes) + grp * 64;

    // ---- packed R1 terms [term][n1p16][n1p32]: chunk ch = columns [32 ch, 32 ch + 32) of every row
    const int crow_items = 3 * n1p16 * 4;                              // 16-byte pieces per chunk
    auto chunk_src = [&](int ch, int item) -> const v4i* {
        const int row = item >> 2, piece = item & 3;                   // row = term * n1p16 + c
        return reinterpret_cast<const v4i*>(R1p + (int64_t)row * n1p32 + ch * 32 + piece * 8);
    };
    auto buf_base = [&](int buf) -> char* { return (sh.alias && buf == 1) ? lds : cb + buf * sh.cbytes; };
    auto chunk_dst = [&](int buf, int item) -> v4i* {
        return reinterpret_cast<v4i*>(buf_base(buf) + (item >> 2) * R3_CPITCH + (item & 3) * 16);
    };
    const int total = sh.ch2 * crow_items;
    const FastDiv dci(crow_items);
    v4i rp[R3_FILLR];
    auto rp_issue = [&]() {
#pragma unroll
        for (int e = 0; e < R3_FILLR; ++e) {
            if (e * nfill < total) {                   // (uniform: small factors need few rounds)
                const int g = tid + e * nfill;
                const int gc = g < total ? g : total - 1;
                const int ch = dci.div(gc);
                rp[e] = *chunk_src(ch, gc - ch * crow_items);
            }
        }
    };
    auto rp_store = [&]() {
#pragma unroll
        for (int e = 0; e < R3_FILLR; ++e) {
            const int g = tid + e * nfill;
            if (e * nfill < total && g < total) {
                const int ch = dci.div(g);
                *chunk_dst(ch, g - ch * crow_items) = rp[e];
            }
        }
        // what did not fit the first round
        for (int base = R3_FILLR * nfill; base < total; base += 8 * nfill) {
            v4i tmp[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int g = base + e * nfill + tid;
                const int gc = g < total ? g : total - 1;
                const int ch = dci.div(gc);
                tmp[e] = *chunk_src(ch, gc - ch * crow_items);
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int g = base + e * nfill + tid;
                if (g < total) {
                    const int ch = dci.div(g);
                    *chunk_dst(ch, g - ch * crow_items) = tmp[e];
                }
            }
        }
    };
    if (early && helper) {
        rp_issue();
        bwla_lds_barrier();                            // the barrier behind the token rows
        rp_store();
        return;                                        // (a wavefront ends only when its LDS writes have)
    }
    if (early) rp_issue();                             // first of all: the largest request of the token
    if (sh.resident && !early) {
        // all chunks at once, eight loads in flight per thread
        for (int base = 0; base < total; base += 8 * nth_all) {
            v4i tmp[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int g = base + e * nth_all + tid_all;
                const int gc = g < total ? g : total - 1;
                const int ch = gc / crow_items;
                tmp[e] = *chunk_src(ch, gc - ch * crow_items);
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int g = base + e * nth_all + tid_all;
                if (g < total) {
                    const int ch = g / crow_items;
                    *chunk_dst(ch, g - ch * crow_items) = tmp[e];
                }
            }
        }
    }
    // LOOP: resident factors and many tokens -- the workgroup keeps the factors and walks over
    // tokens t_first, t_first + t_stride, ...  Otherwise one token per workgroup (the body below is
    // then straight-line code).
    // (DUAL: workgroup b takes tokens 2 b and 2 b + 1, then 2 (b + stride), ...)
    int64_t tp0 = DUAL ? 2 * t_first : t_first;                         // first token of the round
#pragma nounroll
    do {
    const bool live = tp0 + grp < M;
    const int64_t t = live ? tp0 + grp : M - 1;
    // In a loop, lane-derived values are recomputed per token from an opaque copy of the thread
    // index: otherwise every address of the body is hoisted out of the loop and kept in registers.
    int tid_opaque = threadIdx.x;
    if constexpr (LOOP) asm volatile("" : "+v"(tid_opaque));
    const int tid = tid_opaque - grp * 64 * sh.strips, lane = tid & 63, li = lane & 15, lg = lane >> 4;
    // ---- R2 terms of my strip: rows d = 16*strip + li of the packed [term][n2p16][n2p32] planes
    // (read again for every token: kept across the token loop they would not fit the register
    // budget; the opaque zero keeps the loads inside the loop)
    int opaque_zero = 0;
    if constexpr (LOOP) asm volatile("" : "+s"(opaque_zero));
    v4i bfr[R3_MAXK1][3];
#pragma unroll
    for (int kb = 0; kb < R3_MAXK1; ++kb)
#pragma unroll
        for (int p = 0; p < 3; ++p) {
            bfr[kb][p] = v4i{0, 0, 0, 0};
            if (kb < sh.k1)
                bfr[kb][p] = *reinterpret_cast<const v4i*>(R2p + ((int64_t)(p * sh.strips * 16 + wave * 16 + li)) * n2p32 +
                                                           kb * 32 + 8 * lg + opaque_zero);
        }

    // streaming: the loads of chunks 0 and 1 are issued before the token rows are filled, so that
    // all of them share one memory round trip
    v4i ring[R3_ITEMS], first[R3_ITEMS];
    if (!sh.resident) {
#pragma unroll
        for (int e = 0; e < R3_ITEMS; ++e) {
            const int it = tid + e * nthreads;
            const int ic = it < crow_items ? it : crow_items - 1;
            first[e] = *chunk_src(0, ic);
            ring[e] = *chunk_src(sh.ch2 > 1 ? 1 : 0, ic);
        }
    }
    // ---- token rows into LDS (bf16 as stored; zero padding), 8 elements per item, eight loads
    // in flight per thread
    {
        const int per_row = n2p32 >> 3, items = n1p16 * per_row;
        const uint16_t* xrow = X + t * K;
        const FastDiv dpr(per_row);
        if ((n2 & 7) == 0) {
            for (int base = 0; base < items; base += 8 * nthreads) {
                v4i tmp[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int it = base + e * nthreads + tid;
                    const int a = dpr.div(it), b0 = (it - a * per_row) << 3;
                    const bool in = it < items && a < n1 && b0 < n2;
                    const v4i v = *reinterpret_cast<const v4i*>(xrow + (in ? (int64_t)a * n2 + b0 : 0));
                    tmp[e] = in ? v : v4i{0, 0, 0, 0};
                }
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int it = base + e * nthreads + tid;
                    if (it < items) {
                        const int a = dpr.div(it), b0 = (it - a * per_row) << 3;
                        *reinterpret_cast<v4i*>(vt + a * sh.vpitch + b0 * 2) = tmp[e];
                    }
                }
            }
        } else if ((n2 & 1) == 0) {
            // rows start on 4-byte boundaries only: four 4-byte loads per item, eight items in flight
            const uint32_t* x32 = reinterpret_cast<const uint32_t*>(xrow);
            for (int base = 0; base < items; base += 8 * nthreads) {
                uint32_t tmp[8][4];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int it = base + e * nthreads + tid;
                    const int a = dpr.div(it), b0 = (it - a * per_row) << 3;
#pragma unroll
                    for (int p = 0; p < 4; ++p) {
                        const bool in = it < items && a < n1 && b0 + 2 * p < n2;
                        const uint32_t v = x32[in ? ((a * n2 + b0) >> 1) + p : 0];
                        tmp[e][p] = in ? v : 0u;
                    }
                }
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int it = base + e * nthreads + tid;
                    if (it < items) {
                        const int a = dpr.div(it), b0 = (it - a * per_row) << 3;
                        *reinterpret_cast<v4i*>(vt + a * sh.vpitch + b0 * 2) =
                            v4i{(int)tmp[e][0], (int)tmp[e][1], (int)tmp[e][2], (int)tmp[e][3]};
                    }
                }
            }
        } else {
            for (int it = tid; it < items; it += nthreads) {
                const int a = dpr.div(it), b0 = (it - a * per_row) << 3;
                uint32_t w[4] = {0u, 0u, 0u, 0u};
                if (a < n1) {
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        if (b0 + e < n2) w[e >> 1] |= (uint32_t)xrow[(int64_t)a * n2 + b0 + e] << (16 * (e & 1));
                }
                *reinterpret_cast<v4i*>(vt + a * sh.vpitch + b0 * 2) = v4i{(int)w[0], (int)w[1], (int)w[2], (int)w[3]};
            }
        }
    }
    if (!sh.resident) {
#pragma unroll
        for (int e = 0; e < R3_ITEMS; ++e) {
            const int it = tid + e * nthreads;
            if (it < crow_items) *chunk_dst(0, it) = first[e];
        }
    }
    // (a barrier that orders LDS only: loads of later stages, and in a loop the stores of the
    // round before, stay in flight)
    bwla_lds_barrier();

    // ---- stage 1
    v4f z[ATM];
#pragma unroll
    for (int ta = 0; ta < ATM; ++ta) z[ta] = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int g = 0; g < ATM / 2; ++g) {
        if (2 * g < sh.at) {
            const int t0 = 2 * g, t1 = 2 * g + 1 < sh.at ? 2 * g + 1 : 2 * g;      // an odd last tile is done twice
            const char* a0p = vt + (t0 * 16 + li) * sh.vpitch + lg * 16;
            const char* a1p = vt + (t1 * 16 + li) * sh.vpitch + lg * 16;
#pragma unroll
            for (int kb = 0; kb < R3_MAXK1; ++kb) {
                if (kb < sh.k1) {
                    const v8bf a0 = __builtin_bit_cast(v8bf, *reinterpret_cast<const v4i*>(a0p + kb * 64));
                    const v8bf a1 = __builtin_bit_cast(v8bf, *reinterpret_cast<const v4i*>(a1p + kb * 64));
#pragma unroll
                    for (int p = 2; p >= 0; --p) {                     // small terms first
                        const v8bf b = __builtin_bit_cast(v8bf, bfr[kb][p]);
                        z[2 * g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, b, z[2 * g], 0, 0, 0);
                        z[2 * g + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, b, z[2 * g + 1], 0, 0, 0);
                    }
                }
            }
        }
    }
    if ((sh.at & 1) != 0) {                                            // the duplicate of an odd last tile
#pragma unroll
        for (int ta = 1; ta < ATM; ta += 2)
            if (ta == sh.at) z[ta] = v4f{0.f, 0.f, 0.f, 0.f};
    }

    // ---- stage 2: chunk ch contracts a in [32 ch, 32 ch + 32) = accumulator tiles 2 ch, 2 ch + 1
    if (early) {
        rp_store();
        bwla_lds_barrier();
    }
    if (sh.alias) __syncthreads();                     // the token rows make room for a chunk buffer
    v4f y[ATM];
#pragma unroll
    for (int tc = 0; tc < ATM; ++tc) y[tc] = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ch = 0; ch < ATM / 2; ++ch) {
        if (ch < sh.ch2) {
            int buf = ch;
            if (!sh.resident) {
                buf = ch & 1;
                // chunk ch + 1 from the registers into the other buffer (its readers passed the
                // barrier that closed chunk ch - 1), then chunk ch + 2 into the registers
#pragma unroll
                for (int e = 0; e < R3_ITEMS; ++e) {
                    const int it = tid + e * nthreads;
                    if (it < crow_items && ch + 1 < sh.ch2) *chunk_dst((ch + 1) & 1, it) = ring[e];
                }
#pragma unroll
                for (int e = 0; e < R3_ITEMS; ++e) {
                    const int it = tid + e * nthreads;
                    if (it < crow_items && ch + 2 < sh.ch2) ring[e] = *chunk_src(ch + 2, it);
                }
            }
            const float f[8] = {z[2 * ch][0], z[2 * ch][1], z[2 * ch][2], z[2 * ch][3],
                                z[2 * ch + 1][0], z[2 * ch + 1][1], z[2 * ch + 1][2], z[2 * ch + 1][3]};
            v8bf a1, a2, a3;
            r3_split3(f, a1, a2, a3);
            const char* cbase = buf_base(buf) + li * R3_CPITCH + lg * 16;
#pragma unroll
            for (int g = 0; g < ATM / 2; ++g) {
                if (2 * g < sh.at) {
                    const int c0 = 2 * g, c1 = 2 * g + 1 < sh.at ? 2 * g + 1 : 2 * g;
                    v8bf b0[3], b1[3];
#pragma unroll
                    for (int p = 0; p < 3; ++p) {
                        b0[p] = __builtin_bit_cast(v8bf, *reinterpret_cast<const v4i*>(cbase + (p * n1p16 + c0 * 16) * R3_CPITCH));
                        b1[p] = __builtin_bit_cast(v8bf, *reinterpret_cast<const v4i*>(cbase + (p * n1p16 + c1 * 16) * R3_CPITCH));
                    }
                    // the six products whose error is below fp32 rounding, small ones first
                    y[2 * g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a3, b0[0], y[2 * g], 0, 0, 0);
                    y[2 * g + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a3, b1[0], y[2 * g + 1], 0, 0, 0);
                    y[2 * g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, b0[2], y[2 * g], 0, 0, 0);
                    y[2 * g + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, b1[2], y[2 * g + 1], 0, 0, 0);
                    y[2 * g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a2, b0[1], y[2 * g], 0, 0, 0);
                    y[2 * g + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a2, b1[1], y[2 * g + 1], 0, 0, 0);
                    y[2 * g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a2, b0[0], y[2 * g], 0, 0, 0);
                    y[2 * g + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a2, b1[0], y[2 * g + 1], 0, 0, 0);
                    y[2 * g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, b0[1], y[2 * g], 0, 0, 0);
                    y[2 * g + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, b1[1], y[2 * g + 1], 0, 0, 0);
                    y[2 * g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, b0[0], y[2 * g], 0, 0, 0);
                    y[2 * g + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, b1[0], y[2 * g + 1], 0, 0, 0);
                }
            }
            if (!sh.resident) __syncthreads();                         // chunk ch + 1 is published, chunk ch is free
        }
    }

    // ---- per-token max magnitude (padded rows and columns are exact zeros)
    // (symmetric codes need the largest magnitude only: one reduction, stored as hi = -lo)
    float mx = 0.0f, mn = 0.0f;
    if (asym) {
#pragma unroll
        for (int tc = 0; tc < ATM; ++tc)
            if (tc < sh.at) {
#pragma unroll
                for (int v = 0; v < 4; ++v) { mx = fmaxf(mx, y[tc][v]); mn = fminf(mn, y[tc][v]); }
            }
        mx = bwla_wave_max(mx);
        mn = -bwla_wave_max(-mn);
    } else {
#pragma unroll
        for (int tc = 0; tc < ATM; ++tc)
            if (tc < sh.at) {
#pragma unroll
                for (int v = 0; v < 4; ++v) mx = fmaxf(mx, fabsf(y[tc][v]));
            }
        mx = bwla_wave_max(mx);
        mn = -mx;
    }
    if (lane == 0) { red[wave] = mx; red[32 + wave] = mn; }
    bwla_lds_barrier();                                // also: every wave is done with the token rows
    // over the strips (at most ten): one word per lane of a 16-lane row, four exchange steps
    const int s16 = lane & 15;
    float hi = s16 < sh.strips ? red[s16] : 0.0f;
#pragma unroll
    for (int off = 8; off > 0; off >>= 1) hi = fmaxf(hi, __shfl_xor(hi, off, 64));
    float lo = -hi;
    if (asym) {
        lo = s16 < sh.strips ? red[32 + s16] : 0.0f;
#pragma unroll
        for (int off = 8; off > 0; off >>= 1) lo = fminf(lo, __shfl_xor(lo, off, 64));
    }
    const QuantPlan qp = quant_plan(hi, lo, qmax, asym);

    // ---- quantize: lane holds Yt[d = 16*strip + 4*lg + v][c = 16*tc + li], four consecutive d of one c
    // (one token per workgroup and rows of whole words: the codes go straight to global memory,
    // 16 bytes of a row per lane group; else through an image in LDS and out in 16-byte pieces)
    int8_t* codes = reinterpret_cast<int8_t*>(vt);
    const bool direct = !LOOP && (n2 & 3) == 0;
    int8_t* qrow = q + t * K;
    int lsum = 0;
    const int d0 = wave * 16 + 4 * lg;
#pragma unroll
    for (int tc = 0; tc < ATM; ++tc) {
        if (tc < sh.at) {
            const int c = tc * 16 + li;
            int code[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) code[v] = quant_code(y[tc][v], qp);
            if (c < n1) {
                if ((n2 & 3) == 0) {
                    if (d0 < n2) {
                        const int word = (code[0] & 0xff) | ((code[1] & 0xff) << 8) | ((code[2] & 0xff) << 16) |
                                         (code[3] << 24);
                        if (direct) *reinterpret_cast<int*>(qrow + c * n2 + d0) = word;
                        else *reinterpret_cast<int*>(codes + c * n2 + d0) = word;
                        lsum += code[0] + code[1] + code[2] + code[3];
                    }
                } else {
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        if (d0 + v < n2) {
                            codes[c * n2 + d0 + v] = (int8_t)code[v];
                            lsum += code[v];
                        }
                }
            }
        }
    }
    lsum = bwla_wave_sum_i32(lsum);
    int* redi = reinterpret_cast<int*>(red) + 16;
    if (lane == 0) redi[wave] = lsum;
    bwla_lds_barrier();
    if (live) {
        if (!direct) {
            const uint4* src = reinterpret_cast<const uint4*>(codes);
            uint4* dst = reinterpret_cast<uint4*>(q + t * K);
            const int n16 = (int)(K >> 4);
            for (int idx = tid; idx < n16; idx += nthreads) dst[idx] = src[idx];
        }
        if (wave == 0) {
            int tot = s16 < sh.strips ? redi[s16] : 0;
#pragma unroll
            for (int off = 8; off > 0; off >>= 1) tot += __shfl_xor(tot, off, 64);
            if (lane == 0) {
                qsum[t] = tot;
                const float sc = quant_scale(hi, lo, qmax, asym);
                scale[t] = sc;
                quant_extras(tmode, tp, t, asym, shift, qp, sc, tot, K);
            }
        }
    }
    // the code image and the reduction words are free again (LDS only: the round's stores to
    // global memory need not have landed)
    if constexpr (LOOP) bwla_lds_barrier();
    tp0 += DUAL ? 2 * t_stride : t_stride;
    } while (LOOP && tp0 < M);
}

}  // namespace
