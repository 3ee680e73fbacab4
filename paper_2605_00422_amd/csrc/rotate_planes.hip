// Rotation + quantization of many bf16 tokens (prefill; paper Sec. 3.1, Sec. 4.1) with the factors
// resident: one workgroup per CU keeps all of R1 in LDS and its strip of R2 in registers, and walks
// over its share of the tokens.
//
//   stage 1  Z[a,d]  = sum_b V[a,b] R2[b,d]       V: the token's n1 x n2 reshape
//   stage 2  Yt[d,c] = sum_a Z[a,d] R1[a,c]       x~[c n2 + d] = Yt[d,c]
//
// Both stages run on fp16 MFMA (16x16x32) with fp32 accumulation and two-term operands:
//   - the token is scaled by a power of two (its largest magnitude into [2^2, 2^3)) and is then
//     exact in fp16 (bf16 has 8 significant bits; values 2^17 times smaller than the largest lose
//     bits, 2^-28 of it at most), one term;
//   - R1 and R2 are stored at pack time as two fp16 terms of 256 R (22 bits), in the order in which
//     an MFMA lane reads them (1 KiB per operand, no padding, no bank conflicts);
//   - Z (fp32 accumulators, |256 Z| <= 256 sqrt(n2) max|V| < 2^15: inside the fp16 range as it stands)
//     is split into two fp16 terms in registers; of the four products of stage 2 the smallest
//     (lo x lo, 2^-22 of the result) is left out.
// Stage 1 leaves its accumulator tiles in exactly the register layout of a stage-2 A operand, so a
// wavefront alternates: the two 16-row tiles of Z for contraction step ch (2 K1 x 2 MFMAs), then
// their products with R1 into all output tiles (3 n1/16 MFMAs) -- Z is never whole anywhere.
// Wavefront w owns the 16 columns d of strip w.  Tokens are pipelined through registers: while the
// wavefronts work on token j out of LDS, token j + 1 is in flight from HBM into registers, and is
// converted and written to LDS between the two barriers that every token costs.  G groups of
// n2 / 16 wavefronts work on G tokens at a time over the one copy of R1 (small factors would
// otherwise leave most of a CU's SIMDs with a single wavefront).
#include "bwla_internal.h"
#include "rotate_common.h"
#include "wave_dpp.h"

namespace {

typedef _Float16 v8h_r __attribute__((ext_vector_type(8)));

struct RpArgs {
    const uint16_t* X; int64_t M;
    const uint16_t* R2h; const uint16_t* R1h;
    int8_t* q; float* scale; int32_t* qsum;
    float* tmode; int tp; float qmax; int asym, shift;
};

template <int N1, int N2, int G, bool STREAM = false>
struct RpShape {
    static constexpr int K = N1 * N2, AT = N1 / 16, K1 = N2 / 32, CH2 = N1 / 32, STRIPS = N2 / 16;
    static constexpr int GPR = N2 / 8;                  // 16-byte granules (8 values) per token row
    static constexpr int PITCH = N2 * 2 + 16;           // bytes per token row in LDS (fp16), padded
    static constexpr int TG = 64 * STRIPS;              // threads of a group
    static constexpr int THREADS = TG * G;
    static constexpr int ITEMS = N1 * GPR;              // granules per token
    static constexpr int NI = (ITEMS + TG - 1) / TG;    // granules per thread
    static constexpr int CHUNK_BYTES = 2 * AT * 1024;   // both terms of one 32-deep step of R1
    static constexpr int R1_BYTES = STREAM ? 2 * CHUNK_BYTES : CH2 * CHUNK_BYTES;
    static constexpr int XT_BYTES = N1 * PITCH;
    static constexpr int RED_WORDS = 64;                // per group: [0,16) maxima, [16,32) minima, [32,48) token maxima, [48,64) code sums
    static constexpr size_t LDS = (size_t)R1_BYTES + (size_t)G * XT_BYTES + (size_t)G * RED_WORDS * 4;
};

template <int N1, int N2, int G, bool STREAM = false>
__global__ __launch_bounds__((N2 / 16) * 64 * G) void rotate_planes_kernel(RpArgs a) {
    using S = RpShape<N1, N2, G, STREAM>;
    static_assert(!STREAM || G == 1, "streamed R1 terms: one token group");
    constexpr int K = S::K, AT = S::AT, K1 = S::K1, CH2 = S::CH2, STRIPS = S::STRIPS, GPR = S::GPR, PITCH = S::PITCH;
    constexpr int TG = S::TG, NI = S::NI, ITEMS = S::ITEMS;
    extern __shared__ __align__(16) char lds[];
    const int wv = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    const int grp = wv / STRIPS, wave = wv - grp * STRIPS;             // token group, strip
    const int tid = (int)threadIdx.x - grp * TG, lane = tid & 63, li = lane & 15, lg = lane >> 4;
    char* r1 = lds;
    char* xt = lds + S::R1_BYTES + grp * S::XT_BYTES;
    float* red = reinterpret_cast<float*>(lds + S::R1_BYTES + G * S::XT_BYTES) + grp * S::RED_WORDS;
    int* redi = reinterpret_cast<int*>(red) + 48;

    // ---- R1 terms: global -> LDS asynchronously, one KiB per wavefront-wide request.  Resident: all
    // of them, once.  STREAM (R1 too large for LDS): the 2 AT blocks of one 32-deep step at a time into
    // one of two buffers, step g = (token round) * CH2 + ch into buffer g & 1, requested while the
    // step before it is worked on.
    constexpr int NB1 = CH2 * 2 * AT, NW = STRIPS * G;
    auto request_chunk = [&](int g) {
        const int ch = g % CH2;
        for (int b = wv; b < 2 * AT; b += NW)
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void*)(a.R1h + ((ch * 2 * AT + b) * 64 + lane) * 8),
                (__attribute__((address_space(3))) void*)(r1 + (g & 1) * S::CHUNK_BYTES + b * 1024), 16, 0, 0);
    };
    if constexpr (STREAM) {
        request_chunk(0);
    } else {
        for (int b = wv; b < NB1; b += NW)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(a.R1h + (b * 64 + lane) * 8),
                                             (__attribute__((address_space(3))) void*)(r1 + b * 1024), 16, 0, 0);
    }
    // ---- R2 terms of my strip, kept in registers over all tokens
    v8h_r bh[K1], bl[K1];
#pragma unroll
    for (int kb = 0; kb < K1; ++kb) {
        bh[kb] = __builtin_bit_cast(v8h_r, *reinterpret_cast<const v4i*>(a.R2h + (((wave * K1 + kb) * 2 + 0) * 64 + lane) * 8));
        bl[kb] = __builtin_bit_cast(v8h_r, *reinterpret_cast<const v4i*>(a.R2h + (((wave * K1 + kb) * 2 + 1) * 64 + lane) * 8));
    }

    // token of round j for my group; a group without a token left repeats the last one and stores nothing
    const int64_t tstep = (int64_t)gridDim.x * G;
    const int64_t t0 = (int64_t)blockIdx.x * G + grp;
    const int rounds = (int)((a.M + tstep - 1) / tstep);
    v4i xpre[NI];
    auto request = [&](int64_t t) {
        const uint16_t* xrow = a.X + (t < a.M ? t : a.M - 1) * K;
#pragma unroll
        for (int e = 0; e < NI; ++e) {
            const int it = tid + e * TG;
            xpre[e] = *reinterpret_cast<const v4i*>(xrow + (it < ITEMS ? it : 0) * 8);
        }
    };
    // largest magnitude of the token in registers: bf16 magnitudes order like their 15 low bits
    auto token_max = [&]() -> float {
        typedef unsigned short us2 __attribute__((ext_vector_type(2)));
        us2 m = us2{0, 0};
#pragma unroll
        for (int e = 0; e < NI; ++e)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                m = __builtin_elementwise_max(m, __builtin_bit_cast(us2, (uint32_t)xpre[e][i] & 0x7fff7fffu));
        const uint32_t top = m.x > m.y ? m.x : m.y;
        return dl_wave_max_nonneg(__uint_as_float(top << 16));
    };
    // the token in registers -> fp16 rows in LDS, scaled by sx = 2^ex
    auto land = [&](float sx) {
#pragma unroll
        for (int e = 0; e < NI; ++e) {
            const int it = tid + e * TG;
            if (it < ITEMS) {
                v4i o;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t w = (uint32_t)xpre[e][i];
                    const auto h2 = __builtin_amdgcn_cvt_pkrtz(__uint_as_float(w << 16) * sx, __uint_as_float(w & 0xffff0000u) * sx);
                    o[i] = __builtin_bit_cast(int, h2);
                }
                const int row = it / GPR, g = it - row * GPR;
                *reinterpret_cast<v4i*>(xt + row * PITCH + g * 16) = o;
            }
        }
    };
    // power of two that puts a token's largest magnitude into [2^2, 2^3) (1 for an all-zero token)
    auto scale_of = [&](float xmax) -> float {
        int E = (__float_as_int(xmax) >> 23) & 0xff;
        E = E < 40 ? 40 : (E > 230 ? 230 : E);
        return xmax > 0.0f ? __int_as_float((127 + 2 + 127 - E) << 23) : 1.0f;
    };

    // ---- prologue: token 0 into LDS, token 1 into flight
    request(t0);
    {
        const float m = token_max();
        if (lane == 0) red[32 + wave] = m;
    }
    bwla_lds_barrier();
    float xmax = 0.0f;
#pragma unroll
    for (int w = 0; w < STRIPS; ++w) xmax = fmaxf(xmax, red[32 + w]);
    float sx = scale_of(xmax);
    land(sx);
    request(t0 + tstep);
    __builtin_amdgcn_s_waitcnt(0);                      // my share of the R1 terms has landed (and token 1)
    bwla_lds_barrier();

    for (int j = 0; j < rounds; ++j) {
        const int64_t t = t0 + (int64_t)j * tstep;
        const bool live = t < a.M;
        // ================================================================ the two stages, step by step
        // Every LDS operand is requested one step before the MFMAs that use it (a step: the four
        // MFMAs of one 32-deep piece of stage 1, or the three of one output tile of stage 2), so
        // that a wavefront does not stand still for an LDS round trip at every step.
        v4f y[AT];
#pragma unroll
        for (int tc = 0; tc < AT; ++tc) y[tc] = v4f{0.f, 0.f, 0.f, 0.f};
        auto ld_a = [&](int ch, int kb, int half) -> v4i {
            return *reinterpret_cast<const v4i*>(xt + (32 * ch + 16 * half + li) * PITCH + lg * 16 + kb * 64);
        };
        auto ld_b = [&](int ch, int term, int tc) -> v4i {
            if constexpr (STREAM)
                return *reinterpret_cast<const v4i*>(r1 + ((j * CH2 + ch) & 1) * S::CHUNK_BYTES + (term * AT + tc) * 1024 + lane * 16);
            else
                return *reinterpret_cast<const v4i*>(r1 + ((ch * 2 + term) * AT + tc) * 1024 + lane * 16);
        };
        v4i na0 = ld_a(0, 0, 0), na1 = ld_a(0, 0, 1);
#pragma unroll
        for (int ch = 0; ch < CH2; ++ch) {
            v4f z0 = v4f{0.f, 0.f, 0.f, 0.f}, z1 = z0;
            v4i nbh = v4i{0, 0, 0, 0}, nbl = nbh;
#pragma unroll
            for (int kb = 0; kb < K1; ++kb) {
                const v8h_r a0 = __builtin_bit_cast(v8h_r, na0), a1 = __builtin_bit_cast(v8h_r, na1);
                if (kb + 1 < K1) { na0 = ld_a(ch, kb + 1, 0); na1 = ld_a(ch, kb + 1, 1); }
                else if (!STREAM) { nbh = ld_b(ch, 0, 0); nbl = ld_b(ch, 1, 0); }
                z0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a0, bl[kb], z0, 0, 0, 0);      // small term first
                z1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a1, bl[kb], z1, 0, 0, 0);
                z0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a0, bh[kb], z0, 0, 0, 0);
                z1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a1, bh[kb], z1, 0, 0, 0);
            }
            // lane (li, lg) holds Z[a = 32 ch + 4 lg + v (z0), 32 ch + 16 + 4 lg + v (z1)][d = li]: the eight
            // contraction positions of an A operand, in the order the R1 terms were stored in.
            if constexpr (STREAM) {
                // this step's R1 terms have landed, everybody's share; the other buffer is free (all are
                // past the step before): the next step's terms go there while this one is worked on
                __builtin_amdgcn_s_waitcnt(0);
                bwla_lds_barrier();
                if (j + 1 < rounds || ch + 1 < CH2) request_chunk(j * CH2 + ch + 1);
                nbh = ld_b(ch, 0, 0); nbl = ld_b(ch, 1, 0);
            }
            v8h_r ah, al;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float f = e < 4 ? z0[e & 3] : z1[e & 3];
                const _Float16 h = (_Float16)f;
                ah[e] = h;
                al[e] = (_Float16)__builtin_fmaf((float)h, -1.0f, f);
            }
#pragma unroll
            for (int tc = 0; tc < AT; ++tc) {
                const v8h_r ch_ = __builtin_bit_cast(v8h_r, nbh), cl_ = __builtin_bit_cast(v8h_r, nbl);
                if (tc + 1 < AT) { nbh = ld_b(ch, 0, tc + 1); nbl = ld_b(ch, 1, tc + 1); }
                else if (ch + 1 < CH2) { na0 = ld_a(ch + 1, 0, 0); na1 = ld_a(ch + 1, 0, 1); }
                y[tc] = __builtin_amdgcn_mfma_f32_16x16x32_f16(al, ch_, y[tc], 0, 0, 0);
                y[tc] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ah, cl_, y[tc], 0, 0, 0);
                y[tc] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ah, ch_, y[tc], 0, 0, 0);
            }
        }
        // ================================================================ the token's range; the next token's largest value
        const float yun = 1.52587890625e-05f / sx;      // back from 256 R2, 256 R1 and the token's scale
        float mx = 0.0f, mn = 0.0f;
        if (a.asym) {
#pragma unroll
            for (int tc = 0; tc < AT; ++tc)
#pragma unroll
                for (int v = 0; v < 4; ++v) { mx = fmaxf(mx, y[tc][v]); mn = fminf(mn, y[tc][v]); }
            mx = dl_wave_max_nonneg(mx) * yun;
            mn = -dl_wave_max_nonneg(-mn) * yun;
        } else {
#pragma unroll
            for (int tc = 0; tc < AT; ++tc)
#pragma unroll
                for (int v = 0; v < 4; ++v) mx = fmaxf(mx, fabsf(y[tc][v]));
            mx = dl_wave_max_nonneg(mx) * yun;
            mn = -mx;
        }
        __builtin_amdgcn_s_waitcnt(0);                  // the next token is in registers
        const float nm = token_max();
        if (lane == 0) { red[wave] = mx; red[16 + wave] = mn; red[32 + wave] = nm; }
        bwla_lds_barrier();                             // also: everybody is done with the token rows
        float hi = 0.0f, lo = 0.0f;
        xmax = 0.0f;
#pragma unroll
        for (int w = 0; w < STRIPS; ++w) {
            hi = fmaxf(hi, red[w]);
            lo = fminf(lo, red[16 + w]);
            xmax = fmaxf(xmax, red[32 + w]);
        }
        const QuantPlan qp = quant_plan(hi, lo, a.qmax, a.asym != 0);
        // ================================================================ codes, straight to global memory
        // lane holds Yt[d = 16 strip + 4 lg + v][c = 16 tc + li]: four consecutive k = c n2 + d.
        // y * inv + (1.5 * 2^23 + zero point) rounds once, to an integer (ties to even) in the low
        // mantissa bits; clamped as a float, its low byte is the code.
        const float inv = qp.inv * yun, addc = 12582912.0f + qp.zc;
        const float cmin = 12582912.0f + qp.cmin, cmax = 12582912.0f + qp.cmax;
        int lsum = 0;
        int8_t* qrow = a.q + (live ? t : 0) * K;
#pragma unroll
        for (int tc = 0; tc < AT; ++tc) {
            uint32_t cb[4];
#pragma unroll
            for (int v = 0; v < 4; ++v)
                cb[v] = __float_as_uint(__builtin_amdgcn_fmed3f(__builtin_fmaf(y[tc][v], inv, addc), cmin, cmax));
            const uint32_t wlo = __builtin_amdgcn_perm(cb[1], cb[0], 0x0c0c0400u);     // bytes: cb0.b0, cb1.b0, 0, 0
            const uint32_t whi = __builtin_amdgcn_perm(cb[3], cb[2], 0x04000c0cu);     // bytes: 0, 0, cb2.b0, cb3.b0
            const uint32_t word = wlo | whi;
            if (live) *reinterpret_cast<uint32_t*>(qrow + (16 * tc + li) * N2 + 16 * wave + 4 * lg) = word;
            lsum = __builtin_amdgcn_sdot4((int)word, 0x01010101, lsum, false);
        }
        lsum = dl_wave_sum(lsum);
        if (lane == 0) redi[wave] = lsum;
        // ================================================================ next token into LDS, the one after into flight
        sx = scale_of(xmax);
        land(sx);
        if (j + 2 < rounds) request(t + 2 * tstep);
        bwla_lds_barrier();
        if (wave == 0 && live) {
            int tot = 0;
#pragma unroll
            for (int w = 0; w < STRIPS; ++w) tot += redi[w];
            if (lane == 0) {
                a.qsum[t] = tot;
                const float sc = quant_scale(hi, lo, a.qmax, a.asym != 0);
                a.scale[t] = sc;
                quant_extras(a.tmode, a.tp, t, a.asym != 0, a.shift != 0, qp, sc, tot, K);
            }
        }
    }
}

template <int N1, int N2, int G, bool STREAM = false>
hipError_t launch_planes(const RpArgs& a, int cus, hipStream_t st) {
    using S = RpShape<N1, N2, G, STREAM>;
    static_assert(S::LDS <= RQ_LDS_LIMIT, "the factors and the token rows have to fit LDS");
    static_assert(S::STRIPS <= 16 && N1 % 32 == 0 && N2 % 32 == 0, "shape outside the kernel's layout");
    hipError_t e = bwla_ensure_lds((const void*)rotate_planes_kernel<N1, N2, G, STREAM>, S::LDS);
    if (e != hipSuccess) return e;
    int64_t grid = (a.M + G - 1) / G;
    if (grid > cus) grid = cus;
    rotate_planes_kernel<N1, N2, G, STREAM><<<dim3((unsigned)grid), dim3(S::THREADS), S::LDS, st>>>(a);
    return hipGetLastError();
}

}  // namespace

// *done = false (nothing launched) when the shape has no kernel here: bf16 tokens, at least one
// per CU, a factor pair for which the operand-order planes exist and a kernel was built.
hipError_t bwla_launch_rotate_planes(const bwla_layer_t* L, const void* dX, int xdtype, int64_t M, int8_t* dq,
                                     float* dscale, int32_t* dqsum, float* dT, int act_bits, hipStream_t st,
                                     bool* done) {
    *done = false;
    const int n1 = L->n1, n2 = L->n2;
    if (xdtype != BWLA_X_BF16 || L->off_Rd == 0) return hipSuccess;
    const int cus = bwla_device_cus();
    if (M < (int64_t)cus) return hipSuccess;
    const char* blob = (const char*)L->d_blob;
    RpArgs a;
    a.X = (const uint16_t*)dX; a.M = M;
    a.R1h = (const uint16_t*)(blob + L->off_Rd + bwla_decode_planes_r2_bytes(n1, n2));
    a.R2h = a.R1h + bwla_planes_r1h_bytes(n1) / 2;
    a.q = dq; a.scale = dscale; a.qsum = dqsum;
    const int ru = bwla_rank_u(L);
    a.tp = L->r; a.tmode = L->mode != 0 ? dT + ru : nullptr;
    a.asym = (L->mode & BWLA_MODE_ASYM_ACT) ? 1 : 0; a.shift = (L->mode & BWLA_MODE_ROW_SHIFT) ? 1 : 0;
    a.qmax = (float)((1 << (act_bits - 1)) - 1);
    hipError_t e = hipSuccess;
    if (n1 == 160 && n2 == 160) e = launch_planes<160, 160, 1>(a, cus, st);
    else if (n1 == 128 && n2 == 64) e = launch_planes<128, 64, 4>(a, cus, st);
    else if (n1 == 64 && n2 == 64) e = launch_planes<64, 64, 4>(a, cus, st);
    else if (n1 == 224 && n2 == 128) e = launch_planes<224, 128, 1, true>(a, cus, st);     // R1 terms: 196 KB, streamed
    else return hipSuccess;
    if (e == hipSuccess) *done = true;
    return e;
}
