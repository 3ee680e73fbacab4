// One launch for a whole decode layer with a single bf16 token (the memory-bound case of paper
// Sec. 4.4): rotation (Sec. 3.1), INT6 codes, symmetric or asymmetric (Sec. 4.1), binary GEMM (Eq. 3-4), PSP
// branch (Sec. 3.2) and dequantization.
//
// A workgroup owns a few 16-channel tiles of the output and has eight wavefronts:
//   wavefronts 0..3  rotate the token (one 16-column strip of the n1 x n2 reshape each) and
//                    quantize it: the rotation of one token is about a megaflop fed from L2,
//                    cheaper to repeat in every workgroup than to hand its result around;
//   all eight        then contract the codes with the workgroup's sign bits, one 512-column chunk
//                    each, requested as soon as the rotation's operands have landed so that they
//                    stream from HBM while the token is rotated; afterwards each wavefront finishes one round
//                    of tiles (scale, alpha, PSP columns, store).
// The PSP projection T = x U is the one thing that is shared: U is 2 K r bytes, and reading it in
// every workgroup would cost more L2 bandwidth than the whole layer costs HBM bandwidth.  The
// first workgroups each project one eighth of K on fp16 MFMA (x scaled by a power of two per piece
// so that it fits fp16 exactly; U stored in B operand order) and leave their 8 x r partial sums
// in the scratch, each value in one 8-byte word with the call's epoch as a tag; every workgroup
// polls those words with device-scope loads while its rotation is still running, and adds the
// eight slices in slice order.  The epoch comes from the scratch and is bumped once per launch by
// the workgroup that is the last to have read it, so a word written by an earlier call can never
// pass for this call's, and nothing has to be cleared.
// What the kernel is bound by at these sizes is instruction issue and latency, not bandwidth, so
// the serial path is kept short: operands go global -> LDS asynchronously in the order in which
// an MFMA lane reads them (no repacking, no bank conflicts), reductions run on DPP row operations,
// codes are rounded by adding 1.5 * 2^23 (one fused multiply-add per code, round-half-even), and
// wavefronts meet through arrival counts in LDS instead of workgroup barriers wherever only some
// of them have to.
#include <type_traits>

#include "bwla_internal.h"
#include "rotate_common.h"
#include "wave_dpp.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 v8bf;
typedef _Float16 v8h __attribute__((ext_vector_type(8)));

constexpr int DL_THREADS = 512;      // eight wavefronts
constexpr int DL_TPW = 3;            // channel tiles per workgroup and round
constexpr int DL_MAXAT = 8;          // 16-row tiles along n1 (n1 <= 128)
constexpr int DL_MAXK1 = 2;          // 32-deep steps along n2 (n2 <= 64)
constexpr int DL_MAXJTU = 6;         // 16-column tiles of U (PSP rank <= 96)
constexpr int DL_MAXJTV = 7;         // 16-column tiles of V (one more when the layer's mode adds a column)
constexpr int DL_MAXROUNDS = 8;      // rounds of DL_TPW tiles per workgroup (more channels than that: two launches)
constexpr int DL_SLICES = 8;         // slices of K of the shared projection
static_assert(BWLA_WS_HEAD == 1024 + (uint64_t)DL_SLICES * 16 * DL_MAXJTU * 8, "the exchange area is the scratch's head");
constexpr int DL_PRODUCERS = 32;     // workgroups that project (each slice four times: the first to land serves)
constexpr int DL_SPIN_LIMIT = 1 << 22;

// (the pointers every wavefront needs for its first requests are kernel parameters of their own:
// the first 14 dwords of the kernel arguments are preloaded into SGPRs at wavefront launch, which
// takes the argument fetch -- a memory round trip -- out of the path to the first request)
struct DlArgs {
    int8_t* q; float* scale; int32_t* qsum; float* T;      // written by workgroup 0
    float* Y; int32_t* acc_out;
    unsigned* sync;                  // head of the scratch: [0] epoch, [16 (1 + i)] arrival count i < 8, from byte 1024 on the tagged sums
    int N, r, ru, row_tiles, rounds, shift;
    float qmax;                      // largest code, 2^(bits-1) - 1
};


// byte-wise negation of four packed int8 (no value is -128 here)
__device__ __forceinline__ int dl_neg_bytes(int x) {
    const unsigned nx = ~(unsigned)x;
    return (int)(((nx & 0x7f7f7f7fu) + 0x01010101u) ^ (nx & 0x80808080u));
}

// s_waitcnt immediate: at most n vector memory operations still outstanding (other counters not waited for)
constexpr int dl_vmcnt_imm(int n) { return (n & 15) | ((n >> 4) << 14) | (7 << 4) | (15 << 8); }

__device__ __forceinline__ void dl_async_16(const void* src, char* dst_block) {
    // lane l's 16 bytes land at dst_block + 16 l (the hardware's placement)
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                     (__attribute__((address_space(3))) void*)dst_block, 16, 0, 0);
}

// swizzle of the token rows in LDS: row a keeps its 16-byte granule g at slot g ^ dl_swz(a), so that
// the sixteen rows a lane group reads for one MFMA operand fall into sixteen different bank groups
__device__ __forceinline__ int dl_swz(int a, int gpr) { return gpr == 8 ? (a >> 1) & 7 : (a >> 2) & 3; }

// N1, N2: the Kronecker factors (compile-time: at these sizes the kernel is bound by the number of
// instructions on its serial path, and run-time shapes cost address arithmetic and branches).
// JTU, JTV: 16-column tiles of U and of V.  ASYM: asymmetric codes (their own instantiations, so that the
// symmetric path carries none of their instructions).
template <int N1, int N2, int JTU, int JTV, bool ASYM>
__global__ __launch_bounds__(DL_THREADS) void decode_layer_kernel(const uint16_t* __restrict__ pX,
                                                                  const uint16_t* __restrict__ pR1h,
                                                                  const uint16_t* __restrict__ pR2d,
                                                                  const uint4* __restrict__ pbits,
                                                                  const __half* __restrict__ pUt,
                                                                  const __half* __restrict__ pV,
                                                                  const __half* __restrict__ palpha, DlArgs a) {
    constexpr int K = N1 * N2, AT = N1 / 16, K1 = N2 / 32, CH2 = N1 / 32, STRIPS = N2 / 16, CHUNKS = K / 512;
    constexpr int GPR = N2 / 8;                        // 16-byte granules per token row: 8 or 4
    constexpr int SW = K / DL_SLICES, SWW = SW / 4;    // T: columns per slice and per wavefront of a producer
    constexpr int NKS = SWW / 32, RPU = 16 * JTU;      // T: 32-deep steps per wavefront; columns of U
    constexpr int NB1 = CH2 * 2 * AT;                  // 1 KiB blocks of the R1 terms
    static_assert(JTU == 0 || NKS >= 1, "a producer wavefront has at least one step");
    static_assert(STRIPS <= 4 && AT <= DL_MAXAT && CHUNKS <= 16 && CHUNKS >= 2, "shape outside the kernel's wavefront roles");
    extern __shared__ __align__(16) char lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 15, lg = lane >> 4;
    const int grid = (int)gridDim.x, blk = (int)blockIdx.x;

    // ---- LDS map
    char* xt = lds;                                    // token rows, bf16, K * 2 bytes, granules swizzled
    char* r1 = xt + 2 * K;                             // R1 terms [chunk][term][tile of c][lane * 16]: CH2 * 2 * AT KiB
    char* codes = r1 + CH2 * 2 * AT * 1024;            // K code bytes, k order
    char* xh = codes + K;                              // a producer's slice of the token as fp16: SW * 2 bytes
    float* red = reinterpret_cast<float*>(xh + 2 * SW);// [0..3] strip maxima, [4..7] strip code sums, [8..13] six arrival counts, [14] epoch, [16..19] strip minima
    float* tpart = red + 32;                           // [4 wavefronts][16 * DL_MAXJTU] partial T of a producer
    float* txl = tpart + 4 * 16 * DL_MAXJTU;           // [DL_SLICES][16 * DL_MAXJTU] the slices' sums, [DL_SLICES * ...] on: T
    float* tfin = txl + (DL_SLICES + 1) * 16 * DL_MAXJTU;   // [8 wavefronts][16 * DL_MAXJTV] T as an epilogue wavefront reads it
    int* part = reinterpret_cast<int*>(tfin + 8 * 16 * DL_MAXJTV);   // [rounds][DL_TPW][8 chunks][16 channels]

    // arrival counts (rotation wavefronts: token and R2 landed, maxima left, codes written; a producer's
    // wavefronts: partial sums left; wavefront 7: epoch read; rotation wavefronts again: R1 landed), zero before anybody bumps them: this
    // barrier costs nothing, every wavefront would otherwise wait here for its first operands
    int* cnt = reinterpret_cast<int*>(red) + 8;
    if (tid < 6) cnt[tid] = 0;
    bwla_lds_barrier();
    // A subset of the wavefronts meets without holding up the others: each bumps the count when it
    // is ready, and whoever needs them all waits until the count is full.  (The wait is bounded: a
    // wavefront that gave up would compute with incomplete operands, but the kernel always ends.)
    auto arrive = [&](int* c) {
        if (lane == 0) __hip_atomic_fetch_add(c, 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
    };
    auto await = [&](int* c, int n) {
        for (int spin = 0; spin < DL_SPIN_LIMIT; ++spin) {
            if (__hip_atomic_load(c, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) >= n) break;
            __builtin_amdgcn_s_sleep(1);
        }
    };
    auto meet = [&](int* c, int n) { arrive(c); await(c, n); };

    auto tile_id = [&](int rd, int t) -> int { return (rd * DL_TPW + t) * grid + blk; };
    auto tile_of = [&](int rd, int t) -> int {
        const int id = tile_id(rd, t);
        return id < a.row_tiles ? id : a.row_tiles - 1;
    };
    constexpr int GW = 8, CPW = (CHUNKS + GW - 1) / GW;
    const bool rotates = wave < STRIPS, contracts = wave < GW;
    const bool produces = JTU > 0 && wave >= 4 && blk < DL_PRODUCERS;     // my slice: blk & 7
    const int slice = blk & (DL_SLICES - 1);

    // Sign bits of my chunk for a round's tiles.  They are the bulk of the layer's bytes and are not
    // needed before the codes exist, so they are requested only once the rotation's operands have
    // landed: the weight stream then runs in the shadow of the rotation instead of holding up the
    // few kilobytes the rotation waits for.
    v4i wq[DL_TPW][CPW];
#pragma unroll
    for (int t = 0; t < DL_TPW; ++t)
#pragma unroll
        for (int i = 0; i < CPW; ++i) wq[t][i] = v4i{0, 0, 0, 0};
    auto request_bits = [&](int rd) {
#pragma unroll
        for (int t = 0; t < DL_TPW; ++t)
#pragma unroll
            for (int i = 0; i < CPW; ++i) {
                const int c = wave + i * GW;
                if (contracts && c < CHUNKS) {
                    const uint4 x = pbits[(tile_of(rd, t) * CHUNKS + c) * 64 + lane];
                    wq[t][i] = v4i{(int)x.x, (int)x.y, (int)x.z, (int)x.w};
                }
            }
    };
    // epilogue: round 0 is finished by wavefront 5, then 6, 7, 4, 3 .. 0 (wavefronts 4 and 7 have
    // errands of their own, and the rotation wavefronts' first requests are the ones everything
    // waits for); lane o < 16 * DL_TPW channel o & 15 of tile o >> 4
    const int my_round = wave >= 5 ? wave - 5 : (wave == 4 ? 3 : 7 - wave);
    constexpr int VQ = 2 * JTV;                        // 16-byte pieces of a V row
    v4i vrow[VQ > 0 ? VQ : 1];
    uint16_t alpha_raw = 0;
    auto epi_loads = [&](int rd) {
        const int ti = lane >> 4;
        if (ti < DL_TPW) {
            int n = tile_of(rd, ti) * 16 + (lane & 15);
            if (n >= a.N) n = a.N - 1;
            alpha_raw = reinterpret_cast<const uint16_t*>(palpha)[n];
#pragma unroll
            for (int i = 0; i < VQ; ++i) vrow[i] = *reinterpret_cast<const v4i*>(pV + n * (16 * JTV) + 8 * i);
        }
    };
    // ================================================================ requests, critical ones first
    v4i bfr[K1][3];                                    // R2 terms of my strip (rotation wavefronts)
    v4i xq = v4i{0, 0, 0, 0};                          // my piece of the token (a producer's wavefronts)
    v4i uop[NKS > 0 ? NKS : 1][JTU > 0 ? JTU : 1];
    unsigned epoch = 0;
    // (an ordinary load: the word was written by an earlier launch, and this launch moves it on only
    // after every workgroup has read it)
    if (JTU > 0 && wave == 7) epoch = *reinterpret_cast<const volatile unsigned*>(a.sync);
    if (rotates) {
        // the token, asynchronously into LDS: 1 KiB per instruction
#pragma unroll
        for (int i = 0; i < (2 * K / 1024 + STRIPS - 1) / STRIPS; ++i) {
            const int blkx = wave + i * STRIPS;
            if (blkx < 2 * K / 1024) {
                const int row = blkx * (64 / GPR) + lane / GPR;
                const int slot = lane & (GPR - 1);
                dl_async_16(pX + row * N2 + ((slot ^ dl_swz(row, GPR)) << 3), xt + blkx * 1024);
            }
        }
        // R2 terms of my strip and all R1 terms: stored block by block as the MFMAs read them, one
        // contiguous KiB per wavefront-wide request
#pragma unroll
        for (int kb = 0; kb < K1; ++kb)
#pragma unroll
            for (int p = 0; p < 3; ++p)
                bfr[kb][p] = *reinterpret_cast<const v4i*>(pR2d + (((wave * K1 + kb) * 3 + p) * 64 + lane) * 8);
        // (last, and the same number for every rotation wavefront: stage 1 does not wait for them)
        static_assert(NB1 % STRIPS == 0, "every rotation wavefront requests the same number of R1 blocks");
#pragma unroll
        for (int i = 0; i < NB1 / STRIPS; ++i) {
            const int b1 = wave + i * STRIPS;
            dl_async_16(pR1h + (b1 * 64 + lane) * 8, r1 + b1 * 1024);
        }
    } else if (produces) {
        // my SWW columns of the token (16 bytes from each of the first lanes) and of U
        const int col0 = slice * SW + (wave - 4) * SWW;
        if (lane * 8 < SWW) xq = *reinterpret_cast<const v4i*>(pX + col0 + lane * 8);
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks)
#pragma unroll
            for (int jt = 0; jt < JTU; ++jt)
                uop[ks][jt] = *reinterpret_cast<const v4i*>(pUt + ((jt * (K / 32) + col0 / 32 + ks) * 64 + lane) * 8);
    }

    // ================================================================ T = x U, a producer's slice
    if (produces) {
        float m = 0.0f;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t w = (uint32_t)xq[e];
            m = fmaxf(m, fmaxf(fabsf(__uint_as_float(w << 16)), fabsf(__uint_as_float(w & 0xffff0000u))));
        }
        m = dl_wave_max_nonneg(m);
        // power of two that puts the piece's largest magnitude into [2^13, 2^14): bf16 values are
        // then fp16 values exactly, unless they are 2^28 times smaller than that largest one
        int E = (__float_as_int(m) >> 23) & 0xff;
        E = E < 32 ? 32 : (E > 222 ? 222 : E);
        const float sc = __int_as_float((267 - E) << 23);
        const float t_unscale = __int_as_float((E - 13) << 23);
        if (lane * 8 < SWW) {
            v4i o;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t w = (uint32_t)xq[e];
                const auto h2 = __builtin_amdgcn_cvt_pkrtz(__uint_as_float(w << 16) * sc, __uint_as_float(w & 0xffff0000u) * sc);
                o[e] = __builtin_bit_cast(int, h2);
            }
            *reinterpret_cast<v4i*>(xh + ((wave - 4) * SWW + lane * 8) * 2) = o;
        }
        v4f tacc[JTU > 0 ? JTU : 1];
#pragma unroll
        for (int jt = 0; jt < (JTU > 0 ? JTU : 1); ++jt) tacc[jt] = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            // every row of the A operand is the token (the LDS writes above are this wavefront's own)
            const v8h av = __builtin_bit_cast(v8h, *reinterpret_cast<const v4i*>(xh + ((wave - 4) * SWW + 32 * ks + 8 * lg) * 2));
#pragma unroll
            for (int jt = 0; jt < JTU; ++jt)
                tacc[jt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(av, __builtin_bit_cast(v8h, uop[ks][jt]), tacc[jt], 0, 0, 0);
        }
        // row 0 of the result (lanes 0..15) is my part of the slice's sums
        if (lane < 16) {
#pragma unroll
            for (int jt = 0; jt < JTU; ++jt) tpart[(wave - 4) * 16 * DL_MAXJTU + 16 * jt + lane] = tacc[jt][0] * t_unscale;
        }
        arrive(cnt + 3);
    }
    if (JTU > 0 && wave == 7) {
        // the epoch has been read (the bump at the end of the kernel must not come before every
        // workgroup has): hand it to wavefront 4, and count this workgroup in
        if (lane == 0) {
            reinterpret_cast<unsigned*>(red)[14] = epoch;
            // (eight counts, 64 bytes apart, and nobody waits for the result: 256 arrivals at one
            // address would take microseconds)
            __hip_atomic_fetch_add(a.sync + 16 * (1 + (blk & 7)), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        arrive(cnt + 4);
    }
    if (!rotates) {
        // a wavefront that only contracts waits until the rotation's operands are there
        await(cnt + 5, STRIPS);
        request_bits(0);
        if (my_round < a.rounds) epi_loads(my_round);
    }
    if (JTU > 0 && wave == 4) {
        await(cnt + 4, 1);
        const unsigned tag = reinterpret_cast<const unsigned*>(red)[14] + 1u;
        unsigned long long* tx = reinterpret_cast<unsigned long long*>(a.sync + 256);
        if (blk < DL_PRODUCERS) {
            // the slice's sums: four wavefronts' parts in wavefront order; value and tag in one word
            await(cnt + 3, 4);
#pragma unroll
            for (int j = lane; j < RPU; j += 64) {
                float v = 0.0f;
#pragma unroll
                for (int w = 0; w < 4; ++w) v += tpart[w * 16 * DL_MAXJTU + j];
                __hip_atomic_store(tx + slice * 16 * DL_MAXJTU + j,
                                   ((unsigned long long)tag << 32) | (unsigned long long)__float_as_uint(v), __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }
    // All eight slices of this call: the words are asked for before the contraction and looked at
    // behind it, by when they have long been written; should one not carry the call's tag yet, the
    // wavefront polls (bounded; the producers wait for nobody).
    constexpr int NE = (DL_SLICES * RPU + 63) / 64;
    unsigned long long ent[NE > 0 ? NE : 1];
    // (two halves: the request, and -- behind the contraction -- the look at what came back, so that
    // the device-scope round trip is not waited for before the contraction starts)
    auto poll_request = [&](unsigned tag) {
        const unsigned long long* tx = reinterpret_cast<const unsigned long long*>(a.sync + 256);
#pragma unroll
        for (int i = 0; i < NE; ++i) {
            const int idx = lane + 64 * i, sl = idx / (RPU > 0 ? RPU : 1), j = idx - sl * RPU;
            ent[i] = (unsigned long long)tag << 32;
            if (sl < DL_SLICES) ent[i] = __hip_atomic_load(tx + sl * 16 * DL_MAXJTU + j, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    };
    auto poll_check = [&](unsigned tag) -> bool {
        bool ok = true;
#pragma unroll
        for (int i = 0; i < NE; ++i) ok = ok && (unsigned)(ent[i] >> 32) == tag;
        return __all(ok);
    };

    if (rotates) {
        // ---- operands landed: every rotation wavefront waits for its own asynchronous copies, then
        // for the other rotation wavefronts (the T wavefronts go on by themselves)
        // (loads return in the order of their requests: all but the R1 blocks, which came last)
        __builtin_amdgcn_s_waitcnt(dl_vmcnt_imm(NB1 / STRIPS));
        meet(cnt, STRIPS);
        // ============================================================ rotation, stage 1: Z = V R2
        v4f z[AT];
#pragma unroll
        for (int ta = 0; ta < AT; ++ta) z[ta] = v4f{0.f, 0.f, 0.f, 0.f};
        v8bf av[K1][AT];
#pragma unroll
        for (int kb = 0; kb < K1; ++kb)
#pragma unroll
            for (int ta = 0; ta < AT; ++ta) {
                const int row = ta * 16 + li;
                av[kb][ta] = __builtin_bit_cast(v8bf, *reinterpret_cast<const v4i*>(
                                 xt + row * (N2 * 2) + (((4 * kb + lg) ^ dl_swz(row, GPR)) << 4)));
            }
#pragma unroll
        for (int kb = 0; kb < K1; ++kb)
#pragma unroll
            for (int p = 2; p >= 0; --p) {             // small terms first
                const v8bf b = __builtin_bit_cast(v8bf, bfr[kb][p]);
#pragma unroll
                for (int ta = 0; ta < AT; ++ta) z[ta] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[kb][ta], b, z[ta], 0, 0, 0);
            }
        // ---- the R1 terms have landed, everybody's; from here on the weight stream may have the memory pipes
        __builtin_amdgcn_s_waitcnt(dl_vmcnt_imm(0));
        meet(cnt + 5, STRIPS);
        request_bits(0);
        if (my_round < a.rounds) epi_loads(my_round);
        // ============================================================ stage 2: Yt = Zt R1
        // The accumulator tiles of stage 1 are A operands as they stand: lane (li, lg) holds
        // Z[a = 16 ta + 4 lg + v][d = li]; two stacked tiles give the eight contraction positions
        // of a lane group in the order in which the R1 terms are stored.  Both operands as two fp16
        // terms (22 bits): Z of this strip scaled by a power of two so that its largest magnitude is
        // in [2^13, 2^14), R1 stored as 256 R1; of the four products the smallest (lo x lo, 2^-22 of
        // the result) is left out.  The scale is undone in the quantization step.
        float zm = 0.0f;
#pragma unroll
        for (int ta = 0; ta < AT; ++ta)
#pragma unroll
            for (int v = 0; v < 4; ++v) zm = fmaxf(zm, fabsf(z[ta][v]));
        zm = dl_wave_max_nonneg(zm);
        int Ez = (__float_as_int(zm) >> 23) & 0xff;
        Ez = Ez < 32 ? 32 : (Ez > 222 ? 222 : Ez);
        const float zsc = __int_as_float((267 - Ez) << 23);
        const float yun = __int_as_float((Ez - 13 - 8) << 23);       // back from the scaled Z and the 256 R1
        v4f y[AT];
#pragma unroll
        for (int tc = 0; tc < AT; ++tc) y[tc] = v4f{0.f, 0.f, 0.f, 0.f};
        v8h ah[CH2], al[CH2];
#pragma unroll
        for (int ch = 0; ch < CH2; ++ch)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float f = z[2 * ch + (e >> 2)][e & 3] * zsc;
                const _Float16 h = (_Float16)f;
                ah[ch][e] = h;
                al[ch][e] = (_Float16)(f - (float)h);
            }
#pragma unroll
        for (int ch = 0; ch < CH2; ++ch) {
            const char* cb = r1 + ch * 2 * AT * 1024 + lane * 16;
            v8h bh[AT], bl[AT];
#pragma unroll
            for (int tc = 0; tc < AT; ++tc) {
                bh[tc] = __builtin_bit_cast(v8h, *reinterpret_cast<const v4i*>(cb + (0 * AT + tc) * 1024));
                bl[tc] = __builtin_bit_cast(v8h, *reinterpret_cast<const v4i*>(cb + (1 * AT + tc) * 1024));
            }
            // small products first
#pragma unroll
            for (int tc = 0; tc < AT; ++tc) y[tc] = __builtin_amdgcn_mfma_f32_16x16x32_f16(al[ch], bh[tc], y[tc], 0, 0, 0);
#pragma unroll
            for (int tc = 0; tc < AT; ++tc) y[tc] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ah[ch], bl[tc], y[tc], 0, 0, 0);
#pragma unroll
            for (int tc = 0; tc < AT; ++tc) y[tc] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ah[ch], bh[tc], y[tc], 0, 0, 0);
        }
        // ============================================================ range of the token
        // symmetric codes: the largest magnitude; asymmetric codes (Sec. 4.1): the largest and the smallest
        // value, zero included
        float mx = 0.0f, mn = 0.0f;
        if constexpr (ASYM) {
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
        }
        // the rotation wavefronts exchange their extremes among themselves
        if (lane == 0) {
            red[wave] = mx;
            if constexpr (ASYM) red[16 + wave] = mn;
        }
        meet(cnt + 1, STRIPS);
        float amax = 0.0f, amin = 0.0f;
#pragma unroll
        for (int w = 0; w < STRIPS; ++w) {
            amax = fmaxf(amax, red[w]);
            if constexpr (ASYM) amin = fminf(amin, red[16 + w]);
        }
        // (factor on this strip's scaled values; the constant that rounds carries the zero point)
        float inv = amax > 0.0f ? a.qmax * __builtin_amdgcn_rcpf(amax) * yun : 0.0f, addc = 12582912.0f;
        if constexpr (ASYM) {
            const QuantPlan qp = quant_plan(amax, amin, a.qmax, true);
            inv = qp.inv * yun;
            addc = 12582912.0f + qp.zc;
        }
        const float cmin = 12582912.0f - (a.qmax + 1.0f), cmax = 12582912.0f + a.qmax;

        // ============================================================ codes
        // lane holds Yt[d = 16 strip + 4 lg + v][c = 16 tc + li]: four consecutive k = c n2 + d.
        // x * inv + 1.5 * 2^23 (+ zero point) rounds to an integer (ties to even) whose low byte is the
        // code; only asymmetric codes can leave their range (by one, at the top) and are clamped.
        int lsum = 0;
#pragma unroll
        for (int tc = 0; tc < AT; ++tc) {
            uint32_t cb[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                float f = __builtin_fmaf(y[tc][v], inv, addc);
                if constexpr (ASYM) f = __builtin_amdgcn_fmed3f(f, cmin, cmax);
                cb[v] = __float_as_uint(f);
            }
            const uint32_t lo = __builtin_amdgcn_perm(cb[1], cb[0], 0x0c0c0400u);      // bytes: cb0.b0, cb1.b0, 0, 0
            const uint32_t hi = __builtin_amdgcn_perm(cb[3], cb[2], 0x04000c0cu);      // bytes: 0, 0, cb2.b0, cb3.b0
            const uint32_t word = lo | hi;
            *reinterpret_cast<uint32_t*>(codes + (16 * tc + li) * N2 + 16 * wave + 4 * lg) = word;
            lsum = __builtin_amdgcn_sdot4((int)word, 0x01010101, lsum, false);
        }
        lsum = dl_wave_sum(lsum);
        if (lane == 0) reinterpret_cast<int*>(red)[4 + wave] = lsum;
        arrive(cnt + 2);                               // my codes and my code sum are in LDS
    }

    // ================================================================ binary GEMM on the workgroup's tiles
    if (contracts) {
        await(cnt + 2, STRIPS);                        // the token's codes are complete
        // operand codes of my chunks: for digit class j the 16 codes at columns 512 c + 128 lg + 16 j
        // (every token column of the MFMA reads the one token; only column 0 is used)
        v4i b[CPW][8];
#pragma unroll
        for (int i = 0; i < CPW; ++i) {
            const int c = wave + i * GW;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                b[i][j] = v4i{0, 0, 0, 0};
                if (c < CHUNKS) b[i][j] = *reinterpret_cast<const v4i*>(codes + 512 * c + 128 * lg + 16 * j);
            }
            b[i][7] = v4i{dl_neg_bytes(b[i][7].x), dl_neg_bytes(b[i][7].y), dl_neg_bytes(b[i][7].z), dl_neg_bytes(b[i][7].w)};
        }
        bool t_here = false;
        const unsigned tag = JTU > 0 && wave == 4 ? reinterpret_cast<const unsigned*>(red)[14] + 1u : 0u;
        if (JTU > 0 && wave == 4) poll_request(tag);
        // workgroup 0 moves the epoch on once every workgroup has read it: its last wavefront asks
        // for the eight arrival counts here and looks at them behind the contraction
        const bool bumps = JTU > 0 && wave == 7 && blk == 0;
        unsigned seen = 0;
        auto count_arrivals = [&]() {
            seen = lane < 8 ? __hip_atomic_load(a.sync + 16 * (1 + lane), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0u;
        };
        if (bumps) count_arrivals();
        for (int rd = 0; rd < a.rounds; ++rd) {
            int* prt = part + rd * DL_TPW * 8 * 16;

            // the round's tiles (all DL_TPW of them, except in the last round) side by side: per tile
            // and chunk two independent chains through the accumulator (odd and even digit classes),
            // e = S6+S4+S2+S0, o = 2 (S7+S5+S3+S1), exact arithmetic shifts in between
            auto contract = [&](auto nt_) {
                constexpr int NT = decltype(nt_)::value;
                v4i acc_e[NT][CPW], acc_o[NT][CPW];
#pragma unroll
                for (int t = 0; t < NT; ++t)
#pragma unroll
                    for (int i = 0; i < CPW; ++i) acc_e[t][i] = acc_o[t][i] = v4i{0, 0, 0, 0};
#pragma unroll
                for (int jj = 3; jj >= 0; --jj) {
                    const int mo = 0x01010101 << (2 * jj + 1), me = 0x01010101 << (2 * jj);
#pragma unroll
                    for (int t = 0; t < NT; ++t)
#pragma unroll
                        for (int i = 0; i < CPW; ++i) {
                            const v4i w = wq[t][i];
                            const v4i xo = v4i{w.x & mo, w.y & mo, w.z & mo, w.w & mo};
                            acc_o[t][i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(xo, b[i][2 * jj + 1], acc_o[t][i], 0, 0, 0);
                            const v4i xe = v4i{w.x & me, w.y & me, w.z & me, w.w & me};
                            acc_e[t][i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(xe, b[i][2 * jj], acc_e[t][i], 0, 0, 0);
                        }
                    if (jj > 0) {
#pragma unroll
                        for (int t = 0; t < NT; ++t)
#pragma unroll
                            for (int i = 0; i < CPW; ++i) { acc_o[t][i] = acc_o[t][i] >> 2; acc_e[t][i] = acc_e[t][i] >> 2; }
                    }
                }
                // lane (li = token column, lg) holds channels 4 lg .. 4 lg + 3: column 0 is the token
                if (li == 0) {
#pragma unroll
                    for (int t = 0; t < NT; ++t) {
                        v4i sum = acc_e[t][0] + (acc_o[t][0] >> 1);
#pragma unroll
                        for (int i = 1; i < CPW; ++i) sum += acc_e[t][i] + (acc_o[t][i] >> 1);
                        *reinterpret_cast<v4i*>(prt + (t * 8 + wave) * 16 + 4 * lg) = sum;
                    }
                }
            };
            static_assert(DL_TPW == 3, "the dispatch below lists the tile counts");
            if (tile_id(rd, 2) < a.row_tiles) contract(std::integral_constant<int, 3>{});
            else if (tile_id(rd, 1) < a.row_tiles) contract(std::integral_constant<int, 2>{});
            else if (tile_id(rd, 0) < a.row_tiles) contract(std::integral_constant<int, 1>{});
            // next round's sign bits into the same registers
            if (rd + 1 < a.rounds) request_bits(rd + 1);
        }
        if (bumps) {
            for (int spin = 0; spin < DL_SPIN_LIMIT; ++spin) {
                if ((unsigned)dl_wave_sum((int)seen) == (unsigned)grid) break;
                __builtin_amdgcn_s_sleep(8);
                count_arrivals();
            }
            // (all have read it: the counts go back to zero, the epoch moves on; the next launch
            // sees both, being ordered behind this one)
            if (lane < 8) __hip_atomic_store(a.sync + 16 * (1 + lane), 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (lane == 0) __hip_atomic_store(a.sync, epoch + 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        if (JTU > 0 && wave == 4) {
            t_here = poll_check(tag);                  // what the request before the contraction brought
            for (int spin = 0; !t_here && spin < DL_SPIN_LIMIT; ++spin) {
                __builtin_amdgcn_s_sleep(8);
                poll_request(tag);
                t_here = poll_check(tag);
            }
#pragma unroll
            for (int i = 0; i < NE; ++i) {
                const int idx = lane + 64 * i;
                if (idx < DL_SLICES * RPU) txl[idx] = __uint_as_float((unsigned)ent[i]);
            }
            // T: the slices in slice order
#pragma unroll
            for (int j = lane; j < RPU; j += 64) {
                float v = 0.0f;
#pragma unroll
                for (int sl = 0; sl < DL_SLICES; ++sl) v += txl[sl * RPU + j];
                txl[DL_SLICES * 16 * DL_MAXJTU + j] = v;
            }
        }
    }

    // ---- partial sums of all rounds, code sums and partial T are in LDS
    bwla_lds_barrier();

    // token-wide values
    float amax = 0.0f, amin = 0.0f;
    int qs = 0;
#pragma unroll
    for (int w = 0; w < STRIPS; ++w) {
        amax = fmaxf(amax, red[w]);
        if constexpr (ASYM) amin = fminf(amin, red[16 + w]);
        qs += reinterpret_cast<const int*>(red)[4 + w];
    }
    // workgroup 0 also writes the token's codes out
    if (blk == 0) {
        for (int i = tid; i < (K >> 4); i += DL_THREADS)
            reinterpret_cast<uint4*>(a.q)[i] = reinterpret_cast<const uint4*>(codes)[i];
    }
    // ================================================================ epilogue: every wavefront its round
    if (my_round < a.rounds) {
        const int rd = my_round;
        const float st = ASYM ? quant_scale(amax, amin, a.qmax, true) : amax / a.qmax;
        const float zc = ASYM ? quant_plan(amax, amin, a.qmax, true).zc : 0.0f;
        const int jshift = a.ru + (ASYM ? 2 : 0);
        float* tf = tfin + wave * 16 * DL_MAXJTV;
        // T as the epilogue reads it: the PSP columns, then the columns the layer's mode adds
        // (asymmetric codes: -scale * zero point, twice; row shift: scale * sum of (code - zero point))
        if (JTV > 0) {
            for (int j = lane; j < 16 * JTV; j += 64) {
                float tv = 0.0f;
                if (j < a.ru) {
                    tv = txl[DL_SLICES * 16 * DL_MAXJTU + j];
                } else if (j < jshift) {
                    tv = -(st * zc);
                } else if (a.shift && j == jshift) {
                    tv = st * ((float)qs - (float)K * zc);
                }
                tf[j] = tv;
                if (blk == 0 && rd == 0 && j < a.r) a.T[j] = tv;
            }
        }
        // ... and workgroup 0 the token's scale and code sum
        if (blk == 0 && rd == 0 && lane == 0) { a.scale[0] = st; a.qsum[0] = qs; }
        const int* prt = part + rd * DL_TPW * 8 * 16;
        const int ti = lane >> 4, row = lane & 15;
        if (ti < DL_TPW) {
            const int tile = tile_id(rd, ti);
            const int n = tile * 16 + row;
            int tot = 0;
#pragma unroll
            for (int w = 0; w < GW; ++w) tot += prt[(ti * 8 + w) * 16 + row];
            const int ai = 2 * tot - qs;
            float low = 0.0f;
#pragma unroll
            for (int i = 0; i < VQ; ++i) {
                const v4f tq0 = *reinterpret_cast<const v4f*>(tf + 8 * i);
                const v4f tq1 = *reinterpret_cast<const v4f*>(tf + 8 * i + 4);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int vw = vrow[i][e];          // (a copy: a bit cast applied to a vector element reads element 0)
                    const __half2 h = __builtin_bit_cast(__half2, vw);
                    const float t0 = e < 2 ? tq0[2 * e] : tq1[2 * e - 4], t1 = e < 2 ? tq0[2 * e + 1] : tq1[2 * e - 3];
                    low = __builtin_fmaf(t0, __low2float(h), low);
                    low = __builtin_fmaf(t1, __high2float(h), low);
                }
            }
            const float yv = st * __half2float(__ushort_as_half(alpha_raw)) * (float)ai + low;
            if (tile < a.row_tiles && n < a.N) {
                a.Y[n] = yv;
                if (a.acc_out) a.acc_out[n] = ai;
            }
        }
    }
}

using DlKernel = void (*)(const uint16_t*, const uint16_t*, const uint16_t*, const uint4*, const __half*, const __half*,
                          const __half*, DlArgs);
// (asymmetric codes bring at least their two columns of V)
template <int N1, int N2, int JTU, int JTV>
DlKernel dl_kernel_for(bool asym) {
    if constexpr (JTV >= 1) {
        if (asym) return decode_layer_kernel<N1, N2, JTU, JTV, true>;
    }
    return decode_layer_kernel<N1, N2, JTU, JTV, false>;
}

size_t dl_lds_bytes(int K, int n1, int n2, bool with_t) {
    const int at = n1 >> 4, ch2 = n1 >> 5;
    (void)with_t;
    return (size_t)2 * K + (size_t)ch2 * 2 * at * 1024 + K + 2 * (K / DL_SLICES) +
           (32 + 4 * 16 * DL_MAXJTU + (DL_SLICES + 1) * 16 * DL_MAXJTU + 8 * 16 * DL_MAXJTV) * sizeof(float) +
           DL_MAXROUNDS * DL_TPW * 8 * 16 * sizeof(int);
}

}  // namespace


// Single-launch decode layer.  *done = false (and nothing launched) when the shape is outside what
// the kernel takes: one bf16 token; Kronecker factors of 32 or 64, or 128 x 64 (K = 1024 .. 8192, which
// covers the 4096- and 8192-wide models' attention and up/gate projections); PSP rank up to 96 (and then at least
// 512 output channels, so that the projection has its 32 producers); symmetric or asymmetric codes (the
// latter up to 7 bits), with or without the row shift.  dws_head: the first BWLA_WS_HEAD bytes of the caller's scratch.  With
// dry_run nothing is launched and *done only says whether the kernel would serve the call.
hipError_t bwla_launch_decode_layer(const bwla_layer_t* L, const void* dX, int xdtype, int64_t M, int8_t* dq,
                                    float* dscale, int32_t* dqsum, float* dT, void* dws_head, float* dY,
                                    int32_t* dacc, hipStream_t st, bool* done, bool dry_run, int act_bits) {
    *done = false;
    const int n1 = L->n1, n2 = L->n2;
    if (M != 1 || xdtype != BWLA_X_BF16) return hipSuccess;
    if ((n1 != 32 && n1 != 64 && n1 != 128) || (n2 != 32 && n2 != 64)) return hipSuccess;
    const bool asym = (L->mode & BWLA_MODE_ASYM_ACT) != 0;
    if (asym && act_bits > 7) return hipSuccess;          // (the stored code -128 has no negated byte)
    const int ru = bwla_rank_u(L), r = L->r;
    const int jtu = (ru + 15) >> 4, jtv = (r + 15) >> 4;
    if (jtu > DL_MAXJTU || jtv > DL_MAXJTV) return hipSuccess;
    if (asym && jtv < 1) return hipSuccess;               // (cannot be: the mode brings two columns)
    const int K = (int)L->K, chunks = (int)bwla_chunks(L->K), row_tiles = (int)bwla_row_tiles(L->N);
    if (chunks > 16 || chunks < 2 || (K & 511) != 0) return hipSuccess;
    const char* blob = (const char*)L->d_blob;
    const int cus = bwla_device_cus();
    const int grid = row_tiles < cus ? row_tiles : cus;
    DlArgs a;
    const uint16_t* pX = (const uint16_t*)dX;
    if (L->off_Rd == 0) return hipSuccess;
    const uint16_t* pR2d = (const uint16_t*)(blob + L->off_Rd);
    const uint16_t* pR1h = (const uint16_t*)(blob + L->off_Rd + bwla_decode_planes_r2_bytes(n1, n2));
    const uint4* pbits = (const uint4*)(blob + L->off_bits);
    const __half* palpha = (const __half*)(blob + L->off_alpha);
    const __half* pV = (const __half*)(blob + L->off_V);
    const __half* pUt = (const __half*)(blob + L->off_U);
    a.q = dq; a.scale = dscale; a.qsum = dqsum; a.T = dT; a.Y = dY; a.acc_out = dacc;
    a.N = (int)L->N; a.r = r; a.ru = ru; a.row_tiles = row_tiles;
    a.rounds = (row_tiles + DL_TPW * grid - 1) / (DL_TPW * grid);
    if (a.rounds > DL_MAXROUNDS) return hipSuccess;
    // the shared projection needs its producers (the first DL_PRODUCERS workgroups) and the exchange
    // area at the head of the scratch
    if (jtu > 0 && (grid < DL_PRODUCERS || dws_head == nullptr)) return hipSuccess;
    a.sync = (unsigned*)dws_head;
    a.shift = (L->mode & BWLA_MODE_ROW_SHIFT) ? 1 : 0;
    a.qmax = (float)((1 << (act_bits - 1)) - 1);
    const size_t lds = dl_lds_bytes(K, n1, n2, jtu > 0);
    auto launch = [&](auto kern) -> hipError_t {
        if (dry_run) return hipSuccess;                    // the caller only asks whether the shape is served
        hipError_t e = bwla_ensure_lds((const void*)kern, lds);
        if (e != hipSuccess) return e;
        kern<<<dim3((unsigned)grid), dim3(DL_THREADS), lds, st>>>(pX, pR1h, pR2d, pbits, pUt, pV, palpha, a);
        return hipGetLastError();
    };
    hipError_t e = hipSuccess;
    bool found = false;
#define DL_CASE(A_, B_, U_, V_) \
    if (n1 == A_ && n2 == B_ && jtu == U_ && jtv == V_) { found = true; e = launch(dl_kernel_for<A_, B_, U_, V_>(asym)); }
#define DL_RANKS(A_, B_) \
    DL_CASE(A_, B_, 0, 0) DL_CASE(A_, B_, 0, 1) DL_CASE(A_, B_, 1, 1) DL_CASE(A_, B_, 1, 2) DL_CASE(A_, B_, 2, 2) \
    DL_CASE(A_, B_, 2, 3) DL_CASE(A_, B_, 3, 3) DL_CASE(A_, B_, 3, 4) DL_CASE(A_, B_, 4, 4) DL_CASE(A_, B_, 4, 5)
    DL_RANKS(64, 64)
    // (ranks up to 96: the merged q|k|v projection of a 4096-wide block)
    DL_CASE(64, 64, 5, 5) DL_CASE(64, 64, 5, 6) DL_CASE(64, 64, 6, 6) DL_CASE(64, 64, 6, 7)
    // the smaller factor pairs with the ranks their widths would carry
    DL_CASE(32, 64, 0, 0) DL_CASE(32, 64, 1, 1) DL_CASE(32, 64, 2, 2) DL_CASE(64, 32, 0, 0) DL_CASE(64, 32, 1, 1)
    DL_CASE(64, 32, 2, 2) DL_CASE(32, 32, 0, 0) DL_CASE(32, 32, 1, 1)
    // 8192 columns (128 x 64: the 8192-wide models' attention and up / gate projections)
    DL_CASE(128, 64, 0, 0) DL_CASE(128, 64, 2, 2) DL_CASE(128, 64, 4, 4) DL_CASE(128, 64, 4, 5)
#undef DL_RANKS
#undef DL_CASE
    if (!found) return hipSuccess;                         // no kernel built for this pair: the caller's two launches
    if (e == hipSuccess) *done = true;
    return e;
}
