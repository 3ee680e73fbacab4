// bwla_rotate_quant: workgroups [0, M) rotate and quantize one token each; for up to 16
// tokens the workgroups behind them compute the PSP projection T = X U in the same launch.
//
// Rotation (paper Sec. 3.1; App. A.2.2), per token on the row-major n1 x n2 reshape V:
//   X~[t, c*n2 + d] = sum_{a,b} X[t, a*n2 + b] R1[a,c] R2[b,d]   =   (R1^T (V R2))[c,d]
//   stage 1  Z = V R2      stage 2  Y^T = Z^T R1        (fp32 MFMA 16x16x4)
// The token tile lives in LDS, Z^T replaces V in place (through the accumulators), and Y never
// leaves registers before it is quantized:
//   amax = max |Y|, scale = amax / 31, q = clamp(rint(Y * 31 / amax)), qsum = sum q.
// All LDS operands are laid out with the contraction index along the row, so a lane fetches the
// four contraction values of four MFMA steps with one 128-bit read.  When both factors fit into
// LDS next to the token they are loaded once, together with the token ("resident" mode: one
// global round trip, four barriers -- the decode case); otherwise they are streamed in chunks
// of 16 contraction indices through a register ring and an LDS double buffer.
//
// PSP projection (paper Sec. 3.2), T = X U from the un-rotated, un-quantized activations, few
// tokens: a workgroup takes 16 tokens x 512 columns of K, reads its operands (activations and
// the packed fp16 U) straight from global memory and multiplies on fp32 MFMA.  With several
// slices, every workgroup writes its partial tile to scratch and the one that arrives last adds
// them in slice order.

#include "bwla_internal.h"
#include "rotate_common.h"
#include "rotate_f32_device.h"
#include "rotate_bf16_device.h"
#include "rotate_split_device.h"
#include "psp_block_device.h"

namespace {

struct RqArgs {
    const void* X; int64_t M, K; int n1, n2, r;
    const float* R1; const float* R2; const __half* U;
    int8_t* q; float* scale; int32_t* qsum; float* T;
    int* counters; float* partials; int S;
    float* xs; float* pmax;  // split rotation: rotated values (M x K) and per-workgroup extremes (M x G x 2)
    float qmax;              // largest code: 2^(bits-1) - 1
    int tp;                  // row pitch of T (= r, or r + 1 for a layer with row shifts)
    float* tmode;            // T + (PSP rank): first of the entries the layer's mode adds to a row, or NULL
    int asym, shift;         // the layer's mode: asymmetric activation codes, row shift
    int64_t rot_blocks;      // workgroups below this index rotate token blockIdx.x, the rest project
    int JG;                  // projection workgroups per (token tile, slice): groups of rank tiles
    const uint16_t* R1p; const uint16_t* R2p;          // bf16 term planes of the factors
};

// projection workgroup pb of a launch: slice fastest, then the group of rank tiles, then the token tile
template <bool BF16>
__device__ __forceinline__ void psp_block_at(char* lds, const RqArgs& a, int pb, bool finish = true) {
    const int s = pb % a.S, rest = pb / a.S;
    psp_block<BF16>(lds, a.X, a.M, a.K, a.r, a.U, a.T, a.counters, a.partials, a.S, rest / a.JG, s, a.tp, finish,
                    rest % a.JG, a.JG);
}

template <bool BF16>
__global__ __launch_bounds__(RQ_THREADS) void rotate_quant_kernel(RqArgs a) {
    extern __shared__ __align__(16) float lds[];
    if ((int64_t)blockIdx.x < a.rot_blocks) {
        rotate_token<BF16>(lds, a.X, blockIdx.x, a.K, a.n1, a.n2, a.R1, a.R2, a.q, a.scale, a.qsum, a.tmode, a.tp, a.qmax,
                           a.asym != 0, a.shift != 0);
    } else {
        const int pb = (int)(blockIdx.x - a.rot_blocks);
        psp_block_at<BF16>(reinterpret_cast<char*>(lds), a, pb);
    }
}

// rotation on bf16 MFMA (bf16 activations): 64 threads per 16-column strip of n2
template <int ATM, int THREADS, bool LOOP, bool DUAL = false>
__global__ __launch_bounds__(THREADS) void rotate_quant3_kernel(RqArgs a) {
    extern __shared__ __align__(16) float lds[];
    if ((int64_t)blockIdx.x < a.rot_blocks) {
        rotate3_token<ATM, LOOP, DUAL>(reinterpret_cast<char*>(lds), reinterpret_cast<const uint16_t*>(a.X), blockIdx.x,
                           a.rot_blocks, a.M, a.K, a.n1, a.n2, a.R1p, a.R2p, a.q, a.scale, a.qsum, a.tmode,
                           a.tp, a.qmax, a.asym != 0, a.shift != 0);
    } else {
        const int pb = (int)(blockIdx.x - a.rot_blocks);
        psp_block_at<true>(reinterpret_cast<char*>(lds), a, pb);
    }
}

// split rotation: workgroup b < rot_blocks does slice b % G of token b / G
__global__ __launch_bounds__(640) void rotate_split_kernel(RqArgs a) {
    extern __shared__ __align__(16) float lds[];
    if ((int64_t)blockIdx.x < a.rot_blocks) {
        const int G = rs_shape(r3_shape(a.n1, a.n2)).G;
        const int64_t t = blockIdx.x / G;
        rotate_slice_block(reinterpret_cast<char*>(lds), reinterpret_cast<const uint16_t*>(a.X), t,
                           (int)(blockIdx.x - t * G), a.K, a.n1, a.n2, a.R1p, a.R2p, a.xs, a.pmax, a.qsum);
    } else {
        const int pb = (int)(blockIdx.x - a.rot_blocks);
        psp_block_at<true>(reinterpret_cast<char*>(lds), a, pb, false);
    }
}

template <int ATM, int THREADS, bool LOOP, bool DUAL = false>
hipError_t launch_rotate3_v(const RqArgs& a, int64_t blocks, int threads, size_t lds, hipStream_t st) {
    hipError_t e = bwla_ensure_lds((const void*)rotate_quant3_kernel<ATM, THREADS, LOOP, DUAL>, lds);
    if (e != hipSuccess) return e;
    rotate_quant3_kernel<ATM, THREADS, LOOP, DUAL><<<dim3((unsigned)blocks), dim3((unsigned)threads), lds, st>>>(a);
    return hipGetLastError();
}
// the looping variant only when a workgroup really has more than one token; `dual`: two tokens
// at a time (the launcher has then doubled the threads and added the second token area to lds)
template <int ATM, int THREADS>
hipError_t launch_rotate3(const RqArgs& a, int64_t blocks, int threads, size_t lds, hipStream_t st, bool dual) {
    if (dual) {
        if constexpr (ATM <= 8) return launch_rotate3_v<ATM, THREADS, true, true>(a, blocks, threads, lds, st);
        else return hipErrorInvalidValue;
    }
    if (a.rot_blocks < a.M) return launch_rotate3_v<ATM, THREADS, true>(a, blocks, threads, lds, st);
    return launch_rotate3_v<ATM, THREADS, false>(a, blocks, threads, lds, st);
}

__global__ __launch_bounds__(256) void code_sums_kernel(const int8_t* __restrict__ q, int64_t K,
                                                        int32_t* __restrict__ qsum) {
    __shared__ int red[4];
    const int64_t t = blockIdx.x;
    const int* row = reinterpret_cast<const int*>(q + t * K);
    int s = 0;
    for (int i = threadIdx.x; i < (int)(K >> 2); i += 256) {
        const int w = row[i];
        s += (int)(int8_t)(w & 0xff) + (int)(int8_t)((w >> 8) & 0xff) + (int)(int8_t)((w >> 16) & 0xff) + (w >> 24);
    }
    s = bwla_wave_sum_i32(s);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) qsum[t] = red[0] + red[1] + red[2] + red[3];
}

// Nibble packing of 4-bit codes: 32 codes (two 16-code pieces) become 16 bytes, byte b holding code b
// of the first piece in its low and code b of the second piece in its high nibble.  One thread per
// 16 output bytes.
__global__ __launch_bounds__(256) void pack_codes_a4_kernel(const int8_t* __restrict__ q, int64_t pieces,
                                                            uint8_t* __restrict__ q4) {
    const int64_t p = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (p >= pieces) return;
    const uint4 lo = *reinterpret_cast<const uint4*>(q + p * 32);
    const uint4 hi = *reinterpret_cast<const uint4*>(q + p * 32 + 16);
    uint4 o;
    o.x = (lo.x & 0x0f0f0f0fu) | ((hi.x << 4) & 0xf0f0f0f0u);
    o.y = (lo.y & 0x0f0f0f0fu) | ((hi.y << 4) & 0xf0f0f0f0u);
    o.z = (lo.z & 0x0f0f0f0fu) | ((hi.z << 4) & 0xf0f0f0f0u);
    o.w = (lo.w & 0x0f0f0f0fu) | ((hi.w << 4) & 0xf0f0f0f0u);
    *reinterpret_cast<uint4*>(q4 + p * 16) = o;
}

}  // namespace


size_t bwla_rotate_lds_bytes(int n1, int n2) { return rq_shape(n1, n2).lds_bytes; }
// factors that do not fit into LDS are streamed with 16-byte loads, which needs n % 4 == 0
bool bwla_rotate_supported(int n1, int n2) {
    const RqShape sh = rq_shape(n1, n2);
    return sh.lds_bytes <= RQ_LDS_LIMIT && (sh.resident || ((n1 & 3) == 0 && (n2 & 3) == 0));
}
int bwla_rotate_tiles(int n1, int n2) { return (rq_pad16(n1) / 16) * (rq_pad16(n2) / 16); }
int bwla_rotate_max_tiles() { return RQ_MAXT * RQ_WAVES; }

bwla_psp_plan bwla_make_psp_plan(int64_t M, int64_t K, int r) {
    bwla_psp_plan p;
    const int rp = (r + 15) & ~15;
    // The projection rides in the rotation launch while that launch stays within about three
    // workgroups per CU: its short workgroups then finish in the shadow of the rotation, and the
    // separate projection kernel costs about 8 us at these sizes (64 x 80, rank 64, 320 tokens:
    // 33.4 -> 25.6 us with 720 workgroups; 128 x 64, rank 64, 320 tokens: 960 workgroups lose, 36.7 -> 38.8).
    // (ranks of more than two 16-column tiles are dealt to several workgroups per slice)
    const int jg = rp > 16 * PP_GROUPJT ? (rp / 16 + PP_GROUPJT - 1) / PP_GROUPJT : 1;
    const int64_t ride = M + ((M + 15) / 16) * ((K + PP_SLICE - 1) / PP_SLICE) * jg;
    if (M <= 16 || r <= 0 || ride <= 768) {
        p.token_tiles = (int)((M + 15) / 16);
        p.k_per_split = PP_SLICE;
        p.splits = r > 0 ? (int)((K + PP_SLICE - 1) / PP_SLICE) : 1;
        p.tile_rows = 16; p.tile_cols = jg > 1 ? 16 * PP_GROUPJT : rp; p.col_groups = jg;
        return p;
    }
    // many tokens: slices of K in multiples of eight (XCD x works on the slices x, x + 8, ...: any other
    // count leaves some XCDs with one slice more than others), and the fewest that still give every CU
    // a workgroup -- the launch is then resident at once (two workgroups fit a CU) and a tile's partial
    // sums are handed over between as few workgroups as possible.  Measured, rotation + projection:
    // 2048 x 25600 with 8 / 16 / 24 slices 142 / 150 / 165 us; 4096 x 8192 with 8 / 12 / 16: 78 / 96 / 91.
    p.tile_rows = 64;
    p.tile_cols = bwla_psp_prefill_tile_cols(rp);
    p.col_groups = (rp + 63) / 64;
    p.token_tiles = (int)((M + 63) / 64);
    const int64_t units = (int64_t)p.token_tiles * p.col_groups;
    const int64_t cus = bwla_device_cus();
    int64_t S = 8 * ((cus + 8 * units - 1) / (8 * units));
    const int64_t smax = K / 512 > 1 ? K / 512 : 1;
    if (S > smax) S = smax;
    if (S < 1) S = 1;
    const int64_t per = (K + S - 1) / S;
    p.k_per_split = (int)(((per + 127) / 128) * 128);
    p.splits = (int)((K + p.k_per_split - 1) / p.k_per_split);
    return p;
}

hipError_t bwla_launch_rotate_quant(const bwla_layer_t* L, const void* dX, int xdtype, int64_t M, int8_t* dq,
                                    float* dscale, int32_t* dqsum, float* dT, void* dws, const bwla_psp_plan& plan,
                                    hipStream_t st, int act_bits) {
    const char* blob = (const char*)L->d_blob;
    const RqShape sh = rq_shape(L->n1, L->n2);
    RqArgs a;
    const int ru = bwla_rank_u(L);                     // the projection's rank; T has L->r columns
    a.X = dX; a.M = M; a.K = L->K; a.n1 = L->n1; a.n2 = L->n2; a.r = ru;
    a.tp = L->r; a.tmode = L->mode != 0 ? dT + ru : nullptr;
    a.asym = (L->mode & BWLA_MODE_ASYM_ACT) ? 1 : 0; a.shift = (L->mode & BWLA_MODE_ROW_SHIFT) ? 1 : 0;
    a.qmax = (float)((1 << (act_bits - 1)) - 1);
    a.R1 = (const float*)(blob + L->off_R1); a.R2 = (const float*)(blob + L->off_R2);
    a.U = (const __half*)(blob + L->off_U);
    a.R1p = (const uint16_t*)(blob + L->off_R1p); a.R2p = (const uint16_t*)(blob + L->off_R2p);
    a.q = dq; a.scale = dscale; a.qsum = dqsum; a.T = dT;
    a.counters = (int*)dws;
    a.partials = dws ? (float*)((char*)dws + bwla_psp_counter_bytes(M)) : nullptr;
    a.S = plan.splits;
    a.JG = plan.tile_rows == 16 ? plan.col_groups : 1;
    a.xs = nullptr; a.pmax = nullptr;
    // Few tokens: one launch holds rotation and projection workgroups (a second launch would
    // cost more than it saves).  Many tokens: the projection has a kernel of its own.
    const bool merged = ru > 0 && plan.tile_rows == 16;
    const int64_t pblocks = merged ? (int64_t)plan.token_tiles * plan.splits * plan.col_groups : 0;
    const size_t plds = merged ? pp_lds_bytes(ru) : 0;
    a.rot_blocks = M;
    hipError_t e;
    if (!merged) {
        // many bf16 tokens and factors whose operand-order planes fit LDS: the looping kernel with
        // resident factors
        bool done = false;
        e = bwla_launch_rotate_planes(L, dX, xdtype, M, dq, dscale, dqsum, dT, act_bits, st, &done);
        if (e != hipSuccess) return e;
        if (done) return ru > 0 ? bwla_launch_psp_prefill(L, dX, xdtype, M, dT, dws, plan, st) : hipSuccess;
    }
    const R3Shape s3 = r3_shape(L->n1, L->n2);
    const size_t split_bytes = xdtype == BWLA_X_BF16 ? bwla_split_rotation_bytes(L, plan, M) : 0;
    if (split_bytes > 0 && dws != nullptr) {
        // few tokens, R1 too large for LDS: several workgroups per token, then a launch that quantizes
        const RsShape rs = rs_shape(s3);
        a.xs = (float*)((char*)dws + bwla_align256(bwla_psp_ws_bytes(plan, M, ru)));
        a.pmax = a.xs + M * L->K;
        float* zcs = a.pmax + 2 * M * rs.E;            // per token: what the stored codes have to lose
        a.rot_blocks = M * rs.G;
        const int threads3 = s3.strips > 8 ? 64 * s3.strips : 512;     // the projection wants eight wavefronts
        const size_t pl3 = merged ? pp_lds_bytes(ru, threads3 / 64) : 0;
        const size_t lds3 = pl3 > rs.lds_bytes ? pl3 : rs.lds_bytes;
        e = bwla_ensure_lds((const void*)rotate_split_kernel, lds3);
        if (e != hipSuccess) return e;
        rotate_split_kernel<<<dim3((unsigned)(a.rot_blocks + pblocks)), dim3((unsigned)threads3), lds3, st>>>(a);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        // (the projection's workgroups in that launch leave partial tiles; the next one adds them up)
        const bool psum = merged && a.S > 1;
        const PspSum ps{a.partials, a.T, M, M * RS_QB, a.r, a.S};
        quantize_rows_kernel<<<dim3((unsigned)(M * RS_QB + (psum ? plan.token_tiles : 0))), dim3(512), 0, st>>>(
            a.xs, a.pmax, rs.E, L->K, dq, dscale, dqsum, a.qmax, a.asym, a.tmode, a.tp, zcs, ps);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        if (a.shift) {
            shift_column_kernel<<<dim3((unsigned)((M + 255) / 256)), dim3(256), 0, st>>>(
                dscale, dqsum, zcs, M, L->K, a.tmode + (a.asym ? 2 : 0), a.tp);
            e = hipGetLastError();
            if (e != hipSuccess) return e;
        }
        if (ru > 0 && !merged) return bwla_launch_psp_prefill(L, dX, xdtype, M, dT, dws, plan, st);
        return hipSuccess;
    }
    if (xdtype == BWLA_X_BF16 && s3.ok) {
        // projection workgroups in the same launch want all eight wavefronts; so does a rotation
        // workgroup with one token and resident factors (the extra wavefronts help to fetch them)
        int threads = (merged && s3.strips < 8) ? 512 : 64 * s3.strips;
        const size_t pl3 = merged ? pp_lds_bytes(ru, threads / 64) : 0;
        const size_t lds3 = pl3 > s3.lds_bytes ? pl3 : s3.lds_bytes;
        bool dual = false;
        size_t lds_dual = 0;
        // resident factors and many tokens: as many workgroups as fit the chip at once, each
        // walking over its share of the tokens with the factors loaded once
        if (s3.resident && !merged) {
            int64_t per_cu = (int64_t)(RQ_LDS_LIMIT / lds3);
            // the kernels use more than 170 registers: two wavefronts per SIMD, eight per CU (counting
            // what LDS alone allows put 64 x 64 at 1024 tokens on one workgroup per token, 37.8 us;
            // 512 looping workgroups take 28.5)
            const int64_t by_waves = 8 / (threads / 64);
            if (per_cu > by_waves) per_cu = by_waves;
            if (per_cu < 1) per_cu = 1;
            const int64_t cap = per_cu * bwla_device_cus();
            if (M > cap) a.rot_blocks = cap;
            // only one workgroup of at most four wavefronts per CU (large factors): two tokens at a
            // time per workgroup, if the second token's rows still fit (128 x 64: 28 us for 272 to
            // 448 tokens in two rounds of one token, 22 us for 512 tokens two at a time)
            if (per_cu == 1 && M > cap && s3.strips <= 4 && s3.at <= 8 &&
                s3.lds_bytes + (size_t)s3.r0bytes + 256 <= RQ_LDS_LIMIT) {
                dual = true;
                threads = 2 * 64 * s3.strips;
                lds_dual = s3.lds_bytes + (size_t)s3.r0bytes + 256;
                if ((M + 1) / 2 < cap) a.rot_blocks = (M + 1) / 2;
            }
        }
        if (s3.resident && a.rot_blocks == M && s3.strips < 8) threads = 512;
        // register budget: up to 8 wavefronts may use 256 VGPRs, 9 or 10 only 168
        const int64_t grid = a.rot_blocks + pblocks;
        const size_t ldsl = dual ? lds_dual : lds3;
        if (s3.strips <= 8 && s3.at <= 4) e = launch_rotate3<4, 512>(a, grid, threads, ldsl, st, dual);
        else if (s3.strips <= 8 && s3.at <= 8) e = launch_rotate3<8, 512>(a, grid, threads, ldsl, st, dual);
        else if (s3.at <= 12) e = launch_rotate3<12, 640>(a, grid, threads, ldsl, st, dual);
        else e = launch_rotate3<16, 512>(a, grid, threads, ldsl, st, dual);
        if (e != hipSuccess) return e;
        if (ru > 0 && !merged) return bwla_launch_psp_prefill(L, dX, xdtype, M, dT, dws, plan, st);
        return hipSuccess;
    }
    const size_t lds = plds > sh.lds_bytes ? plds : sh.lds_bytes;
    if (xdtype == BWLA_X_BF16) {
        e = bwla_ensure_lds((const void*)rotate_quant_kernel<true>, lds);
        if (e != hipSuccess) return e;
        rotate_quant_kernel<true><<<dim3((unsigned)(M + pblocks)), dim3(RQ_THREADS), lds, st>>>(a);
    } else {
        e = bwla_ensure_lds((const void*)rotate_quant_kernel<false>, lds);
        if (e != hipSuccess) return e;
        rotate_quant_kernel<false><<<dim3((unsigned)(M + pblocks)), dim3(RQ_THREADS), lds, st>>>(a);
    }
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (ru > 0 && !merged) return bwla_launch_psp_prefill(L, dX, xdtype, M, dT, dws, plan, st);
    return hipSuccess;
}

size_t bwla_split_rotation_bytes(const bwla_layer_t* L, const bwla_psp_plan& plan, int64_t M) {
    const R3Shape s3 = r3_shape(L->n1, L->n2);
    if (!s3.ok || L->K > (int64_t)RS_QB * 512 * RS_QI * 4) return 0;
    // Factors that fit LDS: the split still pays when the second product is long (six or more
    // tiles along n1) and either the strips do not spread evenly over the CU's four SIMDs (n2 = 86:
    // six wavefronts, two SIMDs carry two) or there are at most eight tokens, so that the extra
    // workgroups are free (measured, 128 x 64: 12.1 -> 11.1 us at four tokens, 12.2 -> 11.8 at
    // eight, 12.3 -> 12.9 at sixteen; 128 x 86: 16.7 -> 10.9 at one token, 17.1 -> 12.2 at sixteen).
    if (s3.resident && !(s3.at >= 6 && ((s3.strips & 3) != 0 || M <= 8))) return 0;
    const RsShape rs = rs_shape(s3);
    if (!rs.ok) return 0;
    const bool merged = bwla_rank_u(L) > 0 && plan.tile_rows == 16;
    const int64_t pblocks = merged ? (int64_t)plan.token_tiles * plan.splits * plan.col_groups : 0;
    // up to two workgroups per CU (one after the other where LDS lets only one be resident):
    // 224 x 128 at sixteen tokens 21.6 us against 31.2 in one workgroup per token, at thirty-two
    // 34.5 against 32.0; with more tokens the one-workgroup-per-token kernel keeps the chip busy
    if (M * rs.G + pblocks > 2 * bwla_device_cus()) return 0;
    return (size_t)(M * L->K + 2 * M * rs.E + M) * sizeof(float);     // values, extremes, per-token code offset
}

hipError_t bwla_launch_pack_codes_a4(const int8_t* dq, int64_t M, int64_t K, uint8_t* dq4, hipStream_t st) {
    const int64_t pieces = M * (K / 32);
    pack_codes_a4_kernel<<<dim3((unsigned)((pieces + 255) / 256)), dim3(256), 0, st>>>(dq, pieces, dq4);
    return hipGetLastError();
}

hipError_t bwla_launch_code_sums(const int8_t* dq, int64_t M, int64_t K, int32_t* dqsum, hipStream_t st) {
    code_sums_kernel<<<dim3((unsigned)M), dim3(256), 0, st>>>(dq, K, dqsum);
    return hipGetLastError();
}
