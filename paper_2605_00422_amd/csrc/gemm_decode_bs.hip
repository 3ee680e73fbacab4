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
#include "gemm_decode_bs_device.h"

namespace {

// NT: 16-row tiles per step.  JTT: compile-time number of 16-wide rank groups (>= ceil(r/16)).
// FAST: N % 4 == 0 and no accumulator dump, which allows float4 stores.
// MULTI: rows of more than one pass (long-row variant only).
template <int CPW, int DEPTH, int NT, int JTT, bool FAST, bool MULTI = false>
__global__ __launch_bounds__(CPW == BS_CPW ? BS_MAX_THREADS : 64 * (BS_MAXKS_LONG + 1)) void gemm_decode_bs_kernel(
    BsArgs a) {
    extern __shared__ __align__(16) char smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int stride = gridDim.x, first = blockIdx.x;
    const int units = (a.row_tiles + NT - 1) / NT;
    const int n_iter = (units - first + stride - 1) / stride;            // >= 1: grid <= units
    const int PV = (NT * (((a.r + 15) >> 4) * 16) + 31) >> 5;
    if (wave == a.KS) epilogue_wave<DEPTH, NT, JTT, FAST, MULTI>(a, smem, first, stride, n_iter, wave, lane);
    else if (wave <= PV) compute_wave<CPW, DEPTH, NT, true, MULTI>(a, smem, first, stride, n_iter, wave, lane);
    else compute_wave<CPW, DEPTH, NT, false, MULTI>(a, smem, first, stride, n_iter, wave, lane);
}


}  // namespace


bool bwla_gemm_decode_bs_supported(int64_t M, int64_t K, int r) {
    const int chunks = (int)bwla_chunks(K);
    // (rows of more than one pass keep 1 KiB of sums per unit of a workgroup in LDS: at most 64 units)
    return M <= 16 && chunks >= 2 && bs_fits(0, chunks, r, 1, bs_cpw_for(chunks), bs_passes_for(chunks) > 1 ? 64 : 0);
}

// Measured on MI355X: one 16-row tile per step, a prefetch ring of two steps and one workgroup per
// CU is the best launch shape for all decode layers tried (two tiles per step run the steady state
// ~30% faster but pay more at start-up, which dominates at these sizes).
hipError_t bwla_launch_gemm_decode_bs(const bwla_layer_t* L, const int8_t* dq, const float* dscale,
                                      const int32_t* dqsum, const float* dT, int64_t M, float* dY,
                                      int32_t* dacc, hipStream_t st, uint16_t* dH) {
    constexpr int nt = 1;
    int grid = bwla_device_cus();
    const char* blob = (const char*)L->d_blob;
    const int chunks = (int)bwla_chunks(L->K), row_tiles = (int)bwla_row_tiles(L->N);
    const int cpw = bs_cpw_for(chunks), passes = bs_passes_for(chunks);
    const int units0 = (row_tiles + nt - 1) / nt;
    if (grid > units0) grid = units0;
    // with several passes the sums of earlier passes wait in LDS, 1 KiB per tile of the workgroup's units
    const int pass_units = passes > 1 ? (units0 + grid - 1) / grid : 0;
    if (grid < 1 || chunks < 2 || M > 16 || pass_units > 64 ||
        !bs_fits(0, chunks, L->r, nt, cpw, pass_units))
        return hipErrorInvalidValue;
    // up to four tokens: code rows staged in LDS when they fit; else every wave loads its own
    const int direct = (M > 4 || !bs_fits(M, chunks, L->r, nt, cpw, pass_units)) ? 1 : 0;
    const int KS = bs_ks_for(chunks);
    const int JT = (L->r + 15) >> 4, rp = JT * 16;
    const int units = (row_tiles + nt - 1) / nt;
    if (grid > units) grid = units;
    const int jtt = JT <= 3 ? JT : JT <= 4 ? 4 : 8;    // (3: ranks 33..48, e.g. rank 32 plus the columns a layer mode adds)
    const size_t lds = bs_lds_bytes(direct ? 0 : M, chunks, rp, nt, pass_units);
    BsArgs a{(const uint4*)(blob + L->off_bits), chunks, row_tiles, dq, (int)M, (int)L->K, dscale, dqsum,
             (const __half*)(blob + L->off_alpha), (const __half*)(blob + L->off_V), dT, L->r, dY, (int)L->N,
             dacc, KS, direct, passes, dH};
    auto launch = [&](auto kern) -> hipError_t {
        hipError_t e = bwla_ensure_lds((const void*)kern, lds);
        if (e != hipSuccess) return e;
        kern<<<dim3((unsigned)grid), dim3(64 * (KS + 1)), lds, st>>>(a);
        return hipGetLastError();
    };
    const bool fast = (L->N % 4 == 0) && dacc == nullptr;
    // long rows: one launch shape (depth 2, one tile per step)
#define BS_LONG(J)                                                                                         \
    if (cpw == BS_CPW_LONG && jtt == J && passes == 1)                                                     \
        return fast ? launch(gemm_decode_bs_kernel<BS_CPW_LONG, 2, 1, J, true>)                            \
                    : launch(gemm_decode_bs_kernel<BS_CPW_LONG, 2, 1, J, false>);                          \
    if (cpw == BS_CPW_LONG && jtt == J)                                                                    \
        return fast ? launch(gemm_decode_bs_kernel<BS_CPW_LONG, 2, 1, J, true, true>)                      \
                    : launch(gemm_decode_bs_kernel<BS_CPW_LONG, 2, 1, J, false, true>);
    BS_LONG(0) BS_LONG(1) BS_LONG(2) BS_LONG(3) BS_LONG(4) BS_LONG(8)
#undef BS_LONG
#define BS_CASE(J)                                                                                         \
    if (jtt == J)                                                                                          \
        return fast ? launch(gemm_decode_bs_kernel<BS_CPW, 2, 1, J, true>)                                 \
                    : launch(gemm_decode_bs_kernel<BS_CPW, 2, 1, J, false>);
    BS_CASE(0) BS_CASE(1) BS_CASE(2) BS_CASE(3) BS_CASE(4) BS_CASE(8)
#undef BS_CASE
    return hipErrorInvalidValue;
}

namespace {
// h[t, i] = silu(Y[t, 2 i]) * Y[t, 2 i + 1] as bf16, for the GEMM kernels that do not gate in their epilogue
__global__ void swiglu_rows_kernel(const float* __restrict__ Y, int64_t pairs, uint16_t* __restrict__ H) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= pairs) return;
    const float2 gu = reinterpret_cast<const float2*>(Y)[i];
    H[i] = (uint16_t)bs_swiglu_bf16(gu.x, gu.y);
}
}  // namespace

hipError_t bwla_launch_swiglu_rows(const float* dY, int64_t M, int64_t N, uint16_t* dH, hipStream_t st) {
    const int64_t pairs = M * (N / 2);
    swiglu_rows_kernel<<<dim3((unsigned)((pairs + 255) / 256)), dim3(256), 0, st>>>(dY, pairs, dH);
    return hipGetLastError();
}
