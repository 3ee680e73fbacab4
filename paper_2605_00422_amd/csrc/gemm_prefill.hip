// Binary-weight GEMM for token batches (M > 16): a dense int8 contraction on 32x32x32 INT8
// MFMA with exact int32 accumulation.
//
//   acc[t,n] = sum_k q[t,k] Sign(W[n,k]) = 2 * sum_k q[t,k] b[n,k] - qsum_t
//   Y[t,n]   = scale_t * alpha_n * acc[t,n] + sum_j T[t,j] V[n,j]       (paper Eq. 4; Sec. 3.2)
//
// In both kernels of this file the 1-bit weights never touch LDS: each lane keeps the
// 128-column bit slice of its own output channel in four registers and expands a 16-column run
// with (w >> j) & 0x01010101 right before the MFMA that consumes it.
//   gemm_prefill_direct_kernel  the main path (K % 128 == 0, N >= 32): every wavefront streams
//                               its own operands, no workgroup barriers (described further down)
//   gemm_prefill_kernel         the remaining shapes: code tiles shared through LDS, double
//                               buffered, one barrier per 128 columns
#include "bwla_internal.h"
#include <algorithm>

namespace {

constexpr int GP_BK = 128;           // columns per main-loop step = one 16-byte bit slice per row
constexpr int GP_LDA = GP_BK + 16;   // LDS row pitch of the code tile (bytes)

template <int MT, int NTL, int WM, int WN>
__global__ __launch_bounds__(64 * WM * WN) void gemm_prefill_kernel(
    const uint4* __restrict__ bits, int chunks, int row_tiles, const int8_t* __restrict__ q, int M, int K,
    const float* __restrict__ scale, const int32_t* __restrict__ qsum, const __half* __restrict__ alpha,
    const __half* __restrict__ V, const float* __restrict__ T, int r, float* __restrict__ Y, int N,
    int32_t* __restrict__ acc_out, int tiles_m, int tiles_n) {
    constexpr int THREADS = 64 * WM * WN;
    constexpr int BM = WM * MT * 32;
    constexpr int BN = WN * NTL * 32;
    constexpr int PIECES = BM * (GP_BK / 16) / THREADS;     // 16-byte granules of the A tile per thread
    static_assert(BM * (GP_BK / 16) % THREADS == 0, "tile fill must divide evenly");
    extern __shared__ __align__(16) char smem[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, lg = lane >> 5;
    const int wm = wave % WM, wn = wave / WM;

    // XCD-aware tile order: workgroups are dealt round-robin to the 8 XCDs, so give each XCD a
    // contiguous run of tiles (same token rows -> the code tile is shared in that XCD's L2)
    int pid = blockIdx.x;
    const int nblocks = gridDim.x;
    if ((nblocks & 7) == 0) pid = (pid & 7) * (nblocks >> 3) + (pid >> 3);
    const int tm = pid / tiles_n, tn = pid - tm * tiles_n;
    const int m_base = tm * BM, n_base = tn * BN;

    const int nslices = (K + GP_BK - 1) / GP_BK;

    // ---- A tile fill helpers
    uint4 areg[PIECES];
    auto a_fetch = [&](int ks) {
#pragma unroll
        for (int p = 0; p < PIECES; ++p) {
            const int idx = tid + p * THREADS;
            const int row = idx >> 3, gcol = idx & 7;
            const int m = m_base + row, k = ks * GP_BK + gcol * 16;
            areg[p] = make_uint4(0, 0, 0, 0);
            if (m < M && k < K) areg[p] = *reinterpret_cast<const uint4*>(q + (int64_t)m * K + k);
        }
    };
    auto a_store = [&](int buf) {
        char* dst = smem + buf * (BM * GP_LDA);
#pragma unroll
        for (int p = 0; p < PIECES; ++p) {
            const int idx = tid + p * THREADS;
            const int row = idx >> 3, gcol = idx & 7;
            *reinterpret_cast<uint4*>(dst + row * GP_LDA + gcol * 16) = areg[p];
        }
    };
    // ---- weight slice of this lane's output channels
    v4i wcur[NTL], wnext[NTL];
    auto w_fetch = [&](int ks, v4i (&w)[NTL]) {
#pragma unroll
        for (int nt = 0; nt < NTL; ++nt) {
            const int row = n_base + (wn * NTL + nt) * 32 + l32;
            const int rt = row >> 4;
            w[nt] = v4i{0, 0, 0, 0};
            if (rt < row_tiles) {
                const uint4 u = bits[((int64_t)rt * chunks + (ks >> 2)) * 64 + (ks & 3) * 16 + (row & 15)];
                w[nt] = v4i{(int)u.x, (int)u.y, (int)u.z, (int)u.w};
            }
        }
    };

    v16i acc[MT][NTL];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NTL; ++nt)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mt][nt][v] = 0;

    a_fetch(0);
    w_fetch(0, wcur);
    a_store(0);
    __syncthreads();

    for (int ks = 0; ks < nslices; ++ks) {
        const bool more = ks + 1 < nslices;
        if (more) {
            a_fetch(ks + 1);
            w_fetch(ks + 1, wnext);
        }
        const char* As = smem + (ks & 1) * (BM * GP_LDA) + (wm * MT * 32 + l32) * GP_LDA + lg * 16;
        // lane half lg consumes 16-column group 2*s + lg in step s (both operands use this order)
        v4i ws[NTL];
#pragma unroll
        for (int nt = 0; nt < NTL; ++nt) ws[nt] = wcur[nt] >> lg;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            v4i a[MT], b[NTL];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) a[mt] = *reinterpret_cast<const v4i*>(As + mt * 32 * GP_LDA + s * 32);
#pragma unroll
            for (int nt = 0; nt < NTL; ++nt) b[nt] = (ws[nt] >> (2 * s)) & 0x01010101;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int nt = 0; nt < NTL; ++nt)
                    acc[mt][nt] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[mt], b[nt], acc[mt][nt], 0, 0, 0);
        }
        if (more) a_store((ks + 1) & 1);
        __syncthreads();
#pragma unroll
        for (int nt = 0; nt < NTL; ++nt) wcur[nt] = wnext[nt];
    }

    // ---- epilogue.  Accumulator element v of lane (l32, lg): row 8*(v/4) + 4*lg + v%4, column l32.
    const int JT = (r + 15) >> 4;
    const int rp = JT * 16;
    const int half = rp >> 1;                          // lane half lg feeds j in [lg*half, lg*half + half)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int mrow0 = m_base + (wm * MT + mt) * 32;
        if (mrow0 >= M) continue;
#pragma unroll
        for (int nt = 0; nt < NTL; ++nt) {
            const int n = n_base + (wn * NTL + nt) * 32 + l32;
            if (n_base + (wn * NTL + nt) * 32 >= N) continue;
            v16f low;
#pragma unroll
            for (int v = 0; v < 16; ++v) low[v] = 0.0f;
            // low-rank term on fp32 MFMA: D[m][n] = sum_j T[m][j] V[n][j]
            {
                const int tm_row = mrow0 + l32;
                const float* trow = T + (int64_t)tm_row * r;
                const __half* vrow = V + (int64_t)n * rp;
                for (int p = 0; p < half; ++p) {
                    const int j = lg * half + p;
                    const float tv = (tm_row < M && j < r) ? trow[j] : 0.0f;
                    const float vv = (n < N) ? __half2float(vrow[j]) : 0.0f;
                    low = __builtin_amdgcn_mfma_f32_32x32x2f32(tv, vv, low, 0, 0, 0);
                }
            }
            const float al = (n < N) ? __half2float(alpha[n]) : 0.0f;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = mrow0 + 8 * (v >> 2) + 4 * lg + (v & 3);
                if (m < M && n < N) {
                    const int a = 2 * acc[mt][nt][v] - qsum[m];
                    Y[(int64_t)m * N + n] = scale[m] * al * (float)a + low[v];
                    if (acc_out) acc_out[(int64_t)m * N + n] = a;
                }
            }
        }
    }
}

template <int MT, int NTL, int WM, int WN>
hipError_t launch_cfg(const bwla_layer_t* L, const int8_t* dq, const float* dscale, const int32_t* dqsum,
                      const float* dT, int64_t M, float* dY, int32_t* dacc, hipStream_t st) {
    constexpr int BM = WM * MT * 32, BN = WN * NTL * 32;
    const char* blob = (const char*)L->d_blob;
    const int tiles_m = (int)((M + BM - 1) / BM), tiles_n = (int)((L->N + BN - 1) / BN);
    const size_t lds = 2 * (size_t)BM * GP_LDA;
    auto kern = gemm_prefill_kernel<MT, NTL, WM, WN>;
    hipError_t e = bwla_ensure_lds((const void*)kern, lds);
    if (e != hipSuccess) return e;
    kern<<<dim3((unsigned)(tiles_m * tiles_n)), dim3(64 * WM * WN), lds, st>>>(
        (const uint4*)(blob + L->off_bits), (int)bwla_chunks(L->K), (int)bwla_row_tiles(L->N), dq, (int)M,
        (int)L->K, dscale, dqsum, (const __half*)(blob + L->off_alpha), (const __half*)(blob + L->off_V), dT,
        L->r, dY, (int)L->N, dacc, tiles_m, tiles_n);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Large token batches: every wavefront streams its own operands and synchronizes with nobody --
// no workgroup barriers.  A wavefront owns 64 token rows x NTL*32 output channels.  Per
// 128-column slice of K
//   * its 64 code rows travel global -> LDS asynchronously (16 bytes per lane, 8 lanes per
//     128-byte row segment, no registers involved) into a private ring of four swizzled 8 KiB
//     tiles, four slices ahead of their use; the MFMA operand layout is read back from there:
//     lane (row l32, half lg) gets columns [64*lg, 64*lg + 64) of the slice, 16 per step;
//   * the 16-byte bit slice of each of its NTL weight rows goes straight into a ring of four
//     register slots, four slices ahead.
// Step s of a slice contracts the 16-column group 4*lg + s on both operands.  The four
// wavefronts of a workgroup share the weight rows (L1 hits) and take different token rows.
//
// The compiler cannot tell which ring tile an LDS read touches, and with an asynchronous copy
// in flight it turns every wait for a vector-memory result into a wait for all of them.  The
// loop therefore issues its operand reads (LDS) and its weight loads (global) as inline
// assembly and waits explicitly: `s_waitcnt vmcnt(GD_YOUNGER)` for the slice that must have
// landed (the count of younger vector-memory operations is fixed by the issue order documented
// at the loop) and `s_waitcnt lgkmcnt(0)` before an LDS read's registers are consumed.  A
// register written by such a load is not touched between the load and its wait.
constexpr int GD_MT = 2;
constexpr int GD_ROWS = GD_MT * 32;                 // token rows per wavefront
constexpr int GD_TILE = GD_ROWS * 128;              // bytes of one private code tile
constexpr int GD_BUFS = 4;                          // private code tiles per wavefront

typedef __attribute__((ext_vector_type(8))) __bf16 v8bf;

// x = h1 + h2 + h3 exactly, each a bf16
__device__ __forceinline__ void gd_split3(float x, __bf16& h1, __bf16& h2, __bf16& h3) {
    h1 = (__bf16)x;
    const float r1 = x - (float)h1;
    h2 = (__bf16)r1;
    h3 = (__bf16)(r1 - (float)h2);
}

// 16-byte position of piece `c16` of row `row` inside its 128-byte LDS row; the XOR key makes
// the column-wise operand reads conflict free
__device__ __forceinline__ int gd_key(int row) { return (row ^ (row >> 3)) & 7; }
// 64-byte rows (nibble-packed codes): rows r, r + 4, r + 8, r + 12 share a bank group, the key separates them
__device__ __forceinline__ int gd_key4(int row) { return (row >> 2) & 3; }

__device__ __forceinline__ v4i gd_lds_read(uint32_t addr) {
    v4i r;
    asm volatile("ds_read_b128 %0, %1" : "=v"(r) : "v"(addr));
    return r;
}
// s_waitcnt immediate for vmcnt(n) alone on gfx9 encodings: vmcnt = bits 3:0 and 15:14,
// expcnt (6:4) and lgkmcnt (11:8) left at "no wait"
constexpr int gd_vmcnt_imm(int n) { return (n & 15) | ((n >> 4) << 14) | (7 << 4) | (15 << 8); }

// GATED: the rows interleave a gate and an up projection, and instead of Y the kernel stores
// h[t, i] = silu(y[t, 2 i]) * y[t, 2 i + 1] as bf16 (a compile-time variant: the plain kernel's
// register allocation is not to change)
// A4: the codes arrive nibble-packed (two 4-bit codes per byte, 16-code pieces interleaved in pairs:
// byte b of packed piece P holds code b of piece 2P in its low and of piece 2P + 1 in its high nibble).
// A row of a slice is then 64 bytes; a lane reads one packed piece for two contraction steps and
// moves each nibble to the top of its byte, (x << 4) & 0xf0.. and x & 0xf0..: int8 operands worth 16
// times the code, so the accumulators are exact multiples of 16 and are shifted down once at the end.
template <int NTL, int WM, int WK, int NB, bool GATED = false, bool A4 = false, int WN = 1>
__global__ __launch_bounds__(64 * WM * WK * WN, NB == 2 ? 2 : 1) void gemm_prefill_direct_kernel(
    const uint4* __restrict__ bits, int chunks, int row_tiles, const int8_t* __restrict__ q, int M, int K,
    const float* __restrict__ scale, const int32_t* __restrict__ qsum, const __half* __restrict__ alpha,
    const __half* __restrict__ V, const float* __restrict__ T, int r, float* __restrict__ Y, int N,
    int32_t* __restrict__ acc_out, int tiles_m, int tiles_n, uint16_t* __restrict__ H) {
    constexpr int MT = GD_MT;
    // WM wavefronts stacked along the tokens; WK wavefronts share one tile and split its slices of K
    // (small batches: more wavefronts in flight), their accumulators are added through LDS
    // WN wavefronts side by side along the channels (wavefronts with the same token rows then ask for the
    // same code rows at about the same time: the second request is served by the CU's L1)
    static_assert(WN == 1 || WK == 1, "channel-wise stacking is for unsplit K");
    constexpr int BM = WM * GD_ROWS, BN = WN * NTL * 32;
    // vector-memory operations per slice and wavefront: NTL weight loads, then 8 code copies;
    // when slice j + 1 is needed, the operations of slices j + 2 and j + 3 may still be in flight
    // (NB = ring depth, 4 or 2: code tiles in LDS and weight slots in registers)
    static_assert(NB == 4 || NB == 2, "ring depth");
    constexpr int NCOPY = A4 ? 4 : 8;                            // code copies per slice
    constexpr int GD_PER_SLICE = NTL + NCOPY;
    constexpr int GD_YOUNGER = (NB - 2) * GD_PER_SLICE;
    extern __shared__ __align__(16) char smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave % WM, wk = WK == 1 ? 0 : wave / WM, wn = WK == 1 ? wave / WM : 0;
    const int l32 = lane & 31, lg = lane >> 5;
    char* mytile = smem + wave * (NB * GD_TILE);
    const uint32_t mytile_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)mytile;

    // XCD-aware tile order (workgroups are dealt round-robin to the 8 XCDs): one XCD works on
    // runs of tiles with the same token rows, so the codes are fetched once per XCD
    int pid = blockIdx.x;
    const int nblocks = gridDim.x;
    if ((nblocks & 7) == 0) pid = (pid & 7) * (nblocks >> 3) + (pid >> 3);
    const int tm = pid / tiles_n, tn = pid - tm * tiles_n;
    const int m_base = tm * BM + wm * GD_ROWS, n_base = tn * BN + wn * (NTL * 32);
    // my slices of K: [s_begin, s_begin + nslices) of K / 128 (K % 128 == 0, checked by the launcher)
    const int ns_all = K >> 7;
    const int ns_per = (ns_all + WK - 1) / WK;
    const int s_begin = wk * ns_per;
    const int nslices = ns_all - s_begin < ns_per ? (ns_all - s_begin > 0 ? ns_all - s_begin : 0) : ns_per;
    // local slice index -> a slice that exists (indices past my range re-read a valid slice)
    auto slice_of = [&](int ks) -> int {
        const int g = s_begin + (ks < nslices ? ks : nslices - 1);
        return g < 0 ? 0 : (g < ns_all ? g : ns_all - 1);
    };

    // asynchronous copies: instruction j moves rows 8j .. 8j+7; lane i lands at row i/8,
    // position i%8 and therefore fetches piece (i%8) ^ key(row).  Rows past the matrix re-read
    // its last row (their results are not stored).  Addresses are a wave-uniform base plus a
    // 32-bit lane offset (at most 64 rows apart).
    const int m_first = m_base < M ? m_base : M - 1;
    const int KB = A4 ? K >> 1 : K;                              // bytes of a code row
    const int8_t* abase = q + (int64_t)m_first * KB;
    int avofs[NCOPY];
#pragma unroll
    for (int j = 0; j < NCOPY; ++j) {
        // (nibbles: instruction j moves rows 16j .. 16j+15 of 64 bytes, lane i row i/4, position i%4)
        const int row = A4 ? 16 * j + (lane >> 2) : 8 * j + (lane >> 3);
        int m = m_base + row;
        if (m > M - 1) m = M - 1;
        avofs[j] = A4 ? (m - m_first) * KB + (((lane & 3) ^ gd_key4(row)) << 4)
                      : (m - m_first) * KB + (((lane & 7) ^ gd_key(row)) << 4);
    }
    // operand reads: row mt*32 + l32, piece 4*lg + s (nibbles: packed piece 2*lg + s, s < 2)
    uint32_t rofs[MT][4];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int row = mt * 32 + l32;
            rofs[mt][s] = A4 ? mytile_lds + row * 64 + ((((2 * lg + (s & 1)) ^ gd_key4(row)) & 3) << 4)
                             : mytile_lds + row * 128 + ((((4 * lg + s) ^ gd_key(row)) & 7) << 4);
        }
    // weight rows nt*32 + l32 of this workgroup's columns: 16-row tile, row inside it (tiles past
    // the matrix re-read its last tile); offsets in 16-byte units from a uniform base
    int rt_first = n_base >> 4;
    if (rt_first > row_tiles - 1) rt_first = row_tiles - 1;
    const uint4* wbase = bits + (int64_t)rt_first * chunks * 64;
    int wvofs[NTL];
#pragma unroll
    for (int nt = 0; nt < NTL; ++nt) {
        const int row = n_base + nt * 32 + l32;
        int rt = row >> 4;
        if (rt > row_tiles - 1) rt = row_tiles - 1;
        wvofs[nt] = (rt - rt_first) * chunks * 64 + (row & 15);
    }
    const int shamt = 4 * lg;

    auto copy_codes = [&](int ks) {                              // 8 vector-memory operations
        const int kc = slice_of(ks);
        char* dst = mytile + (ks & (NB - 1)) * GD_TILE;
#pragma unroll
        for (int j = 0; j < NCOPY; ++j)
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void*)(abase + (int64_t)kc * (A4 ? 64 : 128) + avofs[j]),
                (__attribute__((address_space(3))) void*)(dst + j * 1024), 16, 0, 0);
    };
    struct Wslot { v4i w[NTL]; };                                // vector values: they stay in registers
    auto fetch_w = [&](Wslot& sl, int ks) {                      // NTL vector-memory operations
        const int kc = slice_of(ks);
        const int so = (kc >> 2) * 64 + (kc & 3) * 16;
#pragma unroll
        for (int nt = 0; nt < NTL; ++nt) {
            const uint4* p = wbase + so + wvofs[nt];
            asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(sl.w[nt]) : "v"(p) : "memory");
        }
    };
    // marks the point after which a slot's registers hold their data (placed behind the wait)
    auto landed = [&](Wslot& sl) {
#pragma unroll
        for (int nt = 0; nt < NTL; ++nt) asm volatile("" : "+v"(sl.w[nt]));
    };

    v16i acc[MT][NTL];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NTL; ++nt)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mt][nt][v] = 0;

    // Operands of one contraction step: code rows from LDS (asynchronous read, to be followed
    // by settle()), expanded weight bits.
    struct Ops { v4i av[MT]; v4i b[NTL]; };
    v4i raw[MT];                                                 // nibbles: the packed piece of steps 2h, 2h + 1
    auto prepare = [&](Ops& o, const Wslot& sl, int ks, int s) {
        const uint32_t bo = (uint32_t)((ks & (NB - 1)) * GD_TILE);
        if constexpr (A4) {
            if ((s & 1) == 0) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) raw[mt] = gd_lds_read(rofs[mt][s >> 1] + bo);
            }
        } else {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) o.av[mt] = gd_lds_read(rofs[mt][s] + bo);
        }
        // slices past the end (the trip count is padded to a multiple of three) contract zeros
        const int mask = ks < nslices ? 0x01010101 : 0;
#pragma unroll
        for (int nt = 0; nt < NTL; ++nt) o.b[nt] = (sl.w[nt] >> (shamt + s)) & mask;
    };
    auto settle = [&](Ops& o, int s) {
        static_assert(MT == 2, "operand list of the wait below");
        if constexpr (A4) {
            if ((s & 1) == 0) {
                asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(raw[0]), "+v"(raw[1]));
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) o.av[mt] = (raw[mt] << 4) & 0xf0f0f0f0;
            } else {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) o.av[mt] = raw[mt] & 0xf0f0f0f0;
            }
        } else {
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(o.av[0]), "+v"(o.av[1]));
        }
    };
    auto contract = [&](const Ops& o) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < NTL; ++nt)
                acc[mt][nt] = __builtin_amdgcn_mfma_i32_32x32x32_i8(o.av[mt], o.b[nt], acc[mt][nt], 0, 0, 0);
    };

    // Issue order of the vector-memory operations (it fixes GD_YOUNGER):
    //   prologue  w(0) codes(0) w(1) codes(1) w(2) codes(2) w(3) codes(3)
    //   step ks   ... w(ks + 4) codes(ks + 4)
    // Step ks reads slice ks from tile ks % 4 and weight slot ks % 4 (its first step's operands
    // were prepared by step ks - 1).  Before its last contraction step it needs slice ks + 1 for
    // the first operands of the next slice: at that point the operations younger than
    // codes(ks + 1) are those of slices ks + 2 and ks + 3.  When step ks is done, its tile and
    // slot are free for slice ks + 4.  Slices past the end (the trip count is padded to a multiple
    // of four) re-read a valid slice and contract zeros.
    Wslot w0, w1, w2, w3;
    Ops ops;
    auto step = [&](Wslot& cur, Wslot& nxt, int ks) {
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            Ops following;
            if (s < 3) {
                prepare(following, cur, ks, s + 1);
            } else {
                __builtin_amdgcn_s_waitcnt(gd_vmcnt_imm(GD_YOUNGER));    // slice ks + 1 has landed
                landed(nxt);
                prepare(following, nxt, ks + 1, 0);
            }
            contract(ops);
            __builtin_amdgcn_sched_barrier(0);
            settle(following, s + 1);                            // (s + 1 = 4: step 0 of the next slice)
            ops = following;
        }
        fetch_w(cur, ks + NB);
        copy_codes(ks + NB);
        __builtin_amdgcn_sched_barrier(0);
    };
    fetch_w(w0, 0); copy_codes(0);
    fetch_w(w1, 1); copy_codes(1);
    if constexpr (NB == 4) {
        fetch_w(w2, 2); copy_codes(2);
        fetch_w(w3, 3); copy_codes(3);
    }
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_waitcnt(gd_vmcnt_imm((NB - 1) * GD_PER_SLICE));  // slice 0 has landed
    landed(w0);
    prepare(ops, w0, 0, 0);
    settle(ops, 0);
    if constexpr (NB == 4) {
        for (int ks0 = 0; ks0 < nslices; ks0 += 4) {
            step(w0, w1, ks0);
            step(w1, w2, ks0 + 1);
            step(w2, w3, ks0 + 2);
            step(w3, w0, ks0 + 3);
        }
    } else {
        for (int ks0 = 0; ks0 < nslices; ks0 += 2) {
            step(w0, w1, ks0);
            step(w1, w0, ks0 + 1);
        }
    }
    // Drain the loads nobody reads.  Their destination registers must stay reserved until they
    // have landed, so the wait names all four slots as operands: without that the code behind
    // the loop may reuse a register that a load still in flight is about to overwrite.
    asm volatile("s_waitcnt vmcnt(0)" : "+v"(w0.w[0]), "+v"(w1.w[0]));
    // the remaining slot registers are used after the wait, hence reserved across it
#pragma unroll
    for (int nt = 1; nt < NTL; ++nt) asm volatile("" : "+v"(w0.w[nt]), "+v"(w1.w[nt]));
    if constexpr (NB == 4) {
#pragma unroll
        for (int nt = 0; nt < NTL; ++nt) asm volatile("" : "+v"(w2.w[nt]), "+v"(w3.w[nt]));
    }

    if constexpr (WK > 1) {
        // every wavefront has drained its copies: the tiles are dead, LDS carries the partial sums
        __syncthreads();
        int* red = reinterpret_cast<int*>(smem);
        constexpr int PER_WAVE = MT * NTL * 16 * 64;
        if (wk > 0) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int nt = 0; nt < NTL; ++nt)
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        red[((wk - 1) * WM + wm) * PER_WAVE + ((mt * NTL + nt) * 16 + v) * 64 + lane] = acc[mt][nt][v];
        }
        __syncthreads();
        if (wk > 0) return;
#pragma unroll
        for (int w = 1; w < WK; ++w)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int nt = 0; nt < NTL; ++nt)
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        acc[mt][nt][v] += red[((w - 1) * WM + wm) * PER_WAVE + ((mt * NTL + nt) * 16 + v) * 64 + lane];
    }

    if constexpr (A4) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < NTL; ++nt) acc[mt][nt] = acc[mt][nt] >> 4;    // exact: every operand was 16 x code
    }
    // ---- epilogue.  Accumulator element v of lane (l32, lg): row 8*(v/4) + 4*lg + v%4, column l32.
    // Low-rank term on fp16 MFMA 32x32x16: V is stored in fp16 and is an operand as it stands; a token's
    // row of T is scaled by a power of two 2^k (largest entry near 2^13) and split into two fp16 terms,
    // T 2^k = hi + lo to 2^-22: two products per 16 ranks and channel tile.  The main term
    // scale_t alpha_n (2 acc - qsum_t) is formed first, times 2^k of its row, in the accumulator's
    // registers, the MFMAs add the low-rank products onto it, and 2^-k is applied at the store (powers of
    // two: exact).  What the epilogue waits for is memory, not arithmetic: all its loads -- scales and code
    // sums of the rows, the tokens' rows of T, the channels' rows of V, up to 64 ranks at a time -- are
    // requested in one go before the first use (they were ten dependent round trips per tile when T and V
    // were fetched step by step: 12 % of the launch at 8192 x 8192 and 4096 tokens).
    typedef _Float16 v8h __attribute__((ext_vector_type(8)));
    constexpr int JC = (NB == 2 || NTL == 5) ? 2 : 4;                          // 16-rank steps per chunk (fewer where registers are short)
    const int JT = (r + 15) >> 4, rp = JT * 16;
    int ncol[NTL];
    float al[NTL];
#pragma unroll
    for (int nt = 0; nt < NTL; ++nt) {
        const int n = n_base + nt * 32 + l32;
        ncol[nt] = n < N ? n : N - 1;
        al[nt] = __half2float(alpha[ncol[nt]]);
    }
    // my token's entries 16 kk + 8 lg .. + 7 of T (zero past the rank)
    auto load_t = [&](float (&tv)[8], int tmr, int kk) {
        const int j0 = kk * 16 + 8 * lg;
        const float* tp = T + (int64_t)tmr * r + j0;
        if ((r & 3) == 0) {
            // whole groups of four are inside or outside the row; clamp the address, zero the value
            const float4 z = make_float4(0.f, 0.f, 0.f, 0.f);
            const float4 t0 = *reinterpret_cast<const float4*>(j0 < r ? tp : T);
            const float4 t1 = *reinterpret_cast<const float4*>(j0 + 4 < r ? tp + 4 : T);
            const float4 u0 = j0 < r ? t0 : z, u1 = j0 + 4 < r ? t1 : z;
            tv[0] = u0.x; tv[1] = u0.y; tv[2] = u0.z; tv[3] = u0.w;
            tv[4] = u1.x; tv[5] = u1.y; tv[6] = u1.z; tv[7] = u1.w;
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) tv[i] = j0 + i < r ? tp[i] : 0.0f;
        }
    };
    uint4 vfr[JC][NTL];                                          // V fragments of the current chunk of ranks
    auto load_v = [&](int c0) {
#pragma unroll
        for (int j = 0; j < JC; ++j) {
            const int kk = c0 + j < JT ? c0 + j : (JT > 0 ? JT - 1 : 0);
#pragma unroll
            for (int nt = 0; nt < NTL; ++nt)
                vfr[j][nt] = JT > 0 ? *reinterpret_cast<const uint4*>(V + (int64_t)ncol[nt] * rp + kk * 16 + 8 * lg)
                                    : make_uint4(0, 0, 0, 0);
        }
    };
    load_v(0);
    const bool one_chunk = JT <= JC;                             // then V stays in registers for both row tiles
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int mrow0 = m_base + mt * 32;
        if (mrow0 >= M) continue;
        int tmr = mrow0 + l32;
        if (tmr > M - 1) tmr = M - 1;
        // the row's largest magnitude, over all of its ranks
        float tmax = 0.0f;
        for (int c0 = 0; c0 < JT; c0 += JC) {
            float tv[JC][8];
#pragma unroll
            for (int j = 0; j < JC; ++j) load_t(tv[j], tmr, c0 + j < JT ? c0 + j : JT - 1);
#pragma unroll
            for (int j = 0; j < JC; ++j)
#pragma unroll
                for (int i = 0; i < 8; ++i) tmax = fmaxf(tmax, fabsf(tv[j][i]));
        }
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));            // the other half of my token's row
        int kexp = 0;
        if (tmax > 0.0f && tmax < 3.0e38f) kexp = 13 - ilogbf(tmax);
        kexp = kexp > 60 ? 60 : (kexp < -60 ? -60 : kexp);
        float sc[16];
        int qs[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            int m = mrow0 + 8 * (v >> 2) + 4 * lg + (v & 3);
            if (m > M - 1) m = M - 1;
            sc[v] = scale[m];
            qs[v] = qsum[m];
        }
        // the main term replaces acc in place (as float bits), times 2^k of its row:
        // result row 8 (v / 4) + 4 lg + v % 4 belongs to the token of lane (that row, any lg)
        int krow[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            krow[v] = __shfl(kexp, 8 * (v >> 2) + 4 * lg + (v & 3), 64);
            const float up = __int_as_float((127 + krow[v]) << 23);
            const int m = mrow0 + 8 * (v >> 2) + 4 * lg + (v & 3);
#pragma unroll
            for (int nt = 0; nt < NTL; ++nt) {
                const int a = 2 * acc[mt][nt][v] - qs[v];
                if constexpr (!GATED) {
                    const int n = n_base + nt * 32 + l32;
                    if (acc_out && m < M && n < N) acc_out[(int64_t)m * N + n] = a;
                }
                acc[mt][nt][v] = __float_as_int(sc[v] * al[nt] * (float)a * up);
            }
        }
        for (int c0 = 0; c0 < JT; c0 += JC) {
            if (c0 > 0 || (mt > 0 && !one_chunk)) load_v(c0);
            float tv[JC][8];
#pragma unroll
            for (int j = 0; j < JC; ++j) load_t(tv[j], tmr, c0 + j < JT ? c0 + j : JT - 1);   // (from the caches)
#pragma unroll
            for (int j = 0; j < JC; ++j) {
                if (c0 + j < JT) {
                    v8h thi, tlo;
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        const float x = ldexpf(tv[j][i], kexp);
                        const _Float16 h = (_Float16)x;
                        thi[i] = h;
                        tlo[i] = (_Float16)(x - (float)h);
                    }
#pragma unroll
                    for (int nt = 0; nt < NTL; ++nt) {
                        const v8h vb = __builtin_bit_cast(v8h, vfr[j][nt]);
                        v16f y = __builtin_bit_cast(v16f, acc[mt][nt]);
                        y = __builtin_amdgcn_mfma_f32_32x32x16_f16(tlo, vb, y, 0, 0, 0);
                        y = __builtin_amdgcn_mfma_f32_32x32x16_f16(thi, vb, y, 0, 0, 0);
                        acc[mt][nt] = __builtin_bit_cast(v16i, y);
                    }
                }
            }
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const float down = __int_as_float((127 - krow[v]) << 23);
            const int m = mrow0 + 8 * (v >> 2) + 4 * lg + (v & 3);
#pragma unroll
            for (int nt = 0; nt < NTL; ++nt) {
                const int n = n_base + nt * 32 + l32;
                const float yv = __int_as_float(acc[mt][nt][v]) * down;
                if constexpr (GATED) {
                    // lane pairs (n even, n + 1) hold (gate, up) of one token; the even lane stores
                    const float up = __shfl_xor(yv, 1, 64);
                    if (m < M && (l32 & 1) == 0 && n + 1 < N) {
                        const float h = yv / (1.0f + __expf(-yv)) * up;
                        H[(int64_t)m * (N >> 1) + (n >> 1)] = __builtin_bit_cast(uint16_t, (__bf16)h);
                    }
                } else if (m < M && n < N) {
                    Y[(int64_t)m * N + n] = yv;
                }
            }
        }
    }
}

template <int NTL, int WM, int WK, int NB, int WN = 1>
hipError_t launch_direct(const bwla_layer_t* L, const int8_t* dq, const float* dscale, const int32_t* dqsum,
                         const float* dT, int64_t M, float* dY, int32_t* dacc, hipStream_t st, uint16_t* dH,
                         bool a4 = false) {
    constexpr int BM = WM * GD_ROWS, BN = WN * NTL * 32;
    const char* blob = (const char*)L->d_blob;
    const int tiles_m = (int)((M + BM - 1) / BM), tiles_n = (int)((L->N + BN - 1) / BN);
    const size_t lds = (size_t)WM * WK * WN * NB * GD_TILE;
    static_assert((size_t)(WK - 1) * WM * GD_MT * NTL * 16 * 64 * 4 <= (size_t)WM * WK * NB * GD_TILE,
                  "the partial sums must fit into the tile rings");
    auto launch = [&](auto kern) -> hipError_t {
        hipError_t e = bwla_ensure_lds((const void*)kern, lds);
        if (e != hipSuccess) return e;
        kern<<<dim3((unsigned)(tiles_m * tiles_n)), dim3(64 * WM * WK * WN), lds, st>>>(
            (const uint4*)(blob + L->off_bits), (int)bwla_chunks(L->K), (int)bwla_row_tiles(L->N), dq, (int)M,
            (int)L->K, dscale, dqsum, (const __half*)(blob + L->off_alpha), (const __half*)(blob + L->off_V), dT,
            L->r, dY, (int)L->N, dacc, tiles_m, tiles_n, dH);
        return hipGetLastError();
    };
    if (a4) return dH != nullptr ? hipErrorInvalidValue : launch(gemm_prefill_direct_kernel<NTL, WM, WK, NB, false, true, WN>);
    if (dH != nullptr) return launch(gemm_prefill_direct_kernel<NTL, WM, WK, NB, true, false, WN>);
    return launch(gemm_prefill_direct_kernel<NTL, WM, WK, NB, false, false, WN>);
}

inline int64_t tiles_for(int64_t M, int64_t N, int BM, int BN) { return ((M + BM - 1) / BM) * ((N + BN - 1) / BN); }

// fraction of the chip kept busy by `tiles` equal workgroups on 256 CUs (last round may be ragged)
inline double wave_eff(int64_t tiles) {
    const int64_t rounds = (tiles + 255) / 256;
    return (double)tiles / (double)(rounds * 256);
}

}  // namespace

// the register-streaming kernel takes the layer (else the LDS-tiled one does)
bool bwla_gemm_prefill_streams(const bwla_layer_t* L) { return L->N >= 32 && (L->K & 127) == 0; }

hipError_t bwla_launch_gemm_prefill(const bwla_layer_t* L, const int8_t* dq, const float* dscale,
                                    const int32_t* dqsum, const float* dT, int64_t M, float* dY,
                                    int32_t* dacc, hipStream_t st, uint16_t* dH, bool a4) {
    const int64_t N = L->N;
    if (bwla_gemm_prefill_streams(L)) {
        // register-streaming kernel.  Large batches: four wavefronts stacked along the tokens,
        // 256 x 160 or 256 x 128 tiles, whichever fills the chip better.  Up to 128 tokens: one or
        // two wavefronts per workgroup and narrow channel tiles, so that enough workgroups exist.
        // (the large tiles need enough workgroups: 4096 x 4096 at 512 tokens has 52 of them and takes
        // 36.9 us against 21.0 with one wavefront per 64 x 32 tile; 8192 x 8192 at 256 tokens 63.0
        // against 35.8; at 104 workgroups the large tiles win, 38.6 against 44.0 and 64.0 against 77.8)
        const int64_t big = std::min(tiles_for(M, N, 256, 160), tiles_for(M, N, 256, 128));
        if (M > 128 && big > 72) {
            const int64_t cus_big = bwla_device_cus();
            // Four wavefronts side by side on the same 64 token rows (64 x 640 tiles) where such tiles come to
            // whole rounds over the CUs: the code rows are then fetched once per CU and slice instead of four
            // times (2048 x 25600 -> 5120: 217 -> 209 us against the 256 x 160 tiles).
            const int64_t t640 = tiles_for(M, N, 64, 640);
            if (N % 640 == 0 && t640 % cus_big == 0)
                return launch_direct<5, 1, 1, 4, 4>(L, dq, dscale, dqsum, dT, M, dY, dacc, st, dH, a4);
            // Output-heavy shapes (short rows of K, many channels: every round of tiles ends in a burst of
            // stores) with an even number of 256 x 128 tiles per CU: two workgroups per CU, each with a
            // ring of two slices (64 KiB of LDS, at most 256 registers), so that one workgroup's epilogue
            // and first loads run under the other's contraction.  Measured against the one-workgroup
            // variants at 4096 tokens: 8192 -> 8192 -3 .. -8 %, 8192 -> 28672 -5 .. -8 %, 28672 -> 8192 -1.5 %.
            const int64_t t128 = tiles_for(M, N, 256, 128);
            if (t128 >= 4 * cus_big && t128 % (2 * cus_big) == 0)
                return launch_direct<4, 4, 1, 2>(L, dq, dscale, dqsum, dT, M, dY, dacc, st, dH, a4);
            const double d160 = wave_eff(tiles_for(M, N, 256, 160)), d128 = wave_eff(tiles_for(M, N, 256, 128));
            if (d160 >= d128) return launch_direct<5, 4, 1, 4>(L, dq, dscale, dqsum, dT, M, dY, dacc, st, dH, a4);
            return launch_direct<4, 4, 1, 4>(L, dq, dscale, dqsum, dT, M, dY, dacc, st, dH, a4);
        }
        // Few tokens (or few large tiles): the kernel is bound by how often the code rows are re-read (every workgroup
        // reads all K of its tokens) and by how many wavefronts are in flight.  With t tiles of
        // 64 x 32: up to one per CU, four wavefronts share a tile and split K; up to two per CU,
        // 64 x 64 tiles shared by four wavefronts (half the code traffic, one workgroup per CU);
        // more, one wavefront per 64 x 32 tile.  Measured (us), in that order of variants:
        // 8192 x 8192 at 64 tokens (256 tiles) 17.1 / 21.6 / 27.8, at 128 (512) 33.3 / 23.1 / 29.1;
        // 4096 -> 11008 at 64 (344) 21.8 / 15.8 / 17.3, at 128 (688) 33.5 / 30.7 / 19.1;
        // 8192 -> 28672 at 64 (896) 62.0 / 42.2 / 31.2.
        const int64_t tiles = ((M + 63) / 64) * ((N + 31) / 32);
        const int64_t cus = bwla_device_cus();
        if (tiles <= cus) return launch_direct<1, 1, 4, 4>(L, dq, dscale, dqsum, dT, M, dY, dacc, st, dH, a4);
        if (tiles <= 2 * cus) return launch_direct<2, 1, 4, 4>(L, dq, dscale, dqsum, dT, M, dY, dacc, st, dH, a4);
        // beyond three per CU the wavefronts' re-reads of the code rows load the L2 -> CU paths: 64 x 64
        // tiles shared by two wavefronts halve them (8192 -> 28672 at 64 tokens, 896 tiles: 37.2 -> 32.2 us)
        if (tiles > 3 * cus) return launch_direct<2, 1, 2, 4>(L, dq, dscale, dqsum, dT, M, dY, dacc, st, dH, a4);
        return launch_direct<1, 1, 1, 4>(L, dq, dscale, dqsum, dT, M, dY, dacc, st, dH, a4);
    }
    // shapes the streaming kernel does not take (K not a multiple of 128, fewer than 32 channels):
    // LDS-tiled kernel, 64 x 128 or 128 x 128 tiles (it does not gate: the caller goes through Y)
    if (dH != nullptr || a4) return hipErrorInvalidValue;
    if (M <= 64) return launch_cfg<1, 2, 2, 2>(L, dq, dscale, dqsum, dT, M, dY, dacc, st);
    return launch_cfg<2, 2, 2, 2>(L, dq, dscale, dqsum, dT, M, dY, dacc, st);
}
