// Internal declarations shared by the translation units of libbwla (not installed).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "bwla.h"

// ---------------------------------------------------------------- packed sign-bit tiling
// A "unit" is 16 output rows x 512 input columns = 1 KiB = 64 lanes x 16 bytes, exactly one
// wavefront-wide 128-bit load.  Lane l of a unit holds row (l & 15), column group g = l >> 4
// (128 columns).  Its four 32-bit words w[0..3] hold
//     bit (8*b + j) of w[d]  <->  column 512*chunk + 128*g + 16*j + 4*d + b
// so that, for a fixed j, (w[d] >> j) & 0x01010101 (d = 0..3) is a 16-byte run of 0/1 bytes for
// 16 consecutive columns: one INT8 MFMA operand, with no cross-lane traffic.
// Units are stored [row tile][chunk], i.e. a row tile's chunks are contiguous.
#define BWLA_TILE_ROWS 16
#define BWLA_CHUNK_COLS 512
#define BWLA_UNIT_BYTES 1024

static inline int64_t bwla_row_tiles(int64_t N) { return (N + BWLA_TILE_ROWS - 1) / BWLA_TILE_ROWS; }
static inline int64_t bwla_chunks(int64_t K) { return (K + BWLA_CHUNK_COLS - 1) / BWLA_CHUNK_COLS; }
static inline uint64_t bwla_align256(uint64_t x) { return (x + 255u) & ~uint64_t(255); }

// compute units of the current device (cached per device; 256 if the query fails)
int bwla_device_cus();

// three bf16 term planes of an n x n factor, rows padded to 16 and columns to 32
inline uint64_t bwla_factor_planes_bytes(int n) {
    return (uint64_t)3 * ((n + 15) & ~15) * ((n + 31) & ~31) * 2;
}

// Factor planes in MFMA operand order (one contiguous KiB per operand), stored for factor pairs
// that are multiples of 32, n1 up to 256 and n2 up to 160 (0 bytes otherwise), three parts:
//   R2d  three bf16 terms of R2, (n2 / 16) strips x (n2 / 32) steps x 3 KiB: only for the pairs the
//        single-launch decode kernel takes (n1 of 32, 64 or 128, n2 of 32 or 64)
//   R1h  two fp16 terms of 256 R1, (n1 / 32) steps x 2 x (n1 / 16) KiB
//   R2h  two fp16 terms of 256 R2, (n2 / 16) strips x (n2 / 32) steps x 2 KiB
inline bool bwla_planes_shape_ok(int n1, int n2) {
    return n1 >= 32 && n2 >= 32 && n1 <= 256 && n2 <= 160 && (n1 & 31) == 0 && (n2 & 31) == 0;
}
inline uint64_t bwla_decode_planes_r2_bytes(int n1, int n2) {
    const bool ok = (n1 == 32 || n1 == 64 || n1 == 128) && (n2 == 32 || n2 == 64);
    return ok ? (uint64_t)(n2 / 16) * (n2 / 32) * 3 * 1024 : 0;
}
inline uint64_t bwla_planes_r1h_bytes(int n1) { return (uint64_t)(n1 / 32) * 2 * (n1 / 16) * 1024; }
inline uint64_t bwla_planes_r2h_bytes(int n2) { return (uint64_t)(n2 / 16) * (n2 / 32) * 2 * 1024; }
inline uint64_t bwla_decode_planes_bytes(int n1, int n2) {
    if (!bwla_planes_shape_ok(n1, n2)) return 0;
    return bwla_decode_planes_r2_bytes(n1, n2) + bwla_planes_r1h_bytes(n1) + bwla_planes_r2h_bytes(n2);
}

// PSP projection (T = X U) launch plan: token tiles x column groups x S slices of K.  Up to 16
// tokens the projection rides in the rotation launch (tiles of 16 tokens x rp columns); above,
// a kernel of its own takes tiles of 64 tokens x up to 64 columns.
struct bwla_psp_plan {
    int token_tiles;
    int splits;        // S
    int k_per_split;   // columns of K per slice
    int tile_rows;     // tokens per tile (16 or 64)
    int tile_cols;     // columns per tile
    int col_groups;    // tiles across the rank
};
bwla_psp_plan bwla_make_psp_plan(int64_t M, int64_t K, int r);
// Every scratch of bwla_rotate_quant starts with the exchange area of the single-launch decode
// kernel -- an epoch word, eight arrival counts (64 bytes apart, from byte 64 on), and from byte
// 1024 on 8 x 96 tagged partial sums of T = x U, 8 bytes each -- at the same place whatever the
// layer and the token count, so that every
// call on a scratch agrees on it and no other kernel writes there.  The counters and partial sums
// of the other kernels follow behind it.
constexpr uint64_t BWLA_WS_HEAD = 1024 + 8 * 96 * 8;
// behind the head: one arrival counter per 16 tokens (whatever the plan), padded to 256 bytes
inline uint64_t bwla_psp_counter_bytes(int64_t M) { return bwla_align256((uint64_t)((M + 15) / 16) * sizeof(int)); }
// columns that a layer's mode adds to V and T behind the PSP columns
inline int bwla_extra_cols(int mode) { return ((mode & BWLA_MODE_ASYM_ACT) ? 2 : 0) + ((mode & BWLA_MODE_ROW_SHIFT) ? 1 : 0); }
// columns of U = rank of the projection T = X U
inline int bwla_rank_u(const bwla_layer_t* L) { return L->r - bwla_extra_cols(L->mode); }
inline size_t bwla_psp_ws_bytes(const bwla_psp_plan& p, int64_t M, int r) {
    if (r <= 0 || p.splits <= 1) return 0;
    return (size_t)(bwla_psp_counter_bytes(M) + (uint64_t)p.token_tiles * p.col_groups * p.splits *
                                                    p.tile_rows * p.tile_cols * sizeof(float));
}
// Bytes the rotation wants behind the projection's scratch when it is split over several
// workgroups per token and a second launch (few bf16 tokens, R1 too large for LDS); else 0.
size_t bwla_split_rotation_bytes(const bwla_layer_t* L, const bwla_psp_plan& plan, int64_t M);
int bwla_psp_prefill_tile_cols(int rp);
hipError_t bwla_launch_psp_prefill(const bwla_layer_t* L, const void* dX, int xdtype, int64_t M, float* dT,
                                   void* dws, const bwla_psp_plan& plan, hipStream_t st);

// Raises a kernel's dynamic-LDS limit, once per kernel, device and size class, so that steady-state
// launches, also under stream capture, issue no attribute calls.  Safe to call from several host
// threads.  (What the library remembers between calls is this table and the CU count per device:
// facts about the process, never about a caller's data.)
hipError_t bwla_ensure_lds(const void* fn, size_t bytes);

// ---------------------------------------------------------------- launchers (one per .hip file)
hipError_t bwla_launch_pack(const float* dW, const float* dR1, const float* dR2, const float* dU,
                            const float* dV, int64_t N, int64_t K, int n1, int n2, int r,
                            const bwla_layer_t* L, hipStream_t st);
hipError_t bwla_launch_unpack(const bwla_layer_t* L, int8_t* d_sgn, float* d_alpha, hipStream_t st);

// one launch: rotation + quantization workgroups, then the PSP projection workgroups
hipError_t bwla_launch_rotate_quant(const bwla_layer_t* L, const void* dX, int xdtype, int64_t M, int8_t* dq,
                                    float* dscale, int32_t* dqsum, float* dT, void* dws, const bwla_psp_plan& plan,
                                    hipStream_t st, int act_bits);
#if defined(__HIPCC__)
// Split-K hand-over between workgroups of one launch.  The GPU has one L2 per XCD, and a
// device-scope fence is paid with a write-back / invalidate of that whole cache.  Instead the
// partial sums themselves are moved with device-scope accesses (they bypass the non-coherent
// levels), and ordering comes from waiting for those stores before the arrival counter is
// bumped: publish = stores + bwla_partials_arrive(), consume = loads after it returned true.
__device__ __forceinline__ void bwla_store_agent(float* p, float v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float bwla_load_agent(const float* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Called by every thread of the workgroup after its partial stores; true in the workgroup that
// arrives last of `expected`.  `flag` is one int of LDS.
// Ordering relied on: the partial stores are device-scope write-through stores; every thread waits
// until the memory system has acknowledged its own (the explicit vmcnt(0) wait below -- a fence of
// workgroup scope does not emit one), the barrier then collects all threads, and only after it does
// one thread bump the device-scope counter.  A workgroup that reads the full count therefore finds
// every partial tile at the device-coherent level, which its device-scope loads read.
__device__ __forceinline__ bool bwla_partials_arrive(int* counter, int expected, int* flag) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0);                             // my stores have been acknowledged
    __syncthreads();
    if (threadIdx.x == 0)
        *flag = __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == expected - 1;
    __syncthreads();
    return *flag != 0;
}
#endif

hipError_t bwla_launch_code_sums(const int8_t* dq, int64_t M, int64_t K, int32_t* dqsum, hipStream_t st);
// the whole layer in one launch for one bf16 token where the shape allows it (*done says whether)
hipError_t bwla_launch_rotate_planes(const bwla_layer_t* L, const void* dX, int xdtype, int64_t M, int8_t* dq,
                                     float* dscale, int32_t* dqsum, float* dT, int act_bits, hipStream_t st,
                                     bool* done);
hipError_t bwla_launch_decode_layer(const bwla_layer_t* L, const void* dX, int xdtype, int64_t M, int8_t* dq,
                                    float* dscale, int32_t* dqsum, float* dT, void* dws_head, float* dY,
                                    int32_t* dacc, hipStream_t st, bool* done, bool dry_run = false, int act_bits = 6);

hipError_t bwla_launch_gemm_decode(const bwla_layer_t* L, const int8_t* dq, const float* dscale,
                                   const int32_t* dqsum, const float* dT, int64_t M, float* dY,
                                   int32_t* dacc, hipStream_t st);
bool bwla_gemm_decode_bs_supported(int64_t M, int64_t K, int r);
// (dH not NULL: gated output h as bf16, M x N / 2, instead of Y -- see bwla_linear_forward_swiglu)
hipError_t bwla_launch_gemm_decode_bs(const bwla_layer_t* L, const int8_t* dq, const float* dscale,
                                      const int32_t* dqsum, const float* dT, int64_t M, float* dY,
                                      int32_t* dacc, hipStream_t st, uint16_t* dH = nullptr);
hipError_t bwla_launch_swiglu_rows(const float* dY, int64_t M, int64_t N, uint16_t* dH, hipStream_t st);
bool bwla_gemm_prefill_streams(const bwla_layer_t* L);
// (dH not NULL: gated bf16 output instead of Y; only when bwla_gemm_prefill_streams(L))
hipError_t bwla_launch_gemm_prefill(const bwla_layer_t* L, const int8_t* dq, const float* dscale,
                                    const int32_t* dqsum, const float* dT, int64_t M, float* dY,
                                    int32_t* dacc, hipStream_t st, uint16_t* dH = nullptr, bool a4 = false);
// (a4: dq holds nibble-packed codes, K / 2 bytes per token; only when bwla_gemm_prefill_streams(L), no gating)
hipError_t bwla_launch_pack_codes_a4(const int8_t* dq, int64_t M, int64_t K, uint8_t* dq4, hipStream_t st);

// ---------------------------------------------------------------- device helpers
#ifdef __HIPCC__
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every
// outstanding global load and store (vmcnt(0)), which would drain the HBM prefetch queue of a
// software-pipelined loop at each barrier.
__device__ __forceinline__ void bwla_lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

__device__ __forceinline__ float bwla_bf16_to_f32(uint16_t h) {
    return __uint_as_float(((uint32_t)h) << 16);
}

__device__ __forceinline__ float bwla_wave_max(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}
__device__ __forceinline__ int bwla_wave_sum_i32(int v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}
#endif
