// Measurement aids, not steps of the method: what this GPU reaches on a pure streaming read of a
// given size and on a loop of nothing but INT8 MFMAs (the benchmark quotes the forward's kernels
// against these measured ceilings next to the published peaks, 8 TB/s and 5.0 POP/s), what a kernel
// launch costs when the kernel does nothing, and how long a dependent load takes.
#include "bwla_internal.h"

namespace {

typedef int v4i_p __attribute__((ext_vector_type(4)));

// Every lane reads 16 bytes per step, a workgroup one contiguous 4 KiB per step, the grid strides
// over the buffer; the xor of all words goes to one word per workgroup so that no load is dead.
__global__ __launch_bounds__(256) void probe_read_kernel(const v4i_p* __restrict__ src, uint64_t n16, uint32_t* __restrict__ sink) {
    uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    const uint64_t stride = (uint64_t)gridDim.x * 256;
    v4i_p a0 = {0, 0, 0, 0}, a1 = a0, a2 = a0, a3 = a0;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const v4i_p v0 = __builtin_nontemporal_load(src + i);
        const v4i_p v1 = __builtin_nontemporal_load(src + i + stride);
        const v4i_p v2 = __builtin_nontemporal_load(src + i + 2 * stride);
        const v4i_p v3 = __builtin_nontemporal_load(src + i + 3 * stride);
        a0 ^= v0; a1 ^= v1; a2 ^= v2; a3 ^= v3;
    }
    for (; i < n16; i += stride) {
        a0 ^= __builtin_nontemporal_load(src + i);
    }
    const v4i_p a = a0 ^ a1 ^ a2 ^ a3;
    uint32_t x = (uint32_t)(a.x ^ a.y ^ a.z ^ a.w);
    for (int o = 32; o > 0; o >>= 1) x ^= __shfl_xor(x, o);
    if ((threadIdx.x & 63) == 0) sink[blockIdx.x * 4 + (threadIdx.x >> 6)] = x;
}

// Four independent accumulator chains per wavefront, operands fixed in registers: the matrix
// cores see back-to-back 16x16x64 INT8 MFMAs and nothing else.
__global__ __launch_bounds__(256) void probe_mfma_i8_kernel(int iters, int32_t* __restrict__ sink) {
    const int lane = threadIdx.x & 63;
    v4i_p a = {lane * 0x01010101, 0x01020304, lane, 0x7f7f7f7f};
    v4i_p b = {0x01010101, lane ^ 0x55, 0x00010001, 0x01000100};
    v4i_p c0 = {0, 0, 0, 0}, c1 = c0, c2 = c0, c3 = c0;
    for (int i = 0; i < iters; ++i) {
        c0 = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_i32_16x16x64_i8(b, a, c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, a, c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_i32_16x16x64_i8(b, b, c3, 0, 0, 0);
    }
    const v4i_p s = c0 + c1 + c2 + c3;
    sink[(blockIdx.x * 256 + threadIdx.x) & 4095] = s.x ^ s.y ^ s.z ^ s.w;
}

// a launch of the decode kernels' shape (one workgroup of 512 threads per CU) that does nothing
__global__ __launch_bounds__(512) void probe_empty_kernel() {}

// One lane walks through the buffer: the index of every load depends on the value the load before it
// returned ((v & 1) is unknown to the compiler), so the loads cannot overlap.  Ticks of the constant
// 100 MHz counter around the walk go to out[0], the last index to out[1] (keeps the chain alive).
__global__ void probe_chase_kernel(const uint32_t* __restrict__ buf, uint64_t n, uint64_t stride, int iters,
                                   uint64_t* __restrict__ out) {
    if (threadIdx.x != 0) return;
    uint64_t idx = 0;
    const uint64_t t0 = wall_clock64();
    for (int i = 0; i < iters; ++i) {
        const uint32_t v = __builtin_nontemporal_load(buf + idx);
        idx += stride + (v & 1u);
        if (idx >= n) idx -= n;
    }
    const uint64_t t1 = wall_clock64();
    out[0] = t1 - t0;
    out[1] = idx;
}

// the constant 100 MHz counter at the moment the kernel runs
__global__ void probe_clock_kernel(uint64_t* __restrict__ out) {
    if (threadIdx.x == 0) out[0] = wall_clock64();
}

}  // namespace

extern "C" {

BWLA_API bwla_status_t bwla_probe_clock(void* d_out, void* stream) {
    if (!d_out) return BWLA_ERR_NULL;
    if ((uintptr_t)d_out & 7) return BWLA_ERR_ALIGN;
    hipLaunchKernelGGL(probe_clock_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream, (uint64_t*)d_out);
    return hipGetLastError() == hipSuccess ? BWLA_OK : BWLA_ERR_HIP;
}

BWLA_API bwla_status_t bwla_probe_empty_launch(void* stream) {
    hipLaunchKernelGGL(probe_empty_kernel, dim3(bwla_device_cus()), dim3(512), 0, (hipStream_t)stream);
    return hipGetLastError() == hipSuccess ? BWLA_OK : BWLA_ERR_HIP;
}

BWLA_API bwla_status_t bwla_probe_load_latency(const void* d_buf, size_t bytes, size_t stride_bytes, int iters,
                                               void* d_out, void* stream) {
    if (!d_buf || !d_out) return BWLA_ERR_NULL;
    if (bytes < 8 || (bytes & 3) || (stride_bytes & 3) || stride_bytes == 0 || stride_bytes + 4 > bytes ||
        iters < 1 || iters > (1 << 24))
        return BWLA_ERR_SHAPE;
    if (((uintptr_t)d_buf & 3) || ((uintptr_t)d_out & 7)) return BWLA_ERR_ALIGN;
    hipLaunchKernelGGL(probe_chase_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream, (const uint32_t*)d_buf,
                       (uint64_t)(bytes / 4), (uint64_t)(stride_bytes / 4), iters, (uint64_t*)d_out);
    return hipGetLastError() == hipSuccess ? BWLA_OK : BWLA_ERR_HIP;
}

BWLA_API bwla_status_t bwla_probe_hbm_read(const void* d_src, size_t bytes, void* d_sink, size_t sink_bytes, void* stream) {
    if (!d_src || !d_sink) return BWLA_ERR_NULL;
    if (bytes < 16 || (bytes & 15) || ((uintptr_t)d_src & 15)) return BWLA_ERR_SHAPE;
    const uint64_t n16 = bytes / 16;
    // enough workgroups to keep every CU's request queues full, never more than the buffer has 4 KiB pieces
    uint64_t grid = (uint64_t)bwla_device_cus() * 8;
    if (grid > (n16 + 255) / 256) grid = (n16 + 255) / 256;
    if (sink_bytes < grid * 16) return BWLA_ERR_BUFSIZE;
    hipLaunchKernelGGL(probe_read_kernel, dim3((unsigned)grid), dim3(256), 0, (hipStream_t)stream,
                       (const v4i_p*)d_src, n16, (uint32_t*)d_sink);
    return hipGetLastError() == hipSuccess ? BWLA_OK : BWLA_ERR_HIP;
}

BWLA_API bwla_status_t bwla_probe_mfma_int8(int iters, void* d_sink, size_t sink_bytes, int64_t* ops_out, void* stream) {
    if (!d_sink || !ops_out) return BWLA_ERR_NULL;
    if (iters < 1 || iters > (1 << 20)) return BWLA_ERR_SHAPE;
    if (sink_bytes < 4096 * 4) return BWLA_ERR_BUFSIZE;
    // eight wavefronts per CU (two per SIMD), four CUs' worth of workgroups per CU in flight
    const int grid = bwla_device_cus() * 4;
    *ops_out = (int64_t)grid * 4 * iters * 4 * (2LL * 16 * 16 * 64);
    hipLaunchKernelGGL(probe_mfma_i8_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream, iters, (int32_t*)d_sink);
    return hipGetLastError() == hipSuccess ? BWLA_OK : BWLA_ERR_HIP;
}

}  // extern "C"
