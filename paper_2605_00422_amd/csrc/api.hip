// C ABI of libbwla: argument validation on the host, then kernel launches on the caller's
// stream.  Nothing here allocates device memory or synchronizes.
#include <math.h>

#include <atomic>
#include <map>
#include <mutex>
#include <utility>

#include "bwla_internal.h"

size_t bwla_rotate_lds_bytes(int n1, int n2);
bool bwla_rotate_supported(int n1, int n2);
int bwla_rotate_tiles(int n1, int n2);
int bwla_rotate_max_tiles();
size_t bwla_gemm_decode_lds(int64_t M, int64_t K);

namespace {

constexpr size_t LDS_LIMIT = 160 * 1024;          // per-workgroup LDS on gfx950
constexpr size_t DECODE_LDS_LIMIT = 128 * 1024;   // code tile of the decode kernel

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

bwla_status_t check_shape(int64_t N, int64_t K, int32_t n1, int32_t n2, int32_t r) {
    if (N <= 0 || K <= 0 || n1 <= 0 || n2 <= 0 || r < 0) return BWLA_ERR_SHAPE;
    if ((int64_t)n1 * (int64_t)n2 != K) return BWLA_ERR_SHAPE;
    if (K % 32 != 0 || K > BWLA_MAX_K || r > BWLA_MAX_RANK) return BWLA_ERR_UNSUPPORTED;
    if (n1 > BWLA_MAX_FACTOR || n2 > BWLA_MAX_FACTOR) return BWLA_ERR_UNSUPPORTED;
    if (N > (int64_t)1 << 24) return BWLA_ERR_UNSUPPORTED;
    if (bwla_rotate_tiles(n1, n2) > bwla_rotate_max_tiles()) return BWLA_ERR_UNSUPPORTED;
    if (!bwla_rotate_supported(n1, n2)) return BWLA_ERR_UNSUPPORTED;
    return BWLA_OK;
}

// r counts the columns of V and T; U keeps the PSP columns only
void fill_layout(bwla_layer_t* L, int64_t N, int64_t K, int32_t n1, int32_t n2, int32_t r, int32_t mode) {
    const uint64_t rp = (uint64_t)((r + 15) & ~15);
    const uint64_t rpu = (uint64_t)((r - bwla_extra_cols(mode) + 15) & ~15);
    uint64_t off = 0;
    L->N = N; L->K = K; L->n1 = n1; L->n2 = n2; L->r = r; L->mode = mode;
    L->off_bits = off;  off = bwla_align256(off + (uint64_t)bwla_row_tiles(N) * bwla_chunks(K) * BWLA_UNIT_BYTES);
    L->off_alpha = off; off = bwla_align256(off + (uint64_t)N * 2);
    L->off_V = off;     off = bwla_align256(off + (uint64_t)N * rp * 2);
    L->off_U = off;     off = bwla_align256(off + (uint64_t)K * rpu * 2);
    L->off_R1 = off;    off = bwla_align256(off + (uint64_t)n1 * n1 * 4);
    L->off_R2 = off;    off = bwla_align256(off + (uint64_t)n2 * n2 * 4);
    L->off_R1p = off;   off = bwla_align256(off + bwla_factor_planes_bytes(n1));
    L->off_R2p = off;   off = bwla_align256(off + bwla_factor_planes_bytes(n2));
    L->off_Rd = 0;
    if (bwla_decode_planes_bytes(n1, n2) > 0) { L->off_Rd = off; off = bwla_align256(off + bwla_decode_planes_bytes(n1, n2)); }
    L->blob_bytes = off;
}

bwla_status_t check_layer(const bwla_layer_t* L) {
    if (!L) return BWLA_ERR_NULL;
    if (!L->d_blob) return BWLA_ERR_NULL;
    bwla_status_t s = check_shape(L->N, L->K, L->n1, L->n2, L->r);
    if (s != BWLA_OK) return s;
    if ((L->mode & ~(BWLA_MODE_ROW_SHIFT | BWLA_MODE_ASYM_ACT)) != 0 || L->r < bwla_extra_cols(L->mode))
        return BWLA_ERR_SHAPE;
    bwla_layer_t ref;
    fill_layout(&ref, L->N, L->K, L->n1, L->n2, L->r, L->mode);
    if (ref.off_bits != L->off_bits || ref.off_alpha != L->off_alpha || ref.off_V != L->off_V ||
        ref.off_U != L->off_U || ref.off_R1 != L->off_R1 || ref.off_R2 != L->off_R2 ||
        ref.off_R1p != L->off_R1p || ref.off_R2p != L->off_R2p || ref.off_Rd != L->off_Rd ||
        ref.blob_bytes != L->blob_bytes)
        return BWLA_ERR_SHAPE;
    if (!aligned16(L->d_blob)) return BWLA_ERR_ALIGN;
    return BWLA_OK;
}

// scratch of bwla_rotate_quant: the head every scratch has, the projection's part, then (256-byte
// aligned) the split rotation's; nothing at all when neither part is needed
size_t rq_ws_bytes(const bwla_layer_t* L, const bwla_psp_plan& p, int64_t M) {
    const size_t split = bwla_split_rotation_bytes(L, p, M);
    const size_t psp = bwla_psp_ws_bytes(p, M, bwla_rank_u(L));
    const size_t body = split ? (size_t)bwla_align256(psp) + split : psp;
    return body ? (size_t)BWLA_WS_HEAD + body : 0;
}
inline void* ws_body(void* d_ws) { return d_ws ? (char*)d_ws + BWLA_WS_HEAD : nullptr; }

}  // namespace

int bwla_device_cus() {
    static std::atomic<int> cached[64];                // 0 = not asked yet
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    n = cached[dev].load(std::memory_order_relaxed);
    if (n > 0) return n;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
    cached[dev].store(n, std::memory_order_relaxed);
    return n;
}

hipError_t bwla_ensure_lds(const void* fn, size_t bytes) {
    if (bytes <= 64 * 1024) return hipSuccess;          // default limit, nothing to raise
    static std::mutex mu;
    static std::map<std::pair<const void*, int>, size_t> granted;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> lock(mu);
    size_t& g = granted[std::make_pair(fn, dev)];
    if (bytes <= g) return hipSuccess;
    e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e == hipSuccess) g = bytes;
    return e;
}

// ---------------------------------------------------------------- scratch of the allocation-free call
// One array per GPU the library runs on, held until the process ends.  `scratch` itself is only the
// host-side name of the symbol: the device address is asked for once per device (with that device
// current) and that pointer is what kernels and fills get.
static __device__ __align__(256) unsigned char scratch[BWLA_STATIC_SCRATCH_BYTES];

namespace {

// what must read zero when a call starts: the eight arrival counts in the scratch's head (words
// 16, 32, .. 128; the epoch and the tagged words beside them must stay as they are) and the
// counters behind the head
__global__ void clear_counts_kernel(uint32_t* ws, int head_words, int n) {
    const int i = (int)(blockIdx.x * blockDim.x + threadIdx.x);
    if (i < n) ws[head_words + i] = 0u;
    if (i < 8) ws[16 * (1 + i)] = 0u;
}

hipError_t static_scratch_ptr(void** out) {
    static std::mutex mu;
    static void* ptrs[64] = {nullptr};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (ptrs[dev] == nullptr) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (p == nullptr) return hipErrorInvalidSymbol;
        ptrs[dev] = p;
    }
    *out = ptrs[dev];
    return hipSuccess;
}

}  // namespace

extern "C" {

const char* bwla_status_string(int status) {
    switch (status) {
        case BWLA_OK: return "ok";
        case BWLA_ERR_NULL: return "null pointer";
        case BWLA_ERR_SHAPE: return "inconsistent shape";
        case BWLA_ERR_ALIGN: return "pointer not 16-byte aligned";
        case BWLA_ERR_BUFSIZE: return "buffer too small";
        case BWLA_ERR_UNSUPPORTED: return "shape outside the supported range";
        case BWLA_ERR_HIP: return "HIP runtime error";
        default: return "unknown status";
    }
}

int bwla_version(void) { return 2; }

bwla_status_t bwla_kron_factor(int64_t K, int32_t* n1, int32_t* n2) {
    if (!n1 || !n2) return BWLA_ERR_NULL;
    if (K < 1) return BWLA_ERR_SHAPE;
    int64_t a = (int64_t)floor(sqrt((double)K));
    while (a * a > K) --a;                 // guard the floating-point square root
    while ((a + 1) * (a + 1) <= K) ++a;
    while (a > 1 && K % a != 0) --a;
    if (K / a > INT32_MAX) return BWLA_ERR_UNSUPPORTED;
    *n2 = (int32_t)a;
    *n1 = (int32_t)(K / a);
    return BWLA_OK;
}

bwla_status_t bwla_packed_size_mode(int64_t N, int64_t K, int32_t n1, int32_t n2, int32_t r, int32_t mode,
                                    size_t* bytes) {
    if (!bytes) return BWLA_ERR_NULL;
    if (r < 0) return BWLA_ERR_SHAPE;
    if ((mode & ~(BWLA_MODE_ROW_SHIFT | BWLA_MODE_ASYM_ACT)) != 0) return BWLA_ERR_UNSUPPORTED;
    bwla_status_t s = check_shape(N, K, n1, n2, r + bwla_extra_cols(mode));
    if (s != BWLA_OK) return s;
    bwla_layer_t L;
    fill_layout(&L, N, K, n1, n2, r + bwla_extra_cols(mode), mode);
    *bytes = (size_t)L.blob_bytes;
    return BWLA_OK;
}

bwla_status_t bwla_packed_size(int64_t N, int64_t K, int32_t n1, int32_t n2, int32_t r, size_t* bytes) {
    return bwla_packed_size_mode(N, K, n1, n2, r, 0, bytes);
}

bwla_status_t bwla_packed_size_centered(int64_t N, int64_t K, int32_t n1, int32_t n2, int32_t r, size_t* bytes) {
    return bwla_packed_size_mode(N, K, n1, n2, r, BWLA_MODE_ROW_SHIFT, bytes);
}

// r is the PSP rank (columns of d_U and d_V); the layer's r also counts the columns of its mode
bwla_status_t bwla_pack_weights_mode(const float* d_W_rot, const float* d_R1, const float* d_R2, const float* d_U,
                                     const float* d_V, int64_t N, int64_t K, int32_t n1, int32_t n2, int32_t r,
                                     int32_t mode, void* d_blob, size_t blob_bytes, void* stream,
                                     bwla_layer_t* out) {
    if (!d_W_rot || !d_R1 || !d_R2 || !d_blob || !out) return BWLA_ERR_NULL;
    if (r < 0) return BWLA_ERR_SHAPE;
    if ((mode & ~(BWLA_MODE_ROW_SHIFT | BWLA_MODE_ASYM_ACT)) != 0) return BWLA_ERR_UNSUPPORTED;
    const int32_t rt = r + bwla_extra_cols(mode);
    bwla_status_t s = check_shape(N, K, n1, n2, rt);
    if (s != BWLA_OK) return s;
    if (r > 0 && (!d_U || !d_V)) return BWLA_ERR_NULL;
    if (!aligned16(d_W_rot) || !aligned16(d_blob) || !aligned16(d_R1) || !aligned16(d_R2)) return BWLA_ERR_ALIGN;
    bwla_layer_t L;
    fill_layout(&L, N, K, n1, n2, rt, mode);
    if (blob_bytes < L.blob_bytes) return BWLA_ERR_BUFSIZE;
    L.d_blob = d_blob;
    hipError_t e = bwla_launch_pack(d_W_rot, d_R1, d_R2, d_U, d_V, N, K, n1, n2, r, &L, (hipStream_t)stream);
    if (e != hipSuccess) return BWLA_ERR_HIP;
    *out = L;
    return BWLA_OK;
}

bwla_status_t bwla_pack_weights(const float* d_W_rot, const float* d_R1, const float* d_R2,
                                const float* d_U, const float* d_V, int64_t N, int64_t K, int32_t n1,
                                int32_t n2, int32_t r, void* d_blob, size_t blob_bytes, void* stream,
                                bwla_layer_t* out) {
    return bwla_pack_weights_mode(d_W_rot, d_R1, d_R2, d_U, d_V, N, K, n1, n2, r, 0, d_blob, blob_bytes, stream, out);
}

bwla_status_t bwla_pack_weights_centered(const float* d_W_rot, const float* d_R1, const float* d_R2,
                                         const float* d_U, const float* d_V, int64_t N, int64_t K, int32_t n1,
                                         int32_t n2, int32_t r, void* d_blob, size_t blob_bytes, void* stream,
                                         bwla_layer_t* out) {
    return bwla_pack_weights_mode(d_W_rot, d_R1, d_R2, d_U, d_V, N, K, n1, n2, r, BWLA_MODE_ROW_SHIFT, d_blob,
                                  blob_bytes, stream, out);
}

bwla_status_t bwla_unpack_signs(const bwla_layer_t* layer, int8_t* d_sgn, float* d_alpha, void* stream) {
    bwla_status_t s = check_layer(layer);
    if (s != BWLA_OK) return s;
    if (!d_sgn) return BWLA_ERR_NULL;
    return bwla_launch_unpack(layer, d_sgn, d_alpha, (hipStream_t)stream) == hipSuccess ? BWLA_OK : BWLA_ERR_HIP;
}

bwla_status_t bwla_psp_workspace_size(const bwla_layer_t* layer, int64_t M, size_t* bytes) {
    if (!bytes) return BWLA_ERR_NULL;
    bwla_status_t s = check_layer(layer);
    if (s != BWLA_OK) return s;
    if (M <= 0) return BWLA_ERR_SHAPE;
    *bytes = rq_ws_bytes(layer, bwla_make_psp_plan(M, layer->K, bwla_rank_u(layer)), M);
    return BWLA_OK;
}

bwla_status_t bwla_rotate_quant(const bwla_layer_t* layer, const void* d_X, int xdtype, int64_t M,
                                int8_t* d_q, float* d_scale, int32_t* d_qsum, float* d_T, void* d_ws,
                                size_t ws_bytes, void* stream) {
    return bwla_rotate_quant_bits(layer, d_X, xdtype, 6, M, d_q, d_scale, d_qsum, d_T, d_ws, ws_bytes, stream);
}

bwla_status_t bwla_rotate_quant_bits(const bwla_layer_t* layer, const void* d_X, int xdtype, int act_bits,
                                     int64_t M, int8_t* d_q, float* d_scale, int32_t* d_qsum, float* d_T,
                                     void* d_ws, size_t ws_bytes, void* stream) {
    if (act_bits < 2 || act_bits > 8) return BWLA_ERR_UNSUPPORTED;
    bwla_status_t s = check_layer(layer);
    if (s != BWLA_OK) return s;
    // asymmetric codes are stored as q - 2^(b-1): with b = 8 that would use -128, which the GEMMs exclude
    if ((layer->mode & BWLA_MODE_ASYM_ACT) && act_bits > 7) return BWLA_ERR_UNSUPPORTED;
    if (!d_X || !d_q || !d_scale || !d_qsum) return BWLA_ERR_NULL;
    if (layer->r > 0 && !d_T) return BWLA_ERR_NULL;
    if (M <= 0 || M > (int64_t)1 << 24) return BWLA_ERR_SHAPE;
    if (xdtype != BWLA_X_F32 && xdtype != BWLA_X_BF16) return BWLA_ERR_UNSUPPORTED;
    if (!aligned16(d_X) || !aligned16(d_q) || (d_T && !aligned16(d_T)) || (d_ws && !aligned16(d_ws)))
        return BWLA_ERR_ALIGN;
    const bwla_psp_plan plan = bwla_make_psp_plan(M, layer->K, bwla_rank_u(layer));
    const size_t need = rq_ws_bytes(layer, plan, M);
    if (need > 0 && (!d_ws || ws_bytes < need)) return d_ws ? BWLA_ERR_BUFSIZE : BWLA_ERR_NULL;
    hipStream_t st = (hipStream_t)stream;
    if (bwla_launch_rotate_quant(layer, d_X, xdtype, M, d_q, d_scale, d_qsum, d_T, ws_body(d_ws), plan, st, act_bits) !=
        hipSuccess)
        return BWLA_ERR_HIP;
    return BWLA_OK;
}

bwla_status_t bwla_decode_forward_bits(const bwla_layer_t* layer, const void* d_X, int xdtype, int act_bits, int64_t M,
                                  int8_t* d_q, float* d_scale, int32_t* d_qsum, float* d_T, void* d_ws,
                                  size_t ws_bytes, float* d_Y, int32_t* d_acc, void* stream) {
    if (act_bits < 2 || act_bits > 8) return BWLA_ERR_UNSUPPORTED;
    bwla_status_t s = check_layer(layer);
    if (s != BWLA_OK) return s;
    if ((layer->mode & BWLA_MODE_ASYM_ACT) && act_bits > 7) return BWLA_ERR_UNSUPPORTED;
    if (!d_X || !d_q || !d_scale || !d_qsum || !d_Y) return BWLA_ERR_NULL;
    if (layer->r > 0 && !d_T) return BWLA_ERR_NULL;
    if (M <= 0 || M > (int64_t)1 << 24) return BWLA_ERR_SHAPE;
    if (xdtype != BWLA_X_F32 && xdtype != BWLA_X_BF16) return BWLA_ERR_UNSUPPORTED;
    if (!aligned16(d_X) || !aligned16(d_q) || !aligned16(d_Y) || (d_T && !aligned16(d_T)) ||
        (d_ws && !aligned16(d_ws)) || (d_acc && !aligned16(d_acc)))
        return BWLA_ERR_ALIGN;
    const bwla_psp_plan plan = bwla_make_psp_plan(M, layer->K, bwla_rank_u(layer));
    const size_t need = rq_ws_bytes(layer, plan, M);
    if (need > 0 && (!d_ws || ws_bytes < need)) return d_ws ? BWLA_ERR_BUFSIZE : BWLA_ERR_NULL;
    hipStream_t st = (hipStream_t)stream;
    // one launch when the shape allows it
    bool done = false;
    if (bwla_launch_decode_layer(layer, d_X, xdtype, M, d_q, d_scale, d_qsum, d_T, need > 0 ? d_ws : nullptr, d_Y, d_acc, st,
                                 &done, false, act_bits) != hipSuccess)
        return BWLA_ERR_HIP;
    if (done) return BWLA_OK;
    s = bwla_rotate_quant_bits(layer, d_X, xdtype, act_bits, M, d_q, d_scale, d_qsum, d_T, d_ws, ws_bytes, stream);
    if (s != BWLA_OK) return s;
    return bwla_linear_forward(layer, d_q, d_scale, d_qsum, d_T, M, d_Y, d_acc, stream);
}

bwla_status_t bwla_decode_forward(const bwla_layer_t* layer, const void* d_X, int xdtype, int64_t M,
                                  int8_t* d_q, float* d_scale, int32_t* d_qsum, float* d_T, void* d_ws,
                                  size_t ws_bytes, float* d_Y, int32_t* d_acc, void* stream) {
    return bwla_decode_forward_bits(layer, d_X, xdtype, 6, M, d_q, d_scale, d_qsum, d_T, d_ws, ws_bytes, d_Y, d_acc, stream);
}

bwla_status_t bwla_decode_forward_launches(const bwla_layer_t* layer, int xdtype, int64_t M, int* launches) {
    bwla_status_t s = check_layer(layer);
    if (s != BWLA_OK) return s;
    if (!launches) return BWLA_ERR_NULL;
    if (M <= 0 || M > (int64_t)1 << 24) return BWLA_ERR_SHAPE;
    if (xdtype != BWLA_X_F32 && xdtype != BWLA_X_BF16) return BWLA_ERR_UNSUPPORTED;
    bool one = false;
    // (a scratch pointer that is not NULL, as a caller that sized it by bwla_psp_workspace_size passes)
    if (bwla_launch_decode_layer(layer, layer->d_blob, xdtype, M, nullptr, nullptr, nullptr, nullptr, const_cast<void*>(layer->d_blob), nullptr,
                                 nullptr, nullptr, &one, true) != hipSuccess)
        return BWLA_ERR_HIP;
    *launches = one ? 1 : 2;
    return BWLA_OK;
}

bwla_status_t bwla_decode_forward_static(const bwla_layer_t* layer, const void* d_X, int xdtype, int64_t M,
                                         int8_t* d_q, float* d_scale, int32_t* d_qsum, float* d_T, float* d_Y,
                                         int32_t* d_acc, void* stream) {
    // everything that can be refused is refused before the scratch is touched
    bwla_status_t s = check_layer(layer);
    if (s != BWLA_OK) return s;
    if (M <= 0 || M > (int64_t)1 << 24) return BWLA_ERR_SHAPE;
    const bwla_psp_plan plan = bwla_make_psp_plan(M, layer->K, bwla_rank_u(layer));
    const size_t need = rq_ws_bytes(layer, plan, M);
    if (need > BWLA_STATIC_SCRATCH_BYTES) return BWLA_ERR_BUFSIZE;
    if (!d_X || !d_q || !d_scale || !d_qsum || !d_Y) return BWLA_ERR_NULL;
    if (layer->r > 0 && !d_T) return BWLA_ERR_NULL;
    if (xdtype != BWLA_X_F32 && xdtype != BWLA_X_BF16) return BWLA_ERR_UNSUPPORTED;
    if (!aligned16(d_X) || !aligned16(d_q) || !aligned16(d_Y) || (d_T && !aligned16(d_T)) ||
        (d_acc && !aligned16(d_acc)))
        return BWLA_ERR_ALIGN;
    void* ws = nullptr;
    if (static_scratch_ptr(&ws) != hipSuccess) return BWLA_ERR_HIP;
    if (need > 0) {
        // the arrival counts of the scratch must read zero; a kernel clears them (a memset node would
        // not replay reliably from a captured graph)
        const int words = (int)(bwla_psp_counter_bytes(M) / sizeof(uint32_t));
        clear_counts_kernel<<<dim3((unsigned)((words + 255) / 256)), dim3(256), 0, (hipStream_t)stream>>>(
            (uint32_t*)ws, (int)(BWLA_WS_HEAD / sizeof(uint32_t)), words);
        if (hipGetLastError() != hipSuccess) return BWLA_ERR_HIP;
    }
    return bwla_decode_forward(layer, d_X, xdtype, M, d_q, d_scale, d_qsum, d_T, ws, BWLA_STATIC_SCRATCH_BYTES, d_Y,
                               d_acc, stream);
}

bwla_status_t bwla_code_sums(const int8_t* d_q, int64_t M, int64_t K, int32_t* d_qsum, void* stream) {
    if (!d_q || !d_qsum) return BWLA_ERR_NULL;
    if (M <= 0 || K <= 0 || M > (int64_t)1 << 24) return BWLA_ERR_SHAPE;
    if (K % 32 != 0 || K > BWLA_MAX_K) return BWLA_ERR_UNSUPPORTED;
    if (!aligned16(d_q)) return BWLA_ERR_ALIGN;
    return bwla_launch_code_sums(d_q, M, K, d_qsum, (hipStream_t)stream) == hipSuccess ? BWLA_OK : BWLA_ERR_HIP;
}

bwla_status_t bwla_linear_forward(const bwla_layer_t* layer, const int8_t* d_q, const float* d_scale,
                                  const int32_t* d_qsum, const float* d_T, int64_t M, float* d_Y,
                                  int32_t* d_acc, void* stream) {
    bwla_status_t s = check_layer(layer);
    if (s != BWLA_OK) return s;
    if (!d_q || !d_scale || !d_qsum || !d_Y) return BWLA_ERR_NULL;
    if (layer->r > 0 && !d_T) return BWLA_ERR_NULL;
    if (M <= 0 || M > (int64_t)1 << 24) return BWLA_ERR_SHAPE;
    if (!aligned16(d_q) || !aligned16(d_Y) || (d_T && !aligned16(d_T)) || (d_acc && !aligned16(d_acc)))
        return BWLA_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    hipError_t e;
    if (bwla_gemm_decode_bs_supported(M, layer->K, layer->r))
        e = bwla_launch_gemm_decode_bs(layer, d_q, d_scale, d_qsum, d_T, M, d_Y, d_acc, st);
    else if (M <= 16 && bwla_gemm_decode_lds(M, layer->K) <= DECODE_LDS_LIMIT)
        e = bwla_launch_gemm_decode(layer, d_q, d_scale, d_qsum, d_T, M, d_Y, d_acc, st);
    else
        e = bwla_launch_gemm_prefill(layer, d_q, d_scale, d_qsum, d_T, M, d_Y, d_acc, st);
    return e == hipSuccess ? BWLA_OK : BWLA_ERR_HIP;
}

bwla_status_t bwla_pack_codes_a4(const int8_t* d_q, int64_t M, int64_t K, uint8_t* d_q4, void* stream) {
    if (!d_q || !d_q4) return BWLA_ERR_NULL;
    if (M <= 0 || K <= 0 || M > (int64_t)1 << 24) return BWLA_ERR_SHAPE;
    if ((K & 31) != 0 || K > BWLA_MAX_K) return BWLA_ERR_UNSUPPORTED;
    if (!aligned16(d_q) || !aligned16(d_q4)) return BWLA_ERR_ALIGN;
    return bwla_launch_pack_codes_a4(d_q, M, K, d_q4, (hipStream_t)stream) == hipSuccess ? BWLA_OK : BWLA_ERR_HIP;
}

bwla_status_t bwla_linear_forward_a4(const bwla_layer_t* layer, const uint8_t* d_q4, const float* d_scale,
                                     const int32_t* d_qsum, const float* d_T, int64_t M, float* d_Y,
                                     int32_t* d_acc, void* stream) {
    bwla_status_t s = check_layer(layer);
    if (s != BWLA_OK) return s;
    if (!d_q4 || !d_scale || !d_qsum || !d_Y) return BWLA_ERR_NULL;
    if (layer->r > 0 && !d_T) return BWLA_ERR_NULL;
    if (M <= 0 || M > (int64_t)1 << 24) return BWLA_ERR_SHAPE;
    if (!aligned16(d_q4) || !aligned16(d_Y) || (d_T && !aligned16(d_T)) || (d_acc && !aligned16(d_acc)))
        return BWLA_ERR_ALIGN;
    // the streaming prefill kernel is the one that unpacks nibbles in its operand path
    if (M <= 16 || !bwla_gemm_prefill_streams(layer)) return BWLA_ERR_UNSUPPORTED;
    const hipError_t e = bwla_launch_gemm_prefill(layer, reinterpret_cast<const int8_t*>(d_q4), d_scale, d_qsum, d_T, M,
                                                  d_Y, d_acc, (hipStream_t)stream, nullptr, true);
    return e == hipSuccess ? BWLA_OK : BWLA_ERR_HIP;
}

// which GEMM serves the layer at M tokens, as bwla_linear_forward picks it, if that kernel can gate
// in its epilogue: 1 decode kernel, 2 streaming prefill kernel, 0 neither (Y goes through scratch)
static int swiglu_path(const bwla_layer_t* layer, int64_t M) {
    if (bwla_gemm_decode_bs_supported(M, layer->K, layer->r)) return 1;
    if (M <= 16 && bwla_gemm_decode_lds(M, layer->K) <= DECODE_LDS_LIMIT) return 0;
    return bwla_gemm_prefill_streams(layer) ? 2 : 0;
}

bwla_status_t bwla_swiglu_workspace_size(const bwla_layer_t* layer, int64_t M, size_t* bytes) {
    if (!bytes) return BWLA_ERR_NULL;
    bwla_status_t s = check_layer(layer);
    if (s != BWLA_OK) return s;
    if (M <= 0 || M > (int64_t)1 << 24 || (layer->N & 1) != 0) return BWLA_ERR_SHAPE;
    *bytes = swiglu_path(layer, M) != 0 ? 0 : (size_t)bwla_align256((uint64_t)M * (uint64_t)layer->N * sizeof(float));
    return BWLA_OK;
}

bwla_status_t bwla_linear_forward_swiglu(const bwla_layer_t* layer, const int8_t* d_q, const float* d_scale,
                                         const int32_t* d_qsum, const float* d_T, int64_t M, void* d_H,
                                         void* d_ws, size_t ws_bytes, void* stream) {
    size_t need = 0;
    bwla_status_t s = bwla_swiglu_workspace_size(layer, M, &need);
    if (s != BWLA_OK) return s;
    if (!d_q || !d_scale || !d_qsum || !d_H) return BWLA_ERR_NULL;
    if (layer->r > 0 && !d_T) return BWLA_ERR_NULL;
    if (need > 0 && !d_ws) return BWLA_ERR_NULL;
    if (ws_bytes < need) return BWLA_ERR_BUFSIZE;
    if (!aligned16(d_q) || !aligned16(d_H) || (d_T && !aligned16(d_T)) || (need > 0 && !aligned16(d_ws)))
        return BWLA_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    const int path = swiglu_path(layer, M);
    if (path == 1)      // the kernel gates in its epilogue: no M x N intermediate exists
        return bwla_launch_gemm_decode_bs(layer, d_q, d_scale, d_qsum, d_T, M, nullptr, nullptr, st,
                                          (uint16_t*)d_H) == hipSuccess ? BWLA_OK : BWLA_ERR_HIP;
    if (path == 2)
        return bwla_launch_gemm_prefill(layer, d_q, d_scale, d_qsum, d_T, M, nullptr, nullptr, st,
                                        (uint16_t*)d_H) == hipSuccess ? BWLA_OK : BWLA_ERR_HIP;
    s = bwla_linear_forward(layer, d_q, d_scale, d_qsum, d_T, M, (float*)d_ws, nullptr, stream);
    if (s != BWLA_OK) return s;
    return bwla_launch_swiglu_rows((const float*)d_ws, M, layer->N, (uint16_t*)d_H, st) == hipSuccess ? BWLA_OK
                                                                                                    : BWLA_ERR_HIP;
}

}  // extern "C"
