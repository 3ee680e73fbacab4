/*
 * bwla.h -- C ABI of the MI355X (gfx950) W1A6 quantized linear forward of BWLA.
 *
 * The layer computes, for activations X (M tokens x K features) and a layer quantized
 * offline by the paper's method,
 *
 *     Y = dequant( INT6( X (R1 (x) R2) ) . Sign(W_rot)^T ) + (X U) V^T
 *
 * i.e. the Orthogonal-Kronecker rotation applied online to the activations (paper Sec. 3.1
 * "Orthogonal-Kronecker Transformation"), per-token low-bit activation quantization (Sec. 4.1
 * "Implementation Details"; here symmetric INT6, codes in [-31, 31]), the product with the
 * binarized weights and their per-output-channel scales (Sec. 3 "Discussion", Eq. 1-4, without
 * the shift), and the rank-r Proximal-SVD-Projection branch added back (Sec. 3.2: the binarized
 * matrix is W - M with M = A B; here V = A (N x r) and U = B^T (K x r)).
 *
 * Conventions for every call
 *   - All `d_*` pointers are DEVICE pointers on the current HIP device, owned by the caller,
 *     at least 16-byte aligned.  The library never allocates or frees device memory and keeps
 *     nothing of a caller's between calls (what it caches per process -- the compute-unit count of
 *     each device, the kernels whose shared-memory limit it has already raised -- is guarded and
 *     may be used from several host threads).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls enqueue
 *     work and return; they do not synchronize.
 *   - Return value is a bwla_status_t.  Arguments are validated on the host before anything is
 *     enqueued; a failed check enqueues nothing.  A failed launch returns BWLA_ERR_HIP.
 *   - Matrices are dense row-major.
 */
#ifndef BWLA_H
#define BWLA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* The entry points below are the only symbols the shared library exports. */
#define BWLA_API __attribute__((visibility("default")))

typedef enum {
    BWLA_OK = 0,
    BWLA_ERR_NULL = 1,         /* a required pointer is NULL */
    BWLA_ERR_SHAPE = 2,        /* inconsistent or non-positive dimensions */
    BWLA_ERR_ALIGN = 3,        /* a device pointer is not 16-byte aligned */
    BWLA_ERR_BUFSIZE = 4,      /* a caller buffer is too small */
    BWLA_ERR_UNSUPPORTED = 5,  /* valid but outside what the kernels cover */
    BWLA_ERR_HIP = 6           /* the HIP runtime reported an error */
} bwla_status_t;

typedef enum {
    BWLA_X_F32 = 0,            /* activations are float */
    BWLA_X_BF16 = 1            /* activations are bfloat16 (raw uint16 storage) */
} bwla_xdtype_t;

/* Limits of the kernels (checked; violations give BWLA_ERR_UNSUPPORTED). */
#define BWLA_MAX_RANK 128      /* PSP rank r */
#define BWLA_MAX_K 32768       /* in-features; also requires K % 32 == 0 */
#define BWLA_MAX_FACTOR 256    /* n1, n2 */

/*
 * Descriptor of one packed layer: plain data, may be copied freely.  Filled by
 * bwla_pack_weights; offsets are byte offsets into the caller-owned device blob.
 * Layout of the blob (each section 256-byte aligned):
 *   bits   sign bits of W_rot, tiled for the kernels (see bwla_unpack_signs for the
 *          interchange view); 16-row tiles x 512-column chunks, 1 KiB each
 *   alpha  N fp16, alpha_n = mean_k |W_rot[n,k]|            (paper App. A.2.4)
 *   V      N x rp fp16 row-major, rp = r rounded up to a multiple of 16, zero padded
 *   U      rp * K fp16 in MFMA operand order: 1 KiB blocks [16-column tile][32-row step], inside a
 *          block lane lg * 16 + li holds U[32 step + 8 lg + e][16 tile + li], e = 0..7; columns
 *          r..rp-1 zero
 *   R1     n1 x n1 fp32 row-major;  R2  n2 x n2 fp32 row-major
 *   R1p, R2p  the same factors transposed and split into three bfloat16 terms each (their sum is
 *          the fp32 value exactly), zero padded: operand layout of the bf16-MFMA rotation
 *   Rd     only for factor pairs that are multiples of 32, n1 up to 256 and n2 up to 160 (off_Rd = 0
 *          otherwise): the
 *          factors once more, in the order in which the kernels with resident factors read them, one
 *          contiguous KiB per MFMA operand -- for pairs of 32 or 64 R2 as three bfloat16 terms (the
 *          single-launch decode kernel's), then R1 and R2 as two fp16 terms of 256 R (22 bits)
 * `mode` is a set of BWLA_MODE_* bits; each adds rank-one terms of the dequantization as extra
 * columns of V (written at pack time) and T (written by bwla_rotate_quant) behind the PSP columns,
 * and r counts them: U keeps r - extra columns.
 *   BWLA_MODE_ASYM_ACT   two columns: V = delta_n * rowsum_n split into two fp16 (rowsum_n = sum_k
 *                        Sign), T = -scale_t * z_t twice (z_t: the token's zero point)
 *   BWLA_MODE_ROW_SHIFT  one column, the last: V = mu_n, T = scale_t * sum_k (q[t,k] - z_t)
 */
#define BWLA_MODE_ROW_SHIFT 1   /* binarization with the row shift (bwla_pack_weights_centered) */
#define BWLA_MODE_ASYM_ACT 2    /* the layer's activations get per-token asymmetric codes */
typedef struct bwla_layer {
    int64_t N, K;
    int32_t n1, n2, r, mode;
    uint64_t off_bits, off_alpha, off_V, off_U, off_R1, off_R2, off_R1p, off_R2p, off_Rd;
    uint64_t blob_bytes;
    const void* d_blob;
} bwla_layer_t;

BWLA_API const char* bwla_status_string(int status);

/* Library ABI version (integer, bumped on incompatible change). */
BWLA_API int bwla_version(void);

/*
 * Kronecker dimension factorization, paper App. A.1 Algorithm 1: n2 is the largest divisor of
 * K not above sqrt(K), n1 = K / n2 (so n1 >= n2).  Host only.
 */
BWLA_API bwla_status_t bwla_kron_factor(int64_t K, int32_t* n1, int32_t* n2);

/* Size in bytes of the packed blob for a layer of this shape.  Host only. */
BWLA_API bwla_status_t bwla_packed_size(int64_t N, int64_t K, int32_t n1, int32_t n2, int32_t r,
                               size_t* bytes);

/*
 * Pack one layer (offline step; paper Algorithm 2, "Final binarization", restricted to sign
 * and scale: bit = (W_rot[n,k] > 0), so Sign(0) = -1 as in Eq. 3; alpha_n = mean_k |W_rot[n,k]|
 * accumulated in fp64 and rounded once to fp16).
 *   d_W_rot  N x K fp32, the weight in rotated, PSP-corrected coordinates
 *   d_R1, d_R2  fp32 orthogonal factors, n1 x n1 and n2 x n2, n1 * n2 == K
 *   d_U  K x r fp32, d_V  N x r fp32 (values are rounded to fp16); both may be NULL iff r == 0
 *   d_blob   output, blob_bytes >= bwla_packed_size(...)
 *   out      host descriptor to fill
 * Runs as kernels on `stream`; the inputs may be released once the stream has drained.
 */
BWLA_API bwla_status_t bwla_pack_weights(const float* d_W_rot, const float* d_R1, const float* d_R2,
                                const float* d_U, const float* d_V,
                                int64_t N, int64_t K, int32_t n1, int32_t n2, int32_t r,
                                void* d_blob, size_t blob_bytes, void* stream,
                                bwla_layer_t* out);

/*
 * The same with the row shift of the paper's binarization (Sec. 3 "Discussion", Eq. 1-2 and 4):
 *   mu_n = mean_k W_rot[n,k] (fp64 accumulation), bit = (W_rot[n,k] - mu_n > 0),
 *   delta_n = mean_k |W_rot[n,k] - mu_n| (stored where alpha is), W_deq = delta_n Sign(.) + mu_n,
 * so that Y[t,n] = scale_t * (delta_n * acc[t,n] + mu_n * qsum_t) + sum_j T[t,j] V[n,j].
 * mu_n is stored in fp16 as one more column of V; the layer's r becomes r + 1 (at most
 * BWLA_MAX_RANK), mode = BWLA_MODE_ROW_SHIFT.  Arguments as for bwla_pack_weights / bwla_packed_size, with r
 * the PSP rank (columns of d_U and d_V).
 */
BWLA_API bwla_status_t bwla_packed_size_centered(int64_t N, int64_t K, int32_t n1, int32_t n2, int32_t r,
                                        size_t* bytes);
BWLA_API bwla_status_t bwla_pack_weights_centered(const float* d_W_rot, const float* d_R1, const float* d_R2,
                                         const float* d_U, const float* d_V,
                                         int64_t N, int64_t K, int32_t n1, int32_t n2, int32_t r,
                                         void* d_blob, size_t blob_bytes, void* stream,
                                         bwla_layer_t* out);

/*
 * The general form: `mode` is any set of BWLA_MODE_* bits (0: bwla_pack_weights; ROW_SHIFT:
 * bwla_pack_weights_centered).  BWLA_MODE_ASYM_ACT prepares the layer for per-token asymmetric
 * activation codes (paper Sec. 4.1 names them; the min-max affine form is this library's reading):
 * bwla_rotate_quant then quantizes each token over [lo, hi] = [min(min_k x, 0), max(max_k x, 0)] with
 * step scale_t = (hi - lo) / (2^b - 1) and zero point z_t = rint(-lo / scale_t), stores the codes
 * with an offset so that they fit int8 (q - 2^(b-1); b <= 7), and the zero point leaves the
 * accumulator as the rank-one term  sum_k (q - z) Sign = sum_k q Sign - z * rowsum_n:
 *   Y[t,n] = scale_t * (delta_n * (acc - z rowsum_n) + mu_n * sum_k (q - z)) + sum_j T[t,j] V[n,j].
 * The layer's r becomes r + (2 if ASYM_ACT) + (1 if ROW_SHIFT), at most BWLA_MAX_RANK.
 */
BWLA_API bwla_status_t bwla_packed_size_mode(int64_t N, int64_t K, int32_t n1, int32_t n2, int32_t r, int32_t mode,
                                    size_t* bytes);
BWLA_API bwla_status_t bwla_pack_weights_mode(const float* d_W_rot, const float* d_R1, const float* d_R2,
                                     const float* d_U, const float* d_V,
                                     int64_t N, int64_t K, int32_t n1, int32_t n2, int32_t r, int32_t mode,
                                     void* d_blob, size_t blob_bytes, void* stream,
                                     bwla_layer_t* out);

/*
 * Inspection helper: expand the packed sign bits to the interchange view, an N x K int8
 * matrix of +1 / -1 (bit 1 <-> +1), and copy alpha as fp32.  d_alpha may be NULL.
 */
BWLA_API bwla_status_t bwla_unpack_signs(const bwla_layer_t* layer, int8_t* d_sgn, float* d_alpha,
                                void* stream);

/*
 * Bytes of scratch bwla_rotate_quant wants for M tokens: split-K partial sums of X U with their
 * arrival counters, and, for a few tokens of a layer with a large factor R1 (six or more 16-row
 * tiles), the rotated values in fp32 and their extremes between the two launches the rotation
 * then takes.  Returns 0 bytes when neither is used.
 * The scratch must be zero-filled once when it is allocated and then left to the library: its
 * first 7168 bytes are the exchange area of bwla_decode_forward's single-launch kernel (an epoch
 * that every such launch moves on, arrival counts that every launch returns to zero, partial
 * sums tagged with their epoch), then comes one arrival counter per 16-token tile, which every
 * call returns to zero; everything behind them is overwritten by each call.  One scratch may
 * serve calls on different layers and token counts; two calls that overlap in time must not
 * share one.
 */
BWLA_API bwla_status_t bwla_psp_workspace_size(const bwla_layer_t* layer, int64_t M, size_t* bytes);

/*
 * Steps 1, 2 and the first half of 4 of the forward:
 *   X~ = X (R1 (x) R2) evaluated as R1^T V R2 on each token reshaped row-major to n1 x n2
 *        (paper Sec. 3.1; App. A.2.2), fp32 accumulation;
 *   amax_t = max_k |X~[t,k]|, scale_t = amax_t / 31, q = clamp(rint(X~ * 31 / amax_t), -31, 31)
 *        with ties to even; an all-zero token gives q = 0 and scale 0;
 *   qsum_t = sum_k q[t,k];
 *   T = X U (M x r, fp32 accumulation, from the un-rotated un-quantized X; Sec. 3.2).
 *   d_X      M x K, float or bf16 according to xdtype
 *   d_q      out, M x K int8;  d_scale out, M fp32;  d_qsum out, M int32
 *   d_T      out, M x r fp32 (NULL iff r == 0); the leading columns are X U, the columns that the
 *            layer's mode adds follow (see bwla_layer_t)
 * For a layer with BWLA_MODE_ASYM_ACT the codes are the asymmetric ones (see bwla_pack_weights_mode):
 * d_q holds q - 2^(b-1), d_qsum their sums, d_scale the step (hi - lo) / (2^b - 1).
 *   d_ws     scratch of ws_bytes >= bwla_psp_workspace_size(layer, M) (NULL allowed when that is 0)
 */
BWLA_API bwla_status_t bwla_rotate_quant(const bwla_layer_t* layer, const void* d_X, int xdtype, int64_t M,
                                int8_t* d_q, float* d_scale, int32_t* d_qsum, float* d_T,
                                void* d_ws, size_t ws_bytes, void* stream);

/*
 * The same with another activation code width (the paper evaluates A6 and A4, Tables 1-3, and times
 * W1A8, Sec. 4.4): symmetric codes in [-qmax, qmax], qmax = 2^(act_bits-1) - 1, scale = amax / qmax,
 * act_bits in 2..8 (else BWLA_ERR_UNSUPPORTED), still one code per int8.  bwla_rotate_quant is
 * act_bits = 6.  bwla_linear_forward takes the codes of any width; bwla_decode_forward is 6-bit.
 */
BWLA_API bwla_status_t bwla_rotate_quant_bits(const bwla_layer_t* layer, const void* d_X, int xdtype, int act_bits,
                                     int64_t M, int8_t* d_q, float* d_scale, int32_t* d_qsum, float* d_T,
                                     void* d_ws, size_t ws_bytes, void* stream);

/* qsum_t = sum_k q[t,k] for codes that did not come from bwla_rotate_quant (codes in [-127, 127],
 * see bwla_linear_forward). */
BWLA_API bwla_status_t bwla_code_sums(const int8_t* d_q, int64_t M, int64_t K, int32_t* d_qsum, void* stream);

/*
 * Steps 3, 4 (second half) and 5:
 *   acc[t,n] = sum_k q[t,k] * Sign(W_rot[n,k])   exact int32 on INT8 MFMA.  The sign bits are
 *              expanded in registers to 0/1-valued int8 digits b, and the +-1 product is
 *              recovered exactly as 2 * sum_k q b - qsum_t;
 *   Y[t,n]   = scale_t * alpha_n * acc[t,n] + sum_j T[t,j] V[n,j]      (paper Eq. 4; Sec. 3.2)
 *   d_q, d_scale, d_qsum, d_T  as produced by bwla_rotate_quant (d_T NULL iff r == 0).  Codes from
 *            elsewhere (with d_qsum from bwla_code_sums) must lie in [-127, 127]: the kernels negate
 *            the operand of the sign digit byte-wise, which has no +128, so a code of -128 would
 *            give wrong sums without any error being reported
 *   d_Y      out, M x N fp32
 *   d_acc    optional out, M x N int32 raw accumulators (NULL to skip)
 */
BWLA_API bwla_status_t bwla_linear_forward(const bwla_layer_t* layer, const int8_t* d_q, const float* d_scale,
                                  const int32_t* d_qsum, const float* d_T, int64_t M,
                                  float* d_Y, int32_t* d_acc, void* stream);

/*
 * The whole forward of one layer, steps 1-5 above (paper Sec. 3.1, Sec. 4.1, Eq. 3-4, Sec. 3.2), in
 * one call: what bwla_rotate_quant followed by bwla_linear_forward compute, with the same
 * buffers (d_q, d_scale, d_qsum, d_T are still written; same arguments, same errors) and to the
 * same accuracy.  Where the single-launch kernel serves the call, its rotation may add the
 * products in another order than the kernel bwla_rotate_quant picks for the shape, so a code
 * whose value lies on a rounding boundary can differ by one between the two.  For a single
 * bf16 token of a layer whose Kronecker factors are 32 or 64 wide, or 128 x 64 (K = 1024 .. 8192: the
 * attention and up / gate projections of the 4096- and 8192-wide models), with a PSP rank up to 96,
 * symmetric or asymmetric codes and with or without the row shift, everything runs in ONE kernel launch: every
 * workgroup rotates and quantizes the token itself while its sign bits stream in; only the
 * projection T = x U is shared: the first 32 workgroups compute it in eight slices of K and
 * leave the sums, tagged with a per-launch epoch, in the first bytes of d_ws, where every
 * workgroup picks them up (bounded polling; no workgroup ever waits for one that has not been
 * started).  That exchange is why calls that share one d_ws must not overlap.  All other cases
 * run the two launches back to back.
 */
BWLA_API bwla_status_t bwla_decode_forward(const bwla_layer_t* layer, const void* d_X, int xdtype, int64_t M,
                                  int8_t* d_q, float* d_scale, int32_t* d_qsum, float* d_T,
                                  void* d_ws, size_t ws_bytes, float* d_Y, int32_t* d_acc,
                                  void* stream);
/* bwla_decode_forward at another width of the activation codes: act_bits as in bwla_rotate_quant_bits
 * (2..8, else BWLA_ERR_UNSUPPORTED; 8 is the width of the paper's speed run, Sec. 4.4).  The
 * single-launch kernel serves every width of the symmetric codes and every width the asymmetric ones allow. */
BWLA_API bwla_status_t bwla_decode_forward_bits(const bwla_layer_t* layer, const void* d_X, int xdtype, int act_bits,
                                                int64_t M, int8_t* d_q, float* d_scale, int32_t* d_qsum, float* d_T,
                                                void* d_ws, size_t ws_bytes, float* d_Y, int32_t* d_acc,
                                                void* stream);

/*
 * Whether bwla_decode_forward serves (layer, xdtype, M) with its single-launch kernel: *launches
 * (host) = 1, else 2 (bwla_rotate_quant's and bwla_linear_forward's launches back to back; the
 * rotation of a long prefill may itself take more than one).  Launches nothing.
 */
BWLA_API bwla_status_t bwla_decode_forward_launches(const bwla_layer_t* layer, int xdtype, int64_t M, int* launches);

/*
 * bwla_decode_forward for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same inputs,
 * outputs, results and errors as bwla_decode_forward, but the scratch (arrival counters and partial
 * sums of the projection, and for a few tokens of a layer with a large factor R1 the rotated values
 * between the rotation's two launches) lives in a fixed array of BWLA_STATIC_SCRATCH_BYTES inside
 * the library's device image, one per GPU, held until the process ends.  The call allocates
 * nothing and calls no allocating routine; it clears the counters it needs with a small kernel.
 *   - A call whose bwla_psp_workspace_size(layer, M) exceeds BWLA_STATIC_SCRATCH_BYTES returns
 *     BWLA_ERR_BUFSIZE and enqueues nothing (decode batches of the common model widths fit; long
 *     prefills do not: use bwla_decode_forward with a workspace of the caller's).
 *   - Every call on a GPU uses that GPU's one array: calls that may overlap in time on one GPU (two
 *     streams, two host threads) race on it and must be serialized by the caller.
 *   - The first call on a device looks the array's address up (once per device and process).
 */
#define BWLA_STATIC_SCRATCH_BYTES (4u << 20)
BWLA_API bwla_status_t bwla_decode_forward_static(const bwla_layer_t* layer, const void* d_X, int xdtype,
                                                  int64_t M, int8_t* d_q, float* d_scale, int32_t* d_qsum,
                                                  float* d_T, float* d_Y, int32_t* d_acc, void* stream);

/*
 * bwla_linear_forward for the merged gate|up projection of an MLP block, with the block's gate
 * applied before anything is stored (the models the paper quantizes have up, gate and down
 * projections in their MLP blocks: paper App., loss trajectories of the MLP blocks; the
 * nonlinearity is the model's, not the paper's method).  The layer's rows interleave the two
 * projections: packed row 2 i is gate channel i, row 2 i + 1 is up channel i (N even, else
 * BWLA_ERR_SHAPE; the caller stacks W, alpha, V that way before bwla_pack_weights).  With Y as
 * bwla_linear_forward defines it,
 *   H[t, i] = silu(Y[t, 2 i]) * Y[t, 2 i + 1],  silu(g) = g / (1 + exp(-g)),
 * evaluated in fp32 and rounded to bfloat16 (nearest even): the activation format that
 * bwla_rotate_quant of the down projection reads.
 *   d_H      out, M x N / 2 bfloat16, 16-byte aligned
 *   d_ws     scratch of ws_bytes >= bwla_swiglu_workspace_size(layer, M): 0 where the GEMM kernel
 *            that serves the shape gates in its epilogue and Y never exists (up to 16 tokens; more
 *            tokens when K is a multiple of 128 and N >= 32), else M x N fp32 for Y, gated by one
 *            more launch (NULL allowed when 0); not kept between calls
 * Other arguments and errors as bwla_linear_forward.
 */
BWLA_API bwla_status_t bwla_swiglu_workspace_size(const bwla_layer_t* layer, int64_t M, size_t* bytes);
BWLA_API bwla_status_t bwla_linear_forward_swiglu(const bwla_layer_t* layer, const int8_t* d_q, const float* d_scale,
                                         const int32_t* d_qsum, const float* d_T, int64_t M, void* d_H,
                                         void* d_ws, size_t ws_bytes, void* stream);

/*
 * 4-bit activation codes two to a byte (paper Table 3 reports W1A4: codes in [-7, 7]), which halves the
 * bytes the prefill GEMM reads per token.
 *   bwla_pack_codes_a4      d_q (M x K int8, every code in [-8, 7], as bwla_rotate_quant_bits writes them
 *                           with act_bits = 4) -> d_q4 (M x K / 2 bytes, 16-byte aligned).  Layout: K is cut
 *                           into runs of 32 codes; byte b (0..15) of run j holds code 32 j + b in its low
 *                           nibble and code 32 j + 16 + b in its high nibble, two's complement.  K must be a
 *                           multiple of 32 (else BWLA_ERR_UNSUPPORTED).
 *   bwla_linear_forward_a4  bwla_linear_forward on such codes; every other argument, the results (bit for bit,
 *                           accumulators included) and the errors as there.  The nibbles are unpacked in the
 *                           operand path of the streaming prefill kernel; shapes that kernel does not take
 *                           (M <= 16, K not a multiple of 128, N < 32) return BWLA_ERR_UNSUPPORTED.
 */
BWLA_API bwla_status_t bwla_pack_codes_a4(const int8_t* d_q, int64_t M, int64_t K, uint8_t* d_q4, void* stream);
BWLA_API bwla_status_t bwla_linear_forward_a4(const bwla_layer_t* layer, const uint8_t* d_q4, const float* d_scale,
                                              const int32_t* d_qsum, const float* d_T, int64_t M, float* d_Y,
                                              int32_t* d_acc, void* stream);

/*
 * Measurement aids for benchmarks, not steps of the method: the ceilings this GPU actually reaches,
 * to quote the forward's kernels against next to the published peaks, and two latencies.
 *   bwla_probe_hbm_read   one launch that reads `bytes` (a multiple of 16) from d_src (device,
 *                         16-byte aligned) with coalesced 16-byte loads and writes a checksum per
 *                         workgroup to d_sink (device, sink_bytes >= 32 KiB is always enough, else
 *                         BWLA_ERR_BUFSIZE).  Bytes / launch duration is the read bandwidth a kernel of
 *                         that size can reach.
 *   bwla_probe_mfma_int8  one launch in which every wavefront issues 4 * iters independent 16x16x64
 *                         INT8 MFMAs (1 <= iters <= 2^20) on register operands; *ops_out (host) gets
 *                         the launch's operation count (2 per multiply-add), d_sink (device,
 *                         >= 16 KiB) a checksum.
 *   bwla_probe_empty_launch  one launch of a kernel that does nothing, in the launch shape of the decode
 *                         kernels (one workgroup of 512 threads per CU): timed back to back from a graph
 *                         it gives the period at which dependent launches can follow one another.
 *   bwla_probe_load_latency  one lane issues `iters` (1 .. 2^24) loads of four bytes from d_buf (device,
 *                         `bytes` long, a multiple of 4), each at an index that depends on the value the
 *                         one before returned: the index moves on by stride_bytes (a multiple of 4,
 *                         0 < stride_bytes <= bytes - 4; plus one word when the loaded word is odd) and wraps
 *                         at the end.  d_out (device, 16 bytes, 8-byte aligned) gets the duration of the
 *                         walk in ticks of the GPU's constant 100 MHz counter (10 ns each) and the last
 *                         index.  Ticks * 10 / iters is the latency of one dependent load in nanoseconds: of
 *                         a miss everywhere when the walk never comes back to a line, of the L2 when the
 *                         buffer was read just before and fits it.
 *   bwla_probe_clock      one launch of one wavefront that writes the GPU's constant 100 MHz counter (ticks
 *                         of 10 ns) to d_out (device, 8 bytes, 8-byte aligned).  Two of them around a
 *                         sequence of launches -- also inside a captured graph -- give the time the GPU
 *                         spent on the sequence without the host's part of getting it started.
 * All enqueue on `stream`, own no memory, and return the usual codes.
 */
BWLA_API bwla_status_t bwla_probe_hbm_read(const void* d_src, size_t bytes, void* d_sink, size_t sink_bytes, void* stream);
BWLA_API bwla_status_t bwla_probe_mfma_int8(int iters, void* d_sink, size_t sink_bytes, int64_t* ops_out, void* stream);
BWLA_API bwla_status_t bwla_probe_empty_launch(void* stream);
BWLA_API bwla_status_t bwla_probe_clock(void* d_out, void* stream);
BWLA_API bwla_status_t bwla_probe_load_latency(const void* d_buf, size_t bytes, size_t stride_bytes, int iters,
                                               void* d_out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* BWLA_H */
