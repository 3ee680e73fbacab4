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
// the transposed fp16 U) straight from global memory and multiplies on fp32 MFMA.  With several
// slices, every workgroup writes its partial tile to scratch and the one that arrives last adds
// them in slice order.
#include "bwla_internal.h"
#include "gemm_decode_bs_device.h"

namespace {

#ifdef BWLA_TRACE
// Development aid (off in the product build): cycle stamps are kept in registers and written
// once at the end of the workgroup, so that taking them adds no memory waits.
__device__ long long bwla_rq_trace_buf[16 * 8 * 16];
#define RQTRACE_DECL long long rq_tr[10] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0}
#define RQTRACE(slot) do { rq_tr[slot] = __builtin_readcyclecounter(); } while (0)
#define RQTRACE_FLUSH do { if ((threadIdx.x & 63) == 0 && blockIdx.x < 16) { _Pragma("unroll") for (int i_ = 0; i_ < 10; ++i_) bwla_rq_trace_buf[(blockIdx.x * 8 + (threadIdx.x >> 6)) * 16 + i_] = rq_tr[i_]; } } while (0)
#else
#define RQTRACE_DECL do { } while (0)
#define RQTRACE(slot) do { } while (0)
#define RQTRACE_FLUSH do { } while (0)
#endif

// How a token is quantized, from its largest and smallest rotated value (hi >= 0 >= lo: the
// reductions start at zero, which also covers the zero padding).
//   symmetric:   codes rint(x * qmax / amax) in [-qmax, qmax], scale = amax / qmax
//   asymmetric:  L = 2 qmax + 1 steps over [lo, hi], scale = (hi - lo) / L, zero point
//                z = rint(-lo / scale); the code q = rint(x / scale) + z in [0, L] is stored as
//                q - (qmax + 1), so zc = z - (qmax + 1) is what the stored code has to lose
struct QuantPlan {
    float inv, zc, cmin, cmax;
};
__device__ __forceinline__ QuantPlan quant_plan(float hi, float lo, float qmax, bool asym) {
    QuantPlan p;
    if (asym) {
        const float L = 2.0f * qmax + 1.0f, span = hi - lo;
        p.inv = span > 0.0f ? L / span : 0.0f;
        p.zc = rintf(-lo * p.inv) - (qmax + 1.0f);
        if (!(span > 0.0f)) p.zc = -(qmax + 1.0f);      // all-zero token: q = z = 0
        p.cmin = -(qmax + 1.0f);
        p.cmax = qmax;
    } else {
        const float amax = fmaxf(hi, -lo);
        p.inv = amax > 0.0f ? qmax / amax : 0.0f;
        p.zc = 0.0f;
        p.cmin = -qmax;
        p.cmax = qmax;
    }
    return p;
}
// the token's step (only the thread that writes it out needs it)
__device__ __forceinline__ float quant_scale(float hi, float lo, float qmax, bool asym) {
    return asym ? (hi - lo) / (2.0f * qmax + 1.0f) : fmaxf(hi, -lo) / qmax;
}
__device__ __forceinline__ int quant_code(float x, const QuantPlan& p) {
    return (int)fminf(fmaxf(rintf(x * p.inv) + p.zc, p.cmin), p.cmax);
}
// The entries of T that the layer's mode adds for token t (tmode points at the first of them in
// row 0, or is NULL): asymmetric codes: -scale * zc, twice; row shift: scale * sum_k (q - z).
__device__ __forceinline__ void quant_extras(float* tmode, int tp, int64_t t, bool asym, bool shift,
                                             const QuantPlan& p, float scale, int tot, int64_t K) {
    if (!tmode) return;
    float* row = tmode + t * tp;
    int c = 0;
    if (asym) { row[0] = row[1] = -(scale * p.zc); c = 2; }
    if (shift) row[c] = scale * ((float)tot - (float)K * p.zc);
}

constexpr int RQ_THREADS = 512;
constexpr int RQ_WAVES = RQ_THREADS / 64;
constexpr int RQ_MAXT = 16;          // 16x16 output tiles per wavefront
constexpr int RQ_CK = 16;            // contraction indices per streamed factor chunk
constexpr int RQ_CLD = RQ_CK + 4;    // LDS pitch of a streamed chunk row
constexpr int RQ_RING = 3;           // streamed chunks in flight (registers)
constexpr int PP_SLICE = 512;        // columns of K per projection workgroup
constexpr int PP_MAXJT = BWLA_MAX_RANK / 16;
constexpr size_t RQ_LDS_LIMIT = 160 * 1024 - 256;   // leaves room for the few static bytes

__host__ __device__ inline int rq_pad16(int n) { return (n + 15) & ~15; }

// LDS layout of a rotation workgroup (floats).  Every matrix is stored so that the MFMA
// contraction index runs along a row with a pitch of (multiple of 16) + 4: a lane then fetches
// four consecutive contraction values of its operand row with one 128-bit read, and the 16 rows
// of a lane group fall into disjoint banks.
//   region  V  [a][b]  pitch ldv   (token, stage-1 A)   later  ZT [d][a]  pitch ldzt (stage-2 A)
//   R2T [d][b] pitch ld2t (stage-1 B),  R1T [c][a] pitch ld1t (stage-2 B)      -- resident mode
//   two chunk buffers [row][16] pitch RQ_CLD                                   -- streaming mode
struct RqShape {
    int n1, n2, n1p, n2p, ldv, ldzt, ld2t, ld1t, region, nmaxp;
    bool resident;
    size_t lds_bytes;
};

__host__ __device__ inline RqShape rq_shape(int n1, int n2) {
    RqShape s;
    s.n1 = n1; s.n2 = n2;
    s.n1p = rq_pad16(n1); s.n2p = rq_pad16(n2);
    s.ldv = s.n2p + 4; s.ldzt = s.n1p + 4; s.ld2t = s.n2p + 4; s.ld1t = s.n1p + 4;
    const int rv = s.n1p * s.ldv, rz = s.n2p * s.ldzt;
    s.region = rv > rz ? rv : rz;
    s.nmaxp = s.n1p > s.n2p ? s.n1p : s.n2p;
    const size_t res = ((size_t)s.region + (size_t)s.n2p * s.ld2t + (size_t)s.n1p * s.ld1t + 64) * sizeof(float);
    const size_t str = ((size_t)s.region + (size_t)2 * s.nmaxp * RQ_CLD + 64) * sizeof(float);
    s.resident = res <= RQ_LDS_LIMIT;
    s.lds_bytes = s.resident ? res : str;
    return s;
}

__host__ __device__ inline size_t pp_lds_bytes(int r, int waves = RQ_WAVES) {
    const int rp = ((r + 15) >> 4) * 16;
    return (size_t)waves * (rp / 16) * 64 * 16 + 16;                   // cross-wave reduction
}

// Exact n / d for n * d < 2^32 with one multiply-high; index arithmetic on run-time factor
// sizes would otherwise cost a ~30-instruction division sequence per use.
struct FastDiv {
    uint32_t d, m;
    __device__ explicit FastDiv(uint32_t dd) : d(dd), m(dd > 1 ? 0xFFFFFFFFu / dd + 1u : 0u) {}
    __device__ __forceinline__ int div(int n) const { return d > 1 ? (int)__umulhi((uint32_t)n, m) : n; }
};

// ================================================================== rotation of one token
template <bool BF16>
__device__ __forceinline__ void store_token_vec(float* d, const uint4& v) {
    // d is 16-byte aligned (pitches and column offsets are multiples of four floats)
    float4* d4 = reinterpret_cast<float4*>(d);
    if (BF16) {
        d4[0] = make_float4(__uint_as_float(v.x << 16), __uint_as_float(v.x & 0xffff0000u),
                            __uint_as_float(v.y << 16), __uint_as_float(v.y & 0xffff0000u));
        d4[1] = make_float4(__uint_as_float(v.z << 16), __uint_as_float(v.z & 0xffff0000u),
                            __uint_as_float(v.w << 16), __uint_as_float(v.w & 0xffff0000u));
    } else {
        d4[0] = make_float4(__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w));
    }
}

// Token (and, in resident mode, R2 and R1 transposed) into LDS.  Every global load of a batch is
// issued before the first use, so that a decode token pays one memory round trip.  Items are
// 16-byte vectors [token | R2 | R1] when the shapes allow it; odd shapes take scalar loops.
template <bool BF16>
__device__ __forceinline__ void fill_lds(const void* __restrict__ X, int64_t row_off, int n1, int n2,
                                         const float* __restrict__ R1, const float* __restrict__ R2,
                                         const RqShape& sh, float* V, float* r2t, float* r1t) {
    constexpr int VEC = BF16 ? 8 : 4;
    const bool with_factors = sh.resident;
    // zero the padding first (disjoint from everything written below)
    if (n2 != sh.n2p || n1 != sh.n1p) {
        for (int idx = threadIdx.x; idx < sh.n1p * sh.n2p; idx += RQ_THREADS) {
            const int a = idx / sh.n2p, b = idx - a * sh.n2p;
            if (a >= n1 || b >= n2) V[a * sh.ldv + b] = 0.0f;
        }
        if (with_factors) {
            for (int idx = threadIdx.x; idx < sh.n2p * sh.n2p; idx += RQ_THREADS) {
                const int d = idx / sh.n2p, b = idx - d * sh.n2p;
                if (d >= n2 || b >= n2) r2t[d * sh.ld2t + b] = 0.0f;
            }
            for (int idx = threadIdx.x; idx < sh.n1p * sh.n1p; idx += RQ_THREADS) {
                const int c = idx / sh.n1p, a = idx - c * sh.n1p;
                if (c >= n1 || a >= n1) r1t[c * sh.ld1t + a] = 0.0f;
            }
        }
    }
    if ((n2 % VEC) == 0 && (n1 & 3) == 0 && (n2 & 3) == 0) {
        const int vpr = n2 / VEC, nx = n1 * vpr;
        // A factor is cut into blocks of 16 rows k x 4 vectors (16 columns x): lane l of an item
        // group takes row (l & 15), vector (l >> 4).  A wave then loads 64-byte row pieces and its
        // four transposed scalar stores each hit 64 distinct LDS banks.
        const int q2 = n2 >> 2, kg2 = (n2 + 15) >> 4, nr2 = with_factors ? 64 * kg2 * ((q2 + 3) >> 2) : 0;
        const int q1 = n1 >> 2, kg1 = (n1 + 15) >> 4, nr1 = with_factors ? 64 * kg1 * ((q1 + 3) >> 2) : 0;
        const int total = nx + nr2 + nr1;
        const FastDiv dvpr(vpr), dkg1(kg1), dkg2(kg2);
        auto factor_item = [&](int it, bool& second, int& k, int& x4) -> bool {
            second = it >= nx + nr2;
            const int j = second ? it - nx - nr2 : it - nx;
            const int l = j & 63, blk = j >> 6;
            const int kg = second ? kg1 : kg2;
            const int xgi = (second ? dkg1 : dkg2).div(blk), kgi = blk - xgi * kg;
            k = 16 * kgi + (l & 15);
            x4 = 4 * xgi + (l >> 4);
            return k < (second ? n1 : n2) && x4 < (second ? q1 : q2);
        };
        for (int base = 0; base < total; base += 8 * RQ_THREADS) {
            uint4 v[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int it = base + e * RQ_THREADS + threadIdx.x;
                v[e] = make_uint4(0, 0, 0, 0);
                if (it < nx) {
                    const int a = dvpr.div(it), b0 = (it - a * vpr) * VEC;
                    const int64_t off = row_off + (int64_t)a * n2 + b0;
                    v[e] = BF16 ? *reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(X) + off)
                                : *reinterpret_cast<const uint4*>(reinterpret_cast<const float*>(X) + off);
                } else if (it < total) {
                    bool second; int k, x4;
                    if (factor_item(it, second, k, x4))
                        v[e] = *reinterpret_cast<const uint4*>((second ? R1 : R2) + (int64_t)k * (second ? n1 : n2) + 4 * x4);
                }
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int it = base + e * RQ_THREADS + threadIdx.x;
                if (it < nx) {
                    const int a = dvpr.div(it), b0 = (it - a * vpr) * VEC;
                    store_token_vec<BF16>(V + a * sh.ldv + b0, v[e]);
                } else if (it < total) {
                    // R[k][x0..x0+3] -> transposed rows x0..x0+3, column k
                    bool second; int k, x4;
                    if (factor_item(it, second, k, x4)) {
                        const int ld = second ? sh.ld1t : sh.ld2t;
                        float* d = (second ? r1t : r2t) + 4 * x4 * ld + k;
                        d[0] = __uint_as_float(v[e].x); d[ld] = __uint_as_float(v[e].y);
                        d[2 * ld] = __uint_as_float(v[e].z); d[3 * ld] = __uint_as_float(v[e].w);
                    }
                }
            }
        }
    } else {
        for (int idx = threadIdx.x; idx < n1 * n2; idx += RQ_THREADS) {
            const int a = idx / n2, b = idx - a * n2;
            const int64_t i = row_off + idx;
            V[a * sh.ldv + b] = BF16 ? bwla_bf16_to_f32(reinterpret_cast<const uint16_t*>(X)[i])
                                     : reinterpret_cast<const float*>(X)[i];
        }
        if (with_factors) {
            for (int idx = threadIdx.x; idx < n2 * n2; idx += RQ_THREADS) {
                const int b = idx / n2, d = idx - b * n2;
                r2t[d * sh.ld2t + b] = R2[idx];
            }
            for (int idx = threadIdx.x; idx < n1 * n1; idx += RQ_THREADS) {
                const int a = idx / n1, c = idx - a * n1;
                r1t[c * sh.ld1t + a] = R1[idx];
            }
        }
    }
}

// one 16-wide contraction group: four MFMA steps fed by one 128-bit LDS read per operand
__device__ __forceinline__ v4f mfma16(const float* ap, const float* bp, v4f acc) {
    const float4 a4 = *reinterpret_cast<const float4*>(ap);
    const float4 b4 = *reinterpret_cast<const float4*>(bp);
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a4.x, b4.x, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a4.y, b4.y, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a4.z, b4.z, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a4.w, b4.w, acc, 0, 0, 0);
    return acc;
}

// Streamed factor chunks (n % 4 == 0): chunk c holds R[16c .. 16c+15][all x]; a thread carries
// two 16-byte vectors of it (slot e: local row kk[e], columns x0[e]..x0[e]+3).  They are stored
// transposed, [x][k_local] with pitch RQ_CLD.
struct ChunkRegs { float4 v[2]; };
struct ChunkSlots { int kk[2], x0[2]; };
// lane l of a 64-item group takes local row (l & 15) and vector (l >> 4) of the group's 16
// columns: 64-byte row pieces from global memory, conflict-free transposed stores (pitch 20
// floats puts the four column groups 16 banks apart)
__device__ __forceinline__ ChunkSlots chunk_slots(int n) {
    ChunkSlots cs;
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const int idx = threadIdx.x + e * RQ_THREADS;
        const int l = idx & 63, grp = idx >> 6;
        cs.x0[e] = (4 * grp + (l >> 4)) << 2;
        cs.kk[e] = cs.x0[e] < n ? (l & 15) : RQ_CK;      // RQ_CK marks an unused slot
    }
    return cs;
}
__device__ __forceinline__ ChunkRegs chunk_fetch(const float* __restrict__ R, int n, int c, const ChunkSlots& cs) {
    ChunkRegs cr;
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const int k = c * RQ_CK + cs.kk[e];
        cr.v[e] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (cs.kk[e] < RQ_CK && k < n) cr.v[e] = *reinterpret_cast<const float4*>(R + (int64_t)k * n + cs.x0[e]);
    }
    return cr;
}
__device__ __forceinline__ void chunk_store(float* dst, const ChunkSlots& cs, const ChunkRegs& cr) {
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        if (cs.kk[e] < RQ_CK) {
            float* d = dst + cs.x0[e] * RQ_CLD + cs.kk[e];
            d[0] = cr.v[e].x; d[RQ_CLD] = cr.v[e].y; d[2 * RQ_CLD] = cr.v[e].z; d[3 * RQ_CLD] = cr.v[e].w;
        }
    }
}

template <bool BF16>
__device__ __forceinline__ void rotate_token(float* lds, const void* __restrict__ X, int64_t t, int64_t K, int n1,
                                             int n2, const float* __restrict__ R1, const float* __restrict__ R2,
                                             int8_t* __restrict__ q, float* __restrict__ scale,
                                             int32_t* __restrict__ qsum, float* __restrict__ tmode, int tp,
                                             float qmax, bool asym, bool shift) {
    const RqShape sh = rq_shape(n1, n2);
    float* reg = lds;                                              // V, later ZT
    float* fac = lds + sh.region;                                  // R2T | R1T (resident) or two chunk buffers
    float* red = fac + (sh.resident ? sh.n2p * sh.ld2t + sh.n1p * sh.ld1t : 2 * sh.nmaxp * RQ_CLD);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // wave-uniform: tile indices stay scalar
    const int li = lane & 15, lg = lane >> 4;
    const int tiles1 = sh.n1p >> 4, tiles2 = sh.n2p >> 4;         // 16-row tiles along a/c and along b/d
    const int tiles = tiles1 * tiles2;
    const int my_tiles = (tiles - wave + RQ_WAVES - 1) / RQ_WAVES;      // tiles wave, wave+8, ...
    const FastDiv dt1(tiles1), dt2(tiles2);
    // Tiles are processed in pairs so that two independent read->MFMA chains overlap; an odd
    // last tile is paired with a copy of itself whose result is never used.
#define RQ_PAIR_SLOTS(g) const int s0 = 2 * (g), s1 = (2 * (g) + 1 < my_tiles) ? 2 * (g) + 1 : 2 * (g)

    v4f acc[RQ_MAXT];
#pragma unroll
    for (int s = 0; s < RQ_MAXT; ++s) acc[s] = v4f{0.f, 0.f, 0.f, 0.f};

    RQTRACE_DECL;
    RQTRACE(0);
    fill_lds<BF16>(X, t * K, n1, n2, R1, R2, sh, reg, fac, fac + sh.n2p * sh.ld2t);

    if (sh.resident) {
        const float* r2t = fac;
        const float* r1t = fac + sh.n2p * sh.ld2t;
        RQTRACE(1);
        __syncthreads();
        RQTRACE(2);
        // stage 1: Z[a][d] = sum_b V[a][b] R2[b][d];   tile (ti over a, tj over d)
#pragma unroll
        for (int g = 0; g < RQ_MAXT / 2; ++g) {
            if (2 * g < my_tiles) {
                RQ_PAIR_SLOTS(g);
                const int tau0 = wave + s0 * RQ_WAVES, tau1 = wave + s1 * RQ_WAVES;
                const int ti0 = dt2.div(tau0), tj0 = tau0 - ti0 * tiles2;
                const int ti1 = dt2.div(tau1), tj1 = tau1 - ti1 * tiles2;
                const float* ap0 = reg + (ti0 * 16 + li) * sh.ldv + 4 * lg;
                const float* bp0 = r2t + (tj0 * 16 + li) * sh.ld2t + 4 * lg;
                const float* ap1 = reg + (ti1 * 16 + li) * sh.ldv + 4 * lg;
                const float* bp1 = r2t + (tj1 * 16 + li) * sh.ld2t + 4 * lg;
#pragma unroll 2
                for (int k = 0; k < sh.n2p; k += 16) {
                    acc[2 * g] = mfma16(ap0 + k, bp0 + k, acc[2 * g]);
                    acc[2 * g + 1] = mfma16(ap1 + k, bp1 + k, acc[2 * g + 1]);
                }
            }
        }
        RQTRACE(3);
        bwla_lds_barrier();                                        // every wave is done reading V
        // lane holds Z[a = ti*16 + 4*lg + v][d = tj*16 + li]: one 128-bit store into ZT[d][a..a+3]
#pragma unroll
        for (int s = 0; s < RQ_MAXT; ++s) {
            if (s < my_tiles) {
                const int tau = wave + s * RQ_WAVES;
                const int ti = dt2.div(tau), tj = tau - ti * tiles2;
                *reinterpret_cast<float4*>(reg + (tj * 16 + li) * sh.ldzt + ti * 16 + 4 * lg) =
                    make_float4(acc[s][0], acc[s][1], acc[s][2], acc[s][3]);
                acc[s] = v4f{0.f, 0.f, 0.f, 0.f};
            }
        }
        bwla_lds_barrier();                                        // ZT is published
        RQTRACE(4);
        // stage 2: Yt[d][c] = sum_a ZT[d][a] R1[a][c];   tile (ti over d, tj over c)
#pragma unroll
        for (int g = 0; g < RQ_MAXT / 2; ++g) {
            if (2 * g < my_tiles) {
                RQ_PAIR_SLOTS(g);
                const int tau0 = wave + s0 * RQ_WAVES, tau1 = wave + s1 * RQ_WAVES;
                const int ti0 = dt1.div(tau0), tj0 = tau0 - ti0 * tiles1;
                const int ti1 = dt1.div(tau1), tj1 = tau1 - ti1 * tiles1;
                const float* ap0 = reg + (ti0 * 16 + li) * sh.ldzt + 4 * lg;
                const float* bp0 = r1t + (tj0 * 16 + li) * sh.ld1t + 4 * lg;
                const float* ap1 = reg + (ti1 * 16 + li) * sh.ldzt + 4 * lg;
                const float* bp1 = r1t + (tj1 * 16 + li) * sh.ld1t + 4 * lg;
#pragma unroll 2
                for (int k = 0; k < sh.n1p; k += 16) {
                    acc[2 * g] = mfma16(ap0 + k, bp0 + k, acc[2 * g]);
                    acc[2 * g + 1] = mfma16(ap1 + k, bp1 + k, acc[2 * g + 1]);
                }
            }
        }
    } else {
        // ---------------- factors streamed in 16-index chunks: RQ_RING chunks in flight in
        // registers, two chunk buffers in LDS, one LDS-only barrier per chunk
        float* cb = fac;
        const int cbs = sh.nmaxp * RQ_CLD;                         // floats per chunk buffer
        for (int idx = tid; idx < 2 * cbs; idx += RQ_THREADS) cb[idx] = 0.0f;    // padded rows stay zero
        __syncthreads();
        for (int stage = 0; stage < 2; ++stage) {
            const float* R = stage == 0 ? R2 : R1;
            const int n = stage == 0 ? n2 : n1;
            const int nchunks = (n + RQ_CK - 1) / RQ_CK;
            const int lda = stage == 0 ? sh.ldv : sh.ldzt;
            const int tdiv = stage == 0 ? tiles2 : tiles1;         // tiles along the operand-B rows
            const FastDiv dtd = stage == 0 ? dt2 : dt1;
            const ChunkSlots cs = chunk_slots(n);
            ChunkRegs ring[RQ_RING];
#pragma unroll
            for (int d = 0; d < RQ_RING; ++d) ring[d] = chunk_fetch(R, n, d, cs);
            chunk_store(cb, cs, ring[0]);
            bwla_lds_barrier();                                    // chunk 0 (and V / ZT) published
            for (int c0 = 0; c0 < nchunks; c0 += RQ_RING) {
#pragma unroll
                for (int d = 0; d < RQ_RING; ++d) {
                    const int c = c0 + d;
                    if (c < nchunks) {
                        const float* cur = cb + (c & 1) * cbs;
#pragma unroll
                        for (int g = 0; g < RQ_MAXT / 2; ++g) {
                            if (2 * g < my_tiles) {
                                RQ_PAIR_SLOTS(g);
                                const int tau0 = wave + s0 * RQ_WAVES, tau1 = wave + s1 * RQ_WAVES;
                                const int ti0 = dtd.div(tau0), tj0 = tau0 - ti0 * tdiv;
                                const int ti1 = dtd.div(tau1), tj1 = tau1 - ti1 * tdiv;
                                acc[2 * g] = mfma16(reg + (ti0 * 16 + li) * lda + c * RQ_CK + 4 * lg,
                                                    cur + (tj0 * 16 + li) * RQ_CLD + 4 * lg, acc[2 * g]);
                                acc[2 * g + 1] = mfma16(reg + (ti1 * 16 + li) * lda + c * RQ_CK + 4 * lg,
                                                        cur + (tj1 * 16 + li) * RQ_CLD + 4 * lg, acc[2 * g + 1]);
                            }
                        }
                    }
                    // chunk c+1 (requested RQ_RING - 1 chunks ago) into the other buffer, whose last
                    // readers passed the previous barrier; then refill this ring slot
                    chunk_store(cb + ((c + 1) & 1) * cbs, cs, ring[(d + 1) % RQ_RING]);
                    ring[d] = chunk_fetch(R, n, c + RQ_RING, cs);
                    bwla_lds_barrier();
                }
            }
            if (stage == 0) RQTRACE(3); else RQTRACE(9);
            if (stage == 0) {
                // lane holds Z[a = ti*16 + 4*lg + v][d = tj*16 + li] -> ZT[d][a..a+3]; V is dead
                // (every wave passed the last barrier of the loop)
#pragma unroll
                for (int s = 0; s < RQ_MAXT; ++s) {
                    if (s < my_tiles) {
                        const int tau = wave + s * RQ_WAVES;
                        const int ti = dt2.div(tau), tj = tau - ti * tiles2;
                        *reinterpret_cast<float4*>(reg + (tj * 16 + li) * sh.ldzt + ti * 16 + 4 * lg) =
                            make_float4(acc[s][0], acc[s][1], acc[s][2], acc[s][3]);
                        acc[s] = v4f{0.f, 0.f, 0.f, 0.f};
                    }
                }
            }
        }
    }

    RQTRACE(5);
    // ================= per-token max magnitude
    float mx = 0.0f, mn = 0.0f;
#pragma unroll
    for (int s = 0; s < RQ_MAXT; ++s)
        if (s < my_tiles) {
#pragma unroll
            for (int v = 0; v < 4; ++v) { mx = fmaxf(mx, acc[s][v]); mn = fminf(mn, acc[s][v]); }
        }
    mx = bwla_wave_max(mx);
    mn = -bwla_wave_max(-mn);
    if (lane == 0) { red[wave] = mx; red[32 + wave] = mn; }
    bwla_lds_barrier();                                // also: every wave is done reading ZT
    float hi = red[0], lo = red[32];
#pragma unroll
    for (int w = 1; w < RQ_WAVES; ++w) { hi = fmaxf(hi, red[w]); lo = fminf(lo, red[32 + w]); }
    const QuantPlan qp = quant_plan(hi, lo, qmax, asym);
    RQTRACE(6);

    // ================= quantize from registers into an LDS byte image of the token's codes:
    // lane holds Yt[d = ti*16 + 4*lg + v][c = tj*16 + li], i.e. four consecutive d of one c
    int8_t* codes = reinterpret_cast<int8_t*>(reg);
    int lsum = 0;
#pragma unroll
    for (int s = 0; s < RQ_MAXT; ++s) {
        if (s < my_tiles) {
            const int tau = wave + s * RQ_WAVES;
            const int ti = dt1.div(tau), tj = tau - ti * tiles1;
            const int c = tj * 16 + li, d0 = ti * 16 + 4 * lg;
            int code[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) code[v] = quant_code(acc[s][v], qp);
            if (c < n1) {
                if ((n2 & 3) == 0) {
                    if (d0 < n2) {
                        *reinterpret_cast<int*>(codes + c * n2 + d0) = (code[0] & 0xff) | ((code[1] & 0xff) << 8) |
                                                                        ((code[2] & 0xff) << 16) | (code[3] << 24);
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
    // coalesced 16-byte stores of the code row (K % 16 == 0)
    {
        const uint4* src = reinterpret_cast<const uint4*>(codes);
        uint4* dst = reinterpret_cast<uint4*>(q + t * K);
        const int n16 = (int)(K >> 4);
        for (int idx = tid; idx < n16; idx += RQ_THREADS) dst[idx] = src[idx];
    }
    RQTRACE(7);
    if (tid == 0) {
        int tot = 0;
#pragma unroll
        for (int w = 0; w < RQ_WAVES; ++w) tot += redi[w];
        qsum[t] = tot;
        const float sc = quant_scale(hi, lo, qmax, asym);
        scale[t] = sc;
        quant_extras(tmode, tp, t, asym, shift, qp, sc, tot, K);
    }
    RQTRACE(8);
    RQTRACE_FLUSH;
#undef RQ_PAIR_SLOTS
}

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
// the workgroup has any (and they are not somebody else's, see LOCAL), carry their share of the R1
// terms and end once it is in LDS.
// LOCAL (fused single-launch decode): the codes, the per-strip maxima and the per-strip code sums
// stay in LDS for the rest of the workgroup (see r3_local); only if `store_out` are they also
// written out.  The body then has exactly R3_LOCAL_BARRIERS barriers, which the workgroup's other
// wavefronts match.
constexpr int R3_FILLR = 12;         // 16-byte pieces of the R1 terms a thread keeps in flight
constexpr int R3_LOCAL_BARRIERS = 4;
template <int ATM, bool LOOP, bool LOCAL = false>
__device__ __forceinline__ void rotate3_token(char* lds, const uint16_t* __restrict__ X, int64_t t_first,
                                              int64_t t_stride, int64_t M, int64_t K, int n1, int n2,
                                              const uint16_t* __restrict__ R1p,
                                              const uint16_t* __restrict__ R2p, int8_t* __restrict__ q,
                                              float* __restrict__ scale, int32_t* __restrict__ qsum,
                                              bool store_out = true, float* __restrict__ tmode = nullptr,
                                              int tp = 0, float qmax = 31.0f, bool asym = false,
                                              bool shift = false) {
    const R3Shape sh = r3_shape(n1, n2);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);         // = strip
    // the workgroup may have more wavefronts than strips (the projection workgroups of the same
    // launch use them): those only help to fetch the R1 terms, or leave at once
    // (more than 8 tiles along n1 never fit LDS whole: no code for them)
    const bool early = !LOOP && ATM <= 8 && sh.resident;
    const bool helper = wave >= sh.strips;
    if (helper && !(early && !LOCAL)) return;
    const int nthreads = 64 * sh.strips;
    const int nfill = (early && !LOCAL) ? (int)blockDim.x : nthreads;
    RQTRACE_DECL;
    RQTRACE(0);
    const int li = lane & 15, lg = lane >> 4;
    const int n1p16 = sh.at * 16, n1p32 = sh.ch2 * 32, n2p32 = sh.k1 * 32;
    char* vt = lds;                                                    // token rows, later the code image
    char* cb = lds + sh.r0bytes;                                       // chunk buffers
    float* red = reinterpret_cast<float*>(lds + sh.r0bytes + (size_t)(sh.alias ? 1 : sh.nbuf) * sh.cbytes);

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
        for (int base = 0; base < total; base += 8 * nthreads) {
            v4i tmp[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int g = base + e * nthreads + tid;
                const int gc = g < total ? g : total - 1;
                const int ch = gc / crow_items;
                tmp[e] = *chunk_src(ch, gc - ch * crow_items);
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int g = base + e * nthreads + tid;
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
    int64_t t = t_first;
#pragma nounroll
    do {
    // In a loop, lane-derived values are recomputed per token from an opaque copy of the thread
    // index: otherwise every address of the body is hoisted out of the loop and kept in registers.
    int tid_opaque = threadIdx.x;
    if constexpr (LOOP) asm volatile("" : "+v"(tid_opaque));
    const int tid = tid_opaque, lane = tid & 63, li = lane & 15, lg = lane >> 4;
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
    RQTRACE(1);
    // (one token per workgroup: a barrier that leaves the loads of later stages in flight)
    if constexpr (LOOP) __syncthreads(); else bwla_lds_barrier();
    RQTRACE(2);

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
    RQTRACE(3);
    if (early) {
        rp_store();
        bwla_lds_barrier();
        RQTRACE(7);
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

    RQTRACE(4);
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
    __syncthreads();                                   // also: every wave is done with the token rows
    float hi = red[0];
    for (int w = 1; w < sh.strips; ++w) hi = fmaxf(hi, red[w]);
    float lo = -hi;
    if (asym) {
        lo = red[32];
        for (int w = 1; w < sh.strips; ++w) lo = fminf(lo, red[32 + w]);
    }
    const QuantPlan qp = quant_plan(hi, lo, qmax, asym);
    RQTRACE(5);

    // ---- quantize: lane holds Yt[d = 16*strip + 4*lg + v][c = 16*tc + li], four consecutive d of one c
    int8_t* codes = reinterpret_cast<int8_t*>(vt);
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
                        *reinterpret_cast<int*>(codes + c * n2 + d0) = (code[0] & 0xff) | ((code[1] & 0xff) << 8) |
                                                                        ((code[2] & 0xff) << 16) | (code[3] << 24);
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
    __syncthreads();
    if (!LOCAL || store_out) {
        {
            const uint4* src = reinterpret_cast<const uint4*>(codes);
            uint4* dst = reinterpret_cast<uint4*>(q + t * K);
            const int n16 = (int)(K >> 4);
            for (int idx = tid; idx < n16; idx += nthreads) dst[idx] = src[idx];
        }
        if (tid == 0) {
            int tot = 0;
            for (int w = 0; w < sh.strips; ++w) tot += redi[w];
            qsum[t] = tot;
            const float sc = quant_scale(hi, lo, qmax, asym);
            scale[t] = sc;
            quant_extras(tmode, tp, t, asym, shift, qp, sc, tot, K);
        }
    }
    RQTRACE(6);
    if constexpr (LOOP) __syncthreads();               // the code image and the reduction words are free again
    t += t_stride;
    } while (LOOP && t < M);
    RQTRACE_FLUSH;
}

// ================================================================== few tokens, factors too large for LDS
// One workgroup per token has to stream all of the R1 terms through one CU, chunk by chunk, with
// a memory round trip per chunk.  With only a few tokens most of the chip is idle meanwhile, so
// the rotation of a token is split over G workgroups: each does stage 1 for the whole token (it
// is cheap) and stage 2 for RS_CT tiles along n1, for which its slice of the R1 terms fits LDS
// whole and is requested at once.  The token's maximum is then not known inside the launch:
// the workgroups write the rotated values (fp32, in k order) and their own maxima to scratch,
// and a second, small launch quantizes.  Same products in the same order as rotate3_token, so
// the codes are the same.
constexpr int RS_CT = 2;             // 16-row tiles along n1 per workgroup (stage 2)
constexpr int RS_FILL = 6;           // 16-byte pieces of the R1 slice a thread keeps in flight

struct RsShape {
    int G, spitch;                   // workgroups per token; bytes of one R1 row in LDS
    size_t lds_bytes;
    bool ok;
};
__host__ __device__ inline RsShape rs_shape(const R3Shape& s3) {
    RsShape r;
    r.G = (s3.at + RS_CT - 1) / RS_CT;
    r.spitch = s3.ch2 * 64 + 16;
    r.lds_bytes = (size_t)s3.vbytes + (size_t)3 * RS_CT * 16 * r.spitch + 256;
    // one wavefront per strip in a 512-thread workgroup; the slice in RS_FILL pieces per thread
    r.ok = s3.at <= R3_MAXA && s3.k1 <= R3_MAXK1 && s3.strips <= 8 && r.lds_bytes <= RQ_LDS_LIMIT &&
           3 * RS_CT * 16 * s3.ch2 * 4 <= RS_FILL * 64 * s3.strips;
    return r;
}

template <int ATM>
__device__ __forceinline__ void rotate_split_block(char* lds, const uint16_t* __restrict__ X, int64_t t, int j,
                                                   int64_t K, int n1, int n2, const uint16_t* __restrict__ R1p,
                                                   const uint16_t* __restrict__ R2p, float* __restrict__ xs,
                                                   float* __restrict__ pmax, int32_t* __restrict__ qsum) {
    const R3Shape sh = r3_shape(n1, n2);
    const RsShape rs = rs_shape(sh);
    const int tid = threadIdx.x, lane = tid & 63, li = lane & 15, lg = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);         // = strip
    if (wave >= sh.strips) return;
    const int nthreads = 64 * sh.strips;
    const int n1p16 = sh.at * 16, n1p32 = sh.ch2 * 32, n2p32 = sh.k1 * 32;
    char* vt = lds;                                                    // token rows
    char* sl = lds + sh.vbytes;                                        // R1 slice [term][c in slice][a]
    float* red = reinterpret_cast<float*>(sl + 3 * RS_CT * 16 * rs.spitch);
    const int c_base = j * RS_CT * 16;                                 // first row c of the slice

    // R2 terms of my strip
    v4i bfr[R3_MAXK1][3];
#pragma unroll
    for (int kb = 0; kb < R3_MAXK1; ++kb)
#pragma unroll
        for (int p = 0; p < 3; ++p) {
            bfr[kb][p] = v4i{0, 0, 0, 0};
            if (kb < sh.k1)
                bfr[kb][p] = *reinterpret_cast<const v4i*>(R2p + ((int64_t)(p * sh.strips * 16 + wave * 16 + li)) * n2p32 +
                                                           kb * 32 + 8 * lg);
        }
    // the slice of the R1 terms: rows c_base .. c_base + 31 of each term (rows past the padded n1
    // repeat the last one and are never used), all requested now and stored after stage 1
    const int row_items = sh.ch2 * 4, slice_items = 3 * RS_CT * 16 * row_items;
    const FastDiv dri(row_items);
    v4i rp[RS_FILL];
    auto slice_issue = [&]() {
#pragma unroll
        for (int e = 0; e < RS_FILL; ++e) {
            const int g = tid + e * nthreads;
            const int gc = g < slice_items ? g : slice_items - 1;
            const int row = dri.div(gc), piece = gc - row * row_items;  // row = term * 32 + c in slice
            const int term = row / (RS_CT * 16), cs = row - term * (RS_CT * 16);
            const int c = c_base + cs < n1p16 ? c_base + cs : n1p16 - 1;
            rp[e] = *reinterpret_cast<const v4i*>(R1p + ((int64_t)(term * n1p16 + c)) * n1p32 + piece * 8);
        }
    };
    // token rows into LDS (bf16 as stored; zero padding), eight loads in flight per thread
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
                if (base == 0) slice_issue();          // behind the first token loads
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int it = base + e * nthreads + tid;
                    if (it < items) {
                        const int a = dpr.div(it), b0 = (it - a * per_row) << 3;
                        *reinterpret_cast<v4i*>(vt + a * sh.vpitch + b0 * 2) = tmp[e];
                    }
                }
            }
        } else {
            slice_issue();
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
    bwla_lds_barrier();

    // ---- stage 1 (as in rotate3_token): Z[a, d] for the whole token, my strip of d
    v4f z[ATM];
#pragma unroll
    for (int ta = 0; ta < ATM; ++ta) z[ta] = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int g = 0; g < ATM / 2; ++g) {
        if (2 * g < sh.at) {
            const int t0 = 2 * g, t1 = 2 * g + 1 < sh.at ? 2 * g + 1 : 2 * g;
            const char* a0p = vt + (t0 * 16 + li) * sh.vpitch + lg * 16;
            const char* a1p = vt + (t1 * 16 + li) * sh.vpitch + lg * 16;
#pragma unroll
            for (int kb = 0; kb < R3_MAXK1; ++kb) {
                if (kb < sh.k1) {
                    const v8bf a0 = __builtin_bit_cast(v8bf, *reinterpret_cast<const v4i*>(a0p + kb * 64));
                    const v8bf a1 = __builtin_bit_cast(v8bf, *reinterpret_cast<const v4i*>(a1p + kb * 64));
#pragma unroll
                    for (int p = 2; p >= 0; --p) {
                        const v8bf b = __builtin_bit_cast(v8bf, bfr[kb][p]);
                        z[2 * g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, b, z[2 * g], 0, 0, 0);
                        z[2 * g + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, b, z[2 * g + 1], 0, 0, 0);
                    }
                }
            }
        }
    }
    if ((sh.at & 1) != 0) {
#pragma unroll
        for (int ta = 1; ta < ATM; ta += 2)
            if (ta == sh.at) z[ta] = v4f{0.f, 0.f, 0.f, 0.f};
    }

    // ---- the slice into LDS
#pragma unroll
    for (int e = 0; e < RS_FILL; ++e) {
        const int g = tid + e * nthreads;
        if (g < slice_items) {
            const int row = dri.div(g), piece = g - row * row_items;
            *reinterpret_cast<v4i*>(sl + row * rs.spitch + piece * 16) = rp[e];
        }
    }
    bwla_lds_barrier();

    // ---- stage 2 for tiles c0 = RS_CT * j, c0 + 1 (products and their order as in rotate3_token)
    v4f y0 = v4f{0.f, 0.f, 0.f, 0.f}, y1 = v4f{0.f, 0.f, 0.f, 0.f};
    const bool two = RS_CT * j + 1 < sh.at;            // an odd last tile is done twice; the copy is dropped
    const char* s0 = sl + li * rs.spitch + lg * 16;
    const char* s1 = sl + ((two ? 16 : 0) + li) * rs.spitch + lg * 16;
#pragma unroll
    for (int ch = 0; ch < ATM / 2; ++ch) {
        if (ch < sh.ch2) {
            const float f[8] = {z[2 * ch][0], z[2 * ch][1], z[2 * ch][2], z[2 * ch][3],
                                z[2 * ch + 1][0], z[2 * ch + 1][1], z[2 * ch + 1][2], z[2 * ch + 1][3]};
            v8bf a1, a2, a3;
            r3_split3(f, a1, a2, a3);
            v8bf b0[3], b1[3];
#pragma unroll
            for (int p = 0; p < 3; ++p) {
                b0[p] = __builtin_bit_cast(v8bf, *reinterpret_cast<const v4i*>(s0 + p * RS_CT * 16 * rs.spitch + ch * 64));
                b1[p] = __builtin_bit_cast(v8bf, *reinterpret_cast<const v4i*>(s1 + p * RS_CT * 16 * rs.spitch + ch * 64));
            }
            y0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a3, b0[0], y0, 0, 0, 0);
            y1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a3, b1[0], y1, 0, 0, 0);
            y0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, b0[2], y0, 0, 0, 0);
            y1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, b1[2], y1, 0, 0, 0);
            y0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a2, b0[1], y0, 0, 0, 0);
            y1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a2, b1[1], y1, 0, 0, 0);
            y0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a2, b0[0], y0, 0, 0, 0);
            y1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a2, b1[0], y1, 0, 0, 0);
            y0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, b0[1], y0, 0, 0, 0);
            y1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, b1[1], y1, 0, 0, 0);
            y0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, b0[0], y0, 0, 0, 0);
            y1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, b1[0], y1, 0, 0, 0);
        }
    }

    // ---- rotated values out (lane: d = 16*strip + 4*lg + v, c = 16*tile + li), and my extremes
    float mx = 0.0f, mn = 0.0f;
    const int d0 = wave * 16 + 4 * lg;
    float* xt = xs + t * K;
#pragma unroll
    for (int u = 0; u < RS_CT; ++u) {
        const v4f y = u == 0 ? y0 : y1;
        const int c = (RS_CT * j + u) * 16 + li;
        if ((u == 0 || two) && c < n1) {
#pragma unroll
            for (int v = 0; v < 4; ++v)
                if (d0 + v < n2) {
                    xt[(int64_t)c * n2 + d0 + v] = y[v];
                    mx = fmaxf(mx, y[v]);
                    mn = fminf(mn, y[v]);
                }
        }
    }
    mx = bwla_wave_max(mx);
    mn = -bwla_wave_max(-mn);
    if (lane == 0) { red[wave] = mx; red[32 + wave] = mn; }
    bwla_lds_barrier();
    if (tid == 0) {
        float hi = red[0], lo = red[32];
        for (int w = 1; w < sh.strips; ++w) { hi = fmaxf(hi, red[w]); lo = fminf(lo, red[32 + w]); }
        pmax[(t * rs.G + j) * 2] = hi;                 // largest and smallest value of my slice (0 included)
        pmax[(t * rs.G + j) * 2 + 1] = lo;
        if (j == 0) qsum[t] = 0;                       // the quantizing launch adds its sums up here
    }
}

// second launch of the split rotation: RS_QB workgroups per token quantize the rotated values, each
// its share of k, every load in flight at once; the code sum is added up in qsum[t], which the
// first launch has set to zero (integer adds: the order does not matter)
constexpr int RS_QB = 8;
constexpr int RS_QI = 4;             // float4 per thread: K <= RS_QB * 512 * RS_QI * 4
__global__ __launch_bounds__(512) void quantize_rows_kernel(const float* __restrict__ xs, const float* __restrict__ pmax,
                                                            int G, int64_t K, int8_t* __restrict__ q,
                                                            float* __restrict__ scale, int32_t* __restrict__ qsum,
                                                            float qmax, int asym, float* __restrict__ tmode, int tp,
                                                            float* __restrict__ zcs) {
    __shared__ int redi[8];
    const int64_t t = blockIdx.x / RS_QB;
    const int part = (int)(blockIdx.x - t * RS_QB);
    const int tid = threadIdx.x;
    const int n4 = (int)(K >> 2);
    const float4* src = reinterpret_cast<const float4*>(xs + t * K);
    float4 x[RS_QI];
#pragma unroll
    for (int e = 0; e < RS_QI; ++e) {
        const int i = (e * RS_QB + part) * 512 + tid;
        x[e] = src[i < n4 ? i : n4 - 1];
    }
    float hi = pmax[t * G * 2], lo = pmax[t * G * 2 + 1];
    for (int j = 1; j < G; ++j) { hi = fmaxf(hi, pmax[(t * G + j) * 2]); lo = fminf(lo, pmax[(t * G + j) * 2 + 1]); }
    const QuantPlan qp = quant_plan(hi, lo, qmax, asym != 0);
    int* dst = reinterpret_cast<int*>(q + t * K);
    int lsum = 0;
#pragma unroll
    for (int e = 0; e < RS_QI; ++e) {
        const int i = (e * RS_QB + part) * 512 + tid;
        if (i < n4) {
            const float f[4] = {x[e].x, x[e].y, x[e].z, x[e].w};
            int code[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                code[v] = quant_code(f[v], qp);
                lsum += code[v];
            }
            dst[i] = (code[0] & 0xff) | ((code[1] & 0xff) << 8) | ((code[2] & 0xff) << 16) | (code[3] << 24);
        }
    }
    lsum = bwla_wave_sum_i32(lsum);
    if ((tid & 63) == 0) redi[tid >> 6] = lsum;
    __syncthreads();
    if (tid == 0) {
        int tot = 0;
        for (int w = 0; w < 8; ++w) tot += redi[w];
        atomicAdd(qsum + t, tot);
        if (part == 0) {
            const float sc = quant_scale(hi, lo, qmax, asym != 0);
            scale[t] = sc;
            zcs[t] = qp.zc;
            if (asym && tmode) tmode[t * tp] = tmode[t * tp + 1] = -(sc * qp.zc);
        }
    }
}

// layers with row shifts, after the split rotation (the code sum is complete only now):
// T[t, last] = scale_t * sum_k (q - z) = scale_t * (qsum_t - K zc_t)
__global__ void shift_column_kernel(const float* __restrict__ scale, const int32_t* __restrict__ qsum,
                                    const float* __restrict__ zcs, int64_t M, int64_t K,
                                    float* __restrict__ tshift, int tp) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < M) tshift[t * tp] = scale[t] * ((float)qsum[t] - (float)K * zcs[t]);
}

// where rotate3_token<.., LOCAL> leaves its results (resident shapes only)
__device__ __forceinline__ FusedLocal r3_local(const char* lds, const R3Shape& sh) {
    // words [0, 16) largest values, [16, 32) code sums, [32, 48) smallest values (of the 64 words
    // behind the chunk buffers)
    const float* red = reinterpret_cast<const float*>(lds + sh.r0bytes + (size_t)sh.nbuf * sh.cbytes);
    return FusedLocal{lds, red, reinterpret_cast<const int*>(red) + 16, sh.strips};
}

// ================================================================== PSP projection T = X U
template <bool BF16>
__device__ __forceinline__ void psp_block(char* smem, const void* __restrict__ X, int64_t M, int64_t K, int r,
                                          const __half* __restrict__ U, float* __restrict__ T,
                                          int* __restrict__ counters, float* __restrict__ partials, int S, int tt,
                                          int s, int tp) {
    __shared__ int is_last;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nw = (int)(blockDim.x >> 6);             // the eight 64-column parts of a slice are dealt to nw waves
    const int li = lane & 15, lg = lane >> 4;
    const int JT = (r + 15) >> 4, rp = JT * 16;
    const int64_t kbase = (int64_t)s * PP_SLICE;

    // wave w takes columns [64w, 64w+64) of the slice in 4 groups of 16: lane (li, lg) owns
    // k = 16*g + 4*lg + e, e = 0..3 -- of token li as MFMA operand A, of column jt*16 + li of U as
    // operand B (8 contiguous bytes of the transposed U).  All loads are issued before the first use.
    int64_t trow = (int64_t)tt * 16 + li;
    if (trow > M - 1) trow = M - 1;                    // padded token rows are never stored
    v4f acc[PP_MAXJT];
#pragma unroll
    for (int jt = 0; jt < PP_MAXJT; ++jt) acc[jt] = v4f{0.f, 0.f, 0.f, 0.f};
    for (int part = wave; part < 8; part += nw) {
    float x[4][4];
    uint2 u[4][PP_MAXJT];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const int64_t kx = kbase + part * 64 + g * 16 + 4 * lg;
        const bool in = kx < K;
        const int64_t kc = in ? kx : K - 4;            // keep the address valid, zero the value
        if (BF16) {
            const uint2 raw = *reinterpret_cast<const uint2*>(reinterpret_cast<const uint16_t*>(X) + trow * K + kc);
            x[g][0] = __uint_as_float(raw.x << 16); x[g][1] = __uint_as_float(raw.x & 0xffff0000u);
            x[g][2] = __uint_as_float(raw.y << 16); x[g][3] = __uint_as_float(raw.y & 0xffff0000u);
        } else {
            const float4 raw = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(X) + trow * K + kc);
            x[g][0] = raw.x; x[g][1] = raw.y; x[g][2] = raw.z; x[g][3] = raw.w;
        }
        if (!in) x[g][0] = x[g][1] = x[g][2] = x[g][3] = 0.0f;
#pragma unroll
        for (int jt = 0; jt < PP_MAXJT; ++jt)
            if (jt < JT) u[g][jt] = *reinterpret_cast<const uint2*>(U + (int64_t)(jt * 16 + li) * K + kc);
    }

#pragma unroll
    for (int g = 0; g < 4; ++g) {
#pragma unroll
        for (int jt = 0; jt < PP_MAXJT; ++jt) {
            if (jt < JT) {
                const __half2 h01 = *reinterpret_cast<const __half2*>(&u[g][jt].x);
                const __half2 h23 = *reinterpret_cast<const __half2*>(&u[g][jt].y);
                const float2 f01 = __half22float2(h01), f23 = __half22float2(h23);
                acc[jt] = __builtin_amdgcn_mfma_f32_16x16x4f32(x[g][0], f01.x, acc[jt], 0, 0, 0);
                acc[jt] = __builtin_amdgcn_mfma_f32_16x16x4f32(x[g][1], f01.y, acc[jt], 0, 0, 0);
                acc[jt] = __builtin_amdgcn_mfma_f32_16x16x4f32(x[g][2], f23.x, acc[jt], 0, 0, 0);
                acc[jt] = __builtin_amdgcn_mfma_f32_16x16x4f32(x[g][3], f23.y, acc[jt], 0, 0, 0);
            }
        }
    }
    }
    v4f* red = reinterpret_cast<v4f*>(smem);           // [wave][jt][lane]
#pragma unroll
    for (int jt = 0; jt < PP_MAXJT; ++jt)
        if (jt < JT) red[(wave * JT + jt) * 64 + lane] = acc[jt];
    __syncthreads();
    // waves share the column tiles; lane holds tokens 4*lg + v, column jt*16 + li
    for (int jt = wave; jt < JT; jt += nw) {
        v4f sum = red[jt * 64 + lane];
        for (int w = 1; w < nw; ++w) sum += red[(w * JT + jt) * 64 + lane];
        const int col = jt * 16 + li;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int row = 4 * lg + v;
            const int64_t tok = (int64_t)tt * 16 + row;
            if (S == 1) {
                if (tok < M && col < r) T[tok * tp + col] = sum[v];
            } else {
                bwla_store_agent(&partials[(((int64_t)tt * S + s) * 16 + row) * rp + col], sum[v]);
            }
        }
    }
    if (S == 1) return;

    if (!bwla_partials_arrive(&counters[tt], S, &is_last)) return;
    // last workgroup of this token tile: add the S partial tiles in slice order
    const int rows = M - (int64_t)tt * 16 < 16 ? (int)(M - (int64_t)tt * 16) : 16;
    for (int idx = tid; idx < rows * rp; idx += (int)blockDim.x) {
        const int row = idx / rp, col = idx - row * rp;
        const int64_t tok = (int64_t)tt * 16 + row;
        if (col < r) {
            // batches of sixteen loads in flight; slices past S re-read the last one and add zero
            float sum = 0.0f;
            for (int ss = 0; ss < S; ss += 16) {
                float v[16];
#pragma unroll
                for (int u = 0; u < 16; ++u) {
                    const int sc = ss + u < S ? ss + u : S - 1;
                    v[u] = bwla_load_agent(&partials[(((int64_t)tt * S + sc) * 16 + row) * rp + col]);
                }
#pragma unroll
                for (int u = 0; u < 16; ++u) sum += ss + u < S ? v[u] : 0.0f;
            }
            T[tok * tp + col] = sum;
        }
    }
    if (tid == 0) counters[tt] = 0;                    // leave the scratch as it was found
}

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
    const uint16_t* R1p; const uint16_t* R2p;          // bf16 term planes of the factors
};

template <bool BF16>
__global__ __launch_bounds__(RQ_THREADS) void rotate_quant_kernel(RqArgs a) {
    extern __shared__ __align__(16) float lds[];
    if ((int64_t)blockIdx.x < a.rot_blocks) {
        rotate_token<BF16>(lds, a.X, blockIdx.x, a.K, a.n1, a.n2, a.R1, a.R2, a.q, a.scale, a.qsum, a.tmode, a.tp, a.qmax,
                           a.asym != 0, a.shift != 0);
    } else {
        const int pb = (int)(blockIdx.x - a.rot_blocks);
        psp_block<BF16>(reinterpret_cast<char*>(lds), a.X, a.M, a.K, a.r, a.U, a.T, a.counters, a.partials, a.S,
                        pb / a.S, pb % a.S, a.tp);
    }
}

// rotation on bf16 MFMA (bf16 activations): 64 threads per 16-column strip of n2
template <int ATM, int THREADS, bool LOOP>
__global__ __launch_bounds__(THREADS) void rotate_quant3_kernel(RqArgs a) {
    extern __shared__ __align__(16) float lds[];
    if ((int64_t)blockIdx.x < a.rot_blocks) {
        rotate3_token<ATM, LOOP>(reinterpret_cast<char*>(lds), reinterpret_cast<const uint16_t*>(a.X), blockIdx.x,
                           a.rot_blocks, a.M, a.K, a.n1, a.n2, a.R1p, a.R2p, a.q, a.scale, a.qsum, true, a.tmode,
                           a.tp, a.qmax, a.asym != 0, a.shift != 0);
    } else {
        const int pb = (int)(blockIdx.x - a.rot_blocks);
        psp_block<true>(reinterpret_cast<char*>(lds), a.X, a.M, a.K, a.r, a.U, a.T, a.counters, a.partials, a.S,
                        pb / a.S, pb % a.S, a.tp);
    }
}

// split rotation: workgroup b < rot_blocks does slice b % G of token b / G
__global__ __launch_bounds__(512) void rotate_split_kernel(RqArgs a) {
    extern __shared__ __align__(16) float lds[];
    if ((int64_t)blockIdx.x < a.rot_blocks) {
        const int G = rs_shape(r3_shape(a.n1, a.n2)).G;
        const int64_t t = blockIdx.x / G;
        rotate_split_block<R3_MAXA>(reinterpret_cast<char*>(lds), reinterpret_cast<const uint16_t*>(a.X), t,
                                    (int)(blockIdx.x - t * G), a.K, a.n1, a.n2, a.R1p, a.R2p, a.xs, a.pmax, a.qsum);
    } else {
        const int pb = (int)(blockIdx.x - a.rot_blocks);
        psp_block<true>(reinterpret_cast<char*>(lds), a.X, a.M, a.K, a.r, a.U, a.T, a.counters, a.partials, a.S,
                        pb / a.S, pb % a.S, a.tp);
    }
}

template <int ATM, int THREADS, bool LOOP>
hipError_t launch_rotate3_v(const RqArgs& a, int64_t blocks, int threads, size_t lds, hipStream_t st) {
    static bwla_lds_attr attr;
    hipError_t e = attr.ensure((const void*)rotate_quant3_kernel<ATM, THREADS, LOOP>, lds);
    if (e != hipSuccess) return e;
    rotate_quant3_kernel<ATM, THREADS, LOOP><<<dim3((unsigned)blocks), dim3((unsigned)threads), lds, st>>>(a);
    return hipGetLastError();
}
// the looping variant only when a workgroup really has more than one token
template <int ATM, int THREADS>
hipError_t launch_rotate3(const RqArgs& a, int64_t blocks, int threads, size_t lds, hipStream_t st) {
    if (a.rot_blocks < a.M) return launch_rotate3_v<ATM, THREADS, true>(a, blocks, threads, lds, st);
    return launch_rotate3_v<ATM, THREADS, false>(a, blocks, threads, lds, st);
}

// ---------------------------------------------------------------------------------------------
// One launch for a whole decode layer with a single token and no low-rank part (r = 0).  Every
// workgroup is a workgroup of the activation-stationary GEMM that first rotates and quantizes the
// token itself: the rotation of one token is a few hundred kFLOP fed from L2, cheaper to repeat
// per workgroup than to hand its result from one workgroup to all the others through memory, and
// nothing crosses workgroups.  Wavefronts [0, strips) rotate while wavefronts
// [strips, strips + KS), the GEMM's compute wavefronts, already have their first weights in
// flight; then wavefront 0 goes on as the GEMM's epilogue wavefront and the other rotation
// wavefronts end.  The first workgroup also writes codes, scale and code sum out.
// (With r > 0 the projection T = x U would have to reach every workgroup inside the launch; the
// arrival counting and the wait that this takes cost more than the second launch saves.)
constexpr int FD_THREADS = 512;
#ifdef BWLA_TRACE
#define FDTRACE(slot) do { if ((threadIdx.x & 63) == 0 && (blockIdx.x & 3) == 0 && blockIdx.x < 256) bwla_trace_buf[((blockIdx.x >> 2) * 16 + 8 + (threadIdx.x >> 6)) * 40 + (slot)] = wall_clock64(); } while (0)
#else
#define FDTRACE(slot) do { } while (0)
#endif
template <int ATM, bool FAST>
__global__ __launch_bounds__(FD_THREADS) void decode_fused_kernel(RqArgs ra, BsArgs ba) {
    extern __shared__ __align__(16) float lds[];
    const R3Shape sh = r3_shape(ra.n1, ra.n2);
    char* rot = reinterpret_cast<char*>(lds);
    char* smem = rot + ((sh.lds_bytes + 255) & ~(size_t)255);
    const FusedLocal fl = r3_local(rot, sh);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int first = (int)blockIdx.x, stride = (int)gridDim.x;
    const int n_iter = (ba.row_tiles - first + stride - 1) / stride;
    if (wave < sh.strips) {
        FDTRACE(0);
        rotate3_token<ATM, false, true>(rot, reinterpret_cast<const uint16_t*>(ra.X), 0, 1, 1, ra.K, ra.n1, ra.n2,
                                        ra.R1p, ra.R2p, ra.q, ra.scale, ra.qsum, first == 0);
        FDTRACE(1);
        if (wave != 0) return;
        epilogue_wave<2, 1, 0, FAST, true>(ba, smem, first, stride, n_iter, ba.KS, lane, fl);
    } else {
        const int cw = wave - sh.strips;
        if (cw >= ba.KS) return;                                   // surplus wavefronts
        // r = 0: only the wavefront that fetches the output scales has a side piece
        if (cw == 0)
            compute_wave<BS_CPW, 2, 1, true, true>(ba, smem, first, stride, n_iter, cw, lane, fl, R3_LOCAL_BARRIERS);
        else
            compute_wave<BS_CPW, 2, 1, false, true>(ba, smem, first, stride, n_iter, cw, lane, fl, R3_LOCAL_BARRIERS);
    }
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

}  // namespace

#ifdef BWLA_TRACE
extern "C" int bwla_fd_trace_dump(long long* host, int n) {
    return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(bwla_trace_buf), (size_t)n * sizeof(long long));
}
extern "C" int bwla_rq_trace_dump(long long* host, int n) {
    return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(bwla_rq_trace_buf), (size_t)n * sizeof(long long));
}
#endif

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
    // The projection rides in the rotation launch while that launch stays within about two
    // workgroups per CU: its short workgroups then finish in the shadow of the rotation.
    const int64_t ride = M + ((M + 15) / 16) * ((K + PP_SLICE - 1) / PP_SLICE);
    if (M <= 16 || r <= 0 || ride <= 512) {
        p.token_tiles = (int)((M + 15) / 16);
        p.k_per_split = PP_SLICE;
        p.splits = r > 0 ? (int)((K + PP_SLICE - 1) / PP_SLICE) : 1;
        p.tile_rows = 16; p.tile_cols = rp; p.col_groups = 1;
        return p;
    }
    // many tokens: about three workgroups per CU, slices a multiple of 128 (4 wavefronts x 32)
    p.tile_rows = 64;
    p.tile_cols = bwla_psp_prefill_tile_cols(rp);
    p.col_groups = (rp + 63) / 64;
    p.token_tiles = (int)((M + 63) / 64);
    const int64_t units = (int64_t)p.token_tiles * p.col_groups;
    int64_t S = (768 + units - 1) / units;
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
    a.xs = nullptr; a.pmax = nullptr;
    // Few tokens: one launch holds rotation and projection workgroups (a second launch would
    // cost more than it saves).  Many tokens: the projection has a kernel of its own.
    const bool merged = ru > 0 && plan.tile_rows == 16;
    const int64_t pblocks = merged ? (int64_t)plan.token_tiles * plan.splits : 0;
    const size_t plds = merged ? pp_lds_bytes(ru) : 0;
    a.rot_blocks = M;
    hipError_t e;
    const R3Shape s3 = r3_shape(L->n1, L->n2);
    const size_t split_bytes = xdtype == BWLA_X_BF16 ? bwla_split_rotation_bytes(L, plan, M) : 0;
    if (split_bytes > 0 && dws != nullptr) {
        // few tokens, R1 too large for LDS: several workgroups per token, then a launch that quantizes
        const RsShape rs = rs_shape(s3);
        a.xs = (float*)((char*)dws + bwla_align256(bwla_psp_ws_bytes(plan, M, ru)));
        a.pmax = a.xs + M * L->K;
        float* zcs = a.pmax + 2 * M * rs.G;            // per token: what the stored codes have to lose
        a.rot_blocks = M * rs.G;
        const size_t pl3 = merged ? pp_lds_bytes(ru, 8) : 0;
        const size_t lds3 = pl3 > rs.lds_bytes ? pl3 : rs.lds_bytes;
        static bwla_lds_attr attr;
        e = attr.ensure((const void*)rotate_split_kernel, lds3);
        if (e != hipSuccess) return e;
        rotate_split_kernel<<<dim3((unsigned)(a.rot_blocks + pblocks)), dim3(512), lds3, st>>>(a);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        quantize_rows_kernel<<<dim3((unsigned)(M * RS_QB)), dim3(512), 0, st>>>(a.xs, a.pmax, rs.G, L->K, dq, dscale,
                                                                                 dqsum, a.qmax, a.asym, a.tmode,
                                                                                 a.tp, zcs);
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
        // resident factors and many tokens: as many workgroups as fit the chip at once, each
        // walking over its share of the tokens with the factors loaded once
        if (s3.resident && !merged) {
            int64_t per_cu = (int64_t)(RQ_LDS_LIMIT / lds3);
            const int64_t by_waves = 32 / (threads / 64);              // at most 32 wavefronts per CU
            if (per_cu > by_waves) per_cu = by_waves;
            if (per_cu < 1) per_cu = 1;
            const int64_t cap = per_cu * bwla_device_cus();
            if (M > cap) a.rot_blocks = cap;
        }
        if (s3.resident && a.rot_blocks == M && s3.strips < 8) threads = 512;
        // register budget: up to 8 wavefronts may use 256 VGPRs, 9 or 10 only 168
        const int64_t grid = a.rot_blocks + pblocks;
        if (s3.strips <= 8 && s3.at <= 4) e = launch_rotate3<4, 512>(a, grid, threads, lds3, st);
        else if (s3.strips <= 8 && s3.at <= 8) e = launch_rotate3<8, 512>(a, grid, threads, lds3, st);
        else if (s3.at <= 12) e = launch_rotate3<12, 640>(a, grid, threads, lds3, st);
        else e = launch_rotate3<16, 512>(a, grid, threads, lds3, st);
        if (e != hipSuccess) return e;
        if (ru > 0 && !merged) return bwla_launch_psp_prefill(L, dX, xdtype, M, dT, dws, plan, st);
        return hipSuccess;
    }
    const size_t lds = plds > sh.lds_bytes ? plds : sh.lds_bytes;
    if (xdtype == BWLA_X_BF16) {
        static bwla_lds_attr attr;
        e = attr.ensure((const void*)rotate_quant_kernel<true>, lds);
        if (e != hipSuccess) return e;
        rotate_quant_kernel<true><<<dim3((unsigned)(M + pblocks)), dim3(RQ_THREADS), lds, st>>>(a);
    } else {
        static bwla_lds_attr attr;
        e = attr.ensure((const void*)rotate_quant_kernel<false>, lds);
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
    if (!s3.ok || s3.resident || (L->n2 & 3) != 0 || L->K > (int64_t)RS_QB * 512 * RS_QI * 4) return 0;
    const RsShape rs = rs_shape(s3);
    if (!rs.ok) return 0;
    const bool merged = bwla_rank_u(L) > 0 && plan.tile_rows == 16;
    const int64_t pblocks = merged ? (int64_t)plan.token_tiles * plan.splits : 0;
    // every workgroup of the launch gets a CU of its own at once; with more tokens than that the
    // one-workgroup-per-token kernel keeps the chip busy anyway
    if (M * rs.G + pblocks > bwla_device_cus()) return 0;
    return (size_t)(M * L->K + 2 * M * rs.G + M) * sizeof(float);     // values, extremes, per-token code offset
}

// Single-launch decode layer.  *done = false (and nothing launched) when the shape is outside what
// the fused kernel takes: one bf16 token, r = 0, factors resident in LDS with at most 8 tiles
// along n1, rotation strips and GEMM compute wavefronts together within the 512-thread workgroup
// (K = 4096 with n2 = 64: 4 + 4), and LDS for both roles side by side.
hipError_t bwla_launch_decode_fused(const bwla_layer_t* L, const void* dX, int xdtype, int64_t M, int8_t* dq,
                                    float* dscale, int32_t* dqsum, float* dY, int32_t* dacc, hipStream_t st,
                                    bool* done) {
    *done = false;
    const R3Shape s3 = r3_shape(L->n1, L->n2);
    const int chunks = (int)bwla_chunks(L->K), row_tiles = (int)bwla_row_tiles(L->N);
    const int KS = (chunks + BS_CPW - 1) / BS_CPW;
    if (M != 1 || L->r != 0 || xdtype != BWLA_X_BF16 || !s3.ok || !s3.resident || s3.at > 8 || (L->K & 15) != 0)
        return hipSuccess;
    if (chunks < 2 || s3.strips + KS > FD_THREADS / 64 || !bs_fits(M, chunks, 0, 1)) return hipSuccess;
    const size_t lds = ((s3.lds_bytes + 255) & ~(size_t)255) + bs_lds_bytes(M, chunks, 0, 1);
    if (lds > 160 * 1024) return hipSuccess;
    const char* blob = (const char*)L->d_blob;
    RqArgs ra{};
    ra.X = dX; ra.M = M; ra.K = L->K; ra.n1 = L->n1; ra.n2 = L->n2; ra.r = 0;
    ra.R1p = (const uint16_t*)(blob + L->off_R1p); ra.R2p = (const uint16_t*)(blob + L->off_R2p);
    ra.q = dq; ra.scale = dscale; ra.qsum = dqsum;
    BsArgs ba{(const uint4*)(blob + L->off_bits), chunks, row_tiles, dq, (int)M, (int)L->K, dscale, dqsum,
              (const __half*)(blob + L->off_alpha), (const __half*)(blob + L->off_V), nullptr, 0, dY, (int)L->N,
              dacc, KS};
    // one workgroup per CU fits (registers)
    const int cus = bwla_device_cus();
    const int G = row_tiles < cus ? row_tiles : cus;
    const bool fast = (L->N % 4 == 0) && dacc == nullptr;
    auto launch = [&](auto kern) -> hipError_t {
        static bwla_lds_attr attr;
        hipError_t e = attr.ensure((const void*)kern, lds);
        if (e != hipSuccess) return e;
        kern<<<dim3((unsigned)G), dim3(FD_THREADS), lds, st>>>(ra, ba);
        return hipGetLastError();
    };
    hipError_t e;
    if (s3.at <= 4) e = fast ? launch(decode_fused_kernel<4, true>) : launch(decode_fused_kernel<4, false>);
    else e = fast ? launch(decode_fused_kernel<8, true>) : launch(decode_fused_kernel<8, false>);
    if (e == hipSuccess) *done = true;
    return e;
}

hipError_t bwla_launch_code_sums(const int8_t* dq, int64_t M, int64_t K, int32_t* dqsum, hipStream_t st) {
    code_sums_kernel<<<dim3((unsigned)M), dim3(256), 0, st>>>(dq, K, dqsum);
    return hipGetLastError();
}
