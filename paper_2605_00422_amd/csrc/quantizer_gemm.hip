// fp64 GEMM of the offline quantizer (paper App. A.1 Algorithm 2: every dense contraction of the
// OKT rotation of the weight rows, of the Procrustes matrices C1 and C2 of App. A.2.2, and of the
// subspace iteration behind the truncated SVD of Sec. 3.2 runs through this one kernel).
//
// v_mfma_f64_16x16x4_f64: lane l holds A[l % 16][l / 16] and B[l / 16][l % 16]; result register v of
// lane l is D[4 v + l / 16][l % 16].  A workgroup of four wavefronts owns a 64 x 64 tile of C, each
// wavefront a 32 x 32 quarter (2 x 2 MFMA tiles); the operands of a 16-deep step of the contraction
// pass through LDS as [k][row] with rows padded to 80 doubles, so that the 16 lanes of a k share
// 128 contiguous bytes and the four k of an operand fall into different banks.  Global loads of the
// next step are in flight while the current one is multiplied.  Operands are read through strides
// (see quantizer_internal.h), so a lane's four loads of a step are either four consecutive doubles
// of its row (k contiguous) or four rows' worth of a coalesced 512-byte run (row index contiguous).
#include "quantizer_internal.h"

namespace {

typedef double d4 __attribute__((ext_vector_type(4)));
constexpr int TM = 64, TN = 64, TK = 16, LD = 80;

__device__ __forceinline__ long q_koff(int k, int kdiv, long kh, long kl) {
    if (kdiv > 0) {
        const int h = k / kdiv;
        return h * kh + (long)(k - h * kdiv) * kl;
    }
    return (long)k * kl;
}

__global__ __launch_bounds__(256) void qgemm_kernel(QGemm g) {
    if (g.skip && *g.skip) return;
    __shared__ double As[2][TK][LD];
    __shared__ double Bs[2][TK][LD];
    const int t = threadIdx.x, lane = t & 63, w = t >> 6;
    const int b = blockIdx.z / g.ksplit, s = blockIdx.z % g.ksplit;
    const int i0 = blockIdx.y * TM, j0 = blockIdx.x * TN;
    const int steps = (g.K + TK - 1) / TK;
    const int per = (steps + g.ksplit - 1) / g.ksplit;
    const int kbeg = min(g.K, s * per * TK), kend = min(g.K, (s + 1) * per * TK);
    const int li = t & 63, lk = (t >> 6) * 4;
    const bool a_ok = i0 + li < g.M, b_ok = j0 + li < g.N;
    const double* Ap = g.A + (long)b * g.bsA + (long)(i0 + li) * g.rsA;
    const double* Bp = g.B + (long)b * g.bsB + (long)(j0 + li) * g.csB;
    double ra[4], rb[4];
    auto gload = [&](int k0) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int k = k0 + lk + u;
            const bool in = k < kend;
            ra[u] = (a_ok && in) ? Ap[q_koff(k, g.kdivA, g.khA, g.klA)] : 0.0;
            rb[u] = (b_ok && in) ? Bp[q_koff(k, g.kdivB, g.khB, g.klB)] : 0.0;
        }
    };
    auto sstore = [&](int buf) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            As[buf][lk + u][li] = ra[u];
            Bs[buf][lk + u][li] = rb[u];
        }
    };
    const int wm = (w & 1) * 32, wn = (w >> 1) * 32, lr = lane & 15, lq = lane >> 4;
    d4 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int c = 0; c < 2; ++c) acc[a][c] = d4{0.0, 0.0, 0.0, 0.0};
    if (kbeg < kend) {
        gload(kbeg);
        sstore(0);
        __syncthreads();
        int buf = 0;
        for (int k0 = kbeg; k0 < kend; k0 += TK) {
            const bool more = k0 + TK < kend;
            if (more) gload(k0 + TK);
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const double a0 = As[buf][ks * 4 + lq][wm + lr], a1 = As[buf][ks * 4 + lq][wm + 16 + lr];
                const double b0 = Bs[buf][ks * 4 + lq][wn + lr], b1 = Bs[buf][ks * 4 + lq][wn + 16 + lr];
                acc[0][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b0, acc[0][0], 0, 0, 0);
                acc[0][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b1, acc[0][1], 0, 0, 0);
                acc[1][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b0, acc[1][0], 0, 0, 0);
                acc[1][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b1, acc[1][1], 0, 0, 0);
            }
            if (more) sstore(buf ^ 1);
            __syncthreads();
            buf ^= 1;
        }
    }
    const bool direct = g.ksplit == 1;
    double* Cb = direct ? g.C + (long)b * g.bsC : g.partials + ((long)s * g.batch + b) * (long)g.M * g.N;
    const double* C0b = (direct && g.C0 && g.beta != 0.0) ? g.C0 + (long)b * g.bsC : nullptr;
    const long rs = direct ? g.rsC : g.N;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = i0 + wm + a * 16 + 4 * v + lq, col = j0 + wn + c * 16 + lr;
                if (row < g.M && col < g.N) {
                    const long o = row * rs + col;
                    double x = acc[a][c][v];
                    if (direct) {
                        x *= g.alpha;
                        if (C0b) x += g.beta * C0b[o];
                    }
                    Cb[o] = x;
                }
            }
}

// adds the ksplit partial products in range order and applies alpha, beta, C0
__global__ __launch_bounds__(256) void qgemm_reduce_kernel(QGemm g) {
    if (g.skip && *g.skip) return;
    const long per = (long)g.M * g.N, total = per * g.batch;
    for (long e = (long)blockIdx.x * 256 + threadIdx.x; e < total; e += (long)gridDim.x * 256) {
        double x = 0.0;
        for (int s = 0; s < g.ksplit; ++s) x += g.partials[(long)s * total + e];
        const long b = e / per, rem = e - b * per;
        const long row = rem / g.N, col = rem - row * g.N;
        const long o = b * g.bsC + row * g.rsC + col;
        x *= g.alpha;
        if (g.C0 && g.beta != 0.0) x += g.beta * g.C0[o];
        g.C[o] = x;
    }
}

}  // namespace

hipError_t bwla_q_launch_gemm(const QGemm& g, hipStream_t st) {
    if (g.M <= 0 || g.N <= 0 || g.batch <= 0) return hipSuccess;
    const dim3 grid((g.N + TN - 1) / TN, (g.M + TM - 1) / TM, g.batch * g.ksplit);
    if (grid.y > 65535u || grid.z > 65535u) return hipErrorInvalidValue;
    hipLaunchKernelGGL(qgemm_kernel, grid, dim3(256), 0, st, g);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || g.ksplit == 1) return e;
    const long total = (long)g.M * g.N * g.batch;
    const int blocks = (int)((total + 255) / 256 < 1024 ? (total + 255) / 256 : 1024);
    hipLaunchKernelGGL(qgemm_reduce_kernel, dim3(blocks), dim3(256), 0, st, g);
    return hipGetLastError();
}
