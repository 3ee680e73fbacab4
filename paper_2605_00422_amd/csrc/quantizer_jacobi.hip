// One-sided Jacobi SVD of a small square matrix in one workgroup (Hestenes' method): the orthogonal
// Procrustes updates of the OKT factors (paper App. A.2.2, "Alternating Procrustes Updates":
// R = U V^T from the SVD of an n1 x n1 or n2 x n2 matrix) and the small eigenproblems of the
// subspace iteration behind the truncated SVD of the proximal step (Sec. 3.2; App. A.2.3).
//
// The columns of G are kept as contiguous rows of a work array (column j = row j), V likewise.
// A sweep visits every pair of columns once, in the round-robin order of a tournament: n / 2
// disjoint pairs per round, n - 1 rounds, the pairs of a round dealt to the 16 wavefronts.  A
// wavefront holds both columns of its pair in registers (up to four elements per lane), takes the
// three inner products by butterflies, and applies the plane rotation that makes the two columns
// orthogonal to them and to the matching columns of V.  Sweeps end when one passes without a
// rotation (every pair orthogonal to 1e-15 relative) or after 60.  At the end the column norms are
// the singular values, the normalized columns U, and V holds the right singular vectors.
#include "quantizer_internal.h"

namespace {

constexpr int JT = 1024, JW = JT / 64, JMAX = 256;

__device__ __forceinline__ double jwave_sum(double v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

__global__ __launch_bounds__(JT) void jacobi_kernel(QJacobi a) {
    if (a.skip && *a.skip) return;
    const int n = a.n, t = threadIdx.x, lane = t & 63, w = t >> 6;
    double* Wc = a.work;
    double* Vc = a.work + (size_t)n * n;
    __shared__ int pos[2][JMAX + 2];
    __shared__ int rotated;
    __shared__ double sg[JMAX];
    __shared__ int ord[JMAX];
    for (int e = t; e < n * n; e += JT) {
        const int j = e / n, i = e - j * n;
        Wc[e] = a.G[(size_t)i * n + j];
        Vc[e] = i == j ? 1.0 : 0.0;
    }
    const int np = (n + 1) & ~1;
    for (int i = t; i < np; i += JT) pos[0][i] = i;
    int cur = 0;
    __syncthreads();
    for (int sweep = 0; sweep < 60; ++sweep) {
        if (t == 0) rotated = 0;
        __syncthreads();
        for (int round = 0; round < np - 1; ++round) {
            for (int pr = w; pr < np / 2; pr += JW) {
                int p = pos[cur][pr], q = pos[cur][np - 1 - pr];
                if (p >= n || q >= n) continue;            // the bye of an odd n
                if (p > q) { const int s = p; p = q; q = s; }
                double* xp = Wc + (size_t)p * n;
                double* yp = Wc + (size_t)q * n;
                double x[4], y[4];
                double al = 0.0, be = 0.0, ga = 0.0;
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int e = lane + 64 * u;
                    x[u] = e < n ? xp[e] : 0.0;
                    y[u] = e < n ? yp[e] : 0.0;
                    al += x[u] * x[u];
                    be += y[u] * y[u];
                    ga += x[u] * y[u];
                }
                al = jwave_sum(al);
                be = jwave_sum(be);
                ga = jwave_sum(ga);
                if (al > 0.0 && be > 0.0 && fabs(ga) > 1.0e-15 * sqrt(al * be)) {
                    const double zeta = (be - al) / (2.0 * ga);
                    const double tt = copysign(1.0, zeta) / (fabs(zeta) + sqrt(1.0 + zeta * zeta));
                    const double cs = 1.0 / sqrt(1.0 + tt * tt), sn = cs * tt;
                    double* vp = Vc + (size_t)p * n;
                    double* vq = Vc + (size_t)q * n;
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int e = lane + 64 * u;
                        if (e < n) {
                            xp[e] = cs * x[u] - sn * y[u];
                            yp[e] = sn * x[u] + cs * y[u];
                            const double vx = vp[e], vy = vq[e];
                            vp[e] = cs * vx - sn * vy;
                            vq[e] = sn * vx + cs * vy;
                        }
                    }
                    if (lane == 0) rotated = 1;
                }
            }
            // next round of the tournament: position 0 stays, the others move on by one
            for (int i = t; i < np; i += JT) pos[cur ^ 1][i] = i == 0 ? pos[cur][0] : (i == 1 ? pos[cur][np - 1] : pos[cur][i - 1]);
            cur ^= 1;
            __syncthreads();
        }
        if (!rotated) break;
        __syncthreads();
    }
    for (int j = w; j < n; j += JW) {
        double s = 0.0;
        for (int e = lane; e < n; e += 64) s += Wc[(size_t)j * n + e] * Wc[(size_t)j * n + e];
        s = jwave_sum(s);
        if (lane == 0) sg[j] = sqrt(s);
    }
    __syncthreads();
    for (int j = t; j < n; j += JT) {
        int rank = 0;
        for (int i = 0; i < n; ++i) rank += (sg[i] > sg[j] || (sg[i] == sg[j] && i < j)) ? 1 : 0;
        ord[rank] = j;
    }
    __syncthreads();
    for (int jj = w; jj < n; jj += JW) {
        const int j = ord[jj];
        const double s = sg[j];
        const double scale = s > 0.0 ? (a.pw == 0.0 ? 1.0 : pow(s, a.pw)) : 0.0;
        for (int e = lane; e < n; e += 64) {
            if (a.Ws) a.Ws[(size_t)jj * n + e] = Wc[(size_t)j * n + e];
            if (a.Vs) a.Vs[(size_t)jj * n + e] = scale * Vc[(size_t)j * n + e];
        }
    }
    if (t == 0 && a.prev_sig && a.done) {
        double worst = 0.0;
        for (int jj = 0; jj < a.lead && jj < n; ++jj) {
            const double s = sg[ord[jj]];
            worst = fmax(worst, fabs(s - a.prev_sig[jj]) / fmax(s, 1.0e-300));
        }
        if (worst <= a.tol) *a.done = 1;
    }
    __syncthreads();
    for (int jj = t; jj < n; jj += JT) {
        const double s = sg[ord[jj]];
        if (a.sig) a.sig[jj] = s;
        if (a.prev_sig) a.prev_sig[jj] = s;
    }
}

}  // namespace

hipError_t bwla_q_launch_jacobi(const QJacobi& j, hipStream_t st) {
    if (j.n < 1 || j.n > JMAX) return hipErrorInvalidValue;
    hipLaunchKernelGGL(jacobi_kernel, dim3(1), dim3(JT), 0, st, j);
    return hipGetLastError();
}
