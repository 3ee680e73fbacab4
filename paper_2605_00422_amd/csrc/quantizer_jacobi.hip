// One-sided Jacobi SVD of a small square matrix in one workgroup (Hestenes' method): the orthogonal
// Procrustes updates of the OKT factors (paper App. A.2.2, "Alternating Procrustes Updates":
// R = U V^T from the SVD of an n1 x n1 or n2 x n2 matrix) and the small eigenproblems of the
// subspace iteration behind the truncated SVD of the proximal step (Sec. 3.2; App. A.2.3).
//
// The columns of G are kept as contiguous rows of a work array (column j = row j), V likewise.
// A sweep visits every pair of columns once, in the round-robin order of a tournament: n / 2
// disjoint pairs per round, n - 1 rounds.  A pair belongs to a group of lanes that holds both columns
// in registers (up to four elements per lane), takes the three inner products, and applies the plane
// rotation that makes the two columns orthogonal to them and to the matching columns of V.  Up to
// n = 64 a group is one row of 16 lanes -- four pairs per wavefront, all pairs of a round at once,
// the inner products summed on DPP row operations alone; larger matrices give a pair two rows (one
// lane exchange more) or a whole wavefront (row sums on DPP, the four rows added through lane reads).  Sweeps end when one passes
// without a rotation (every pair orthogonal to 1e-15 relative) or after 60.  At the end the column
// norms are the singular values, the normalized columns U, and V holds the right singular vectors.
// Up to n = 96 both arrays (2 n^2 doubles, at most 144 KiB) live in LDS, where a round costs an LDS
// round trip instead of an L2 one; larger matrices work in the caller's scratch (L2-resident).
// For a symmetric positive semidefinite matrix (the Gram matrices of the subspace iteration) V is not
// kept at all -- its columns are the normalized columns of the rotated matrix -- so that matrices up
// to 136 wide fit LDS; there a pair takes two rows of lanes up to n = 128.
#include "bwla_internal.h"
#include "quantizer_internal.h"

namespace {

constexpr int JMAX = 256, JLDS = BWLA_Q_JACOBI_LDS, JLDS_SYM = BWLA_Q_JACOBI_SYM_LDS;
// threads of the workgroup: a row of 16 lanes per pair serves 32 pairs (n <= 64) with 512 threads
constexpr int jacobi_threads(int gw) { return gw == 16 ? 512 : 1024; }

template <int CTRL>
__device__ __forceinline__ double jdpp(double v) {
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), CTRL, 0xf, 0xf, true);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), CTRL, 0xf, 0xf, true);
    return __hiloint2double(hi, lo);
}
// sum over a row of 16 lanes, the same value in each of them
__device__ __forceinline__ double jrow_sum(double v) {
    v += jdpp<0xB1>(v);      // quad_perm [1,0,3,2]
    v += jdpp<0x4E>(v);      // quad_perm [2,3,0,1]
    v += jdpp<0x141>(v);     // row_half_mirror
    v += jdpp<0x140>(v);     // row_mirror
    return v;
}
__device__ __forceinline__ double jread(double v, int lane) {
    return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(v), lane),
                            __builtin_amdgcn_readlane(__double2loint(v), lane));
}
template <int GW>
__device__ __forceinline__ double jgroup_sum(double v) {
    v = jrow_sum(v);
    if (GW == 32) v += __shfl_xor(v, 16, 64);          // the other row of the pair's two
    if (GW == 64) v = (jread(v, 0) + jread(v, 16)) + (jread(v, 32) + jread(v, 48));
    return v;
}

// GW: lanes per pair (16 for n <= 64, 32 for n <= 128, else 64); LDS: the work arrays live in dynamic LDS.
// ACCV: the rotations are accumulated into V.  Without it (a symmetric positive semidefinite G, whose
// left and right singular vectors coincide) the right singular vectors are the normalized columns of
// the rotated G themselves -- orthogonal to the tolerance of the sweeps, and as accurate as eigenvectors
// as the accumulated ones (both diagonalize G up to eps ||G||) -- at half the work and half the memory.
template <int GW, bool LDS, bool ACCV>
__global__ __launch_bounds__(jacobi_threads(GW)) void jacobi_kernel(QJacobi a) {
    if (a.skip && *a.skip) return;
    constexpr int JT = jacobi_threads(GW), JW = JT / 64;
    const int n = a.n, t = threadIdx.x, lane = t & 63, w = t >> 6;
    extern __shared__ double jlds[];
    double* Wc = LDS ? jlds : a.work;
    double* Vc = Wc + (size_t)n * n;
    __shared__ int pos[2][JMAX + 2];
    __shared__ int rotated;
    __shared__ double sg[JMAX];
    __shared__ int ord[JMAX];
    for (int e = t; e < n * n; e += JT) {
        const int j = e / n, i = e - j * n;
        Wc[e] = a.G[(size_t)i * n + j];
        if (ACCV) Vc[e] = i == j ? 1.0 : 0.0;
    }
    const int np = (n + 1) & ~1;
    for (int i = t; i < np; i += JT) pos[0][i] = i;
    int cur = 0;
    constexpr int GROUPS = JT / GW;
    const int gid = t / GW, sl = t % GW;
    __syncthreads();
    for (int sweep = 0; sweep < 60; ++sweep) {
        if (t == 0) rotated = 0;
        __syncthreads();
        for (int round = 0; round < np - 1; ++round) {
            for (int base = 0; base < np / 2; base += GROUPS) {        // the same trip count in every lane
                const int pr = base + gid;
                int p = 0, q = 0;
                bool live = pr < np / 2;
                if (live) {
                    p = pos[cur][pr];
                    q = pos[cur][np - 1 - pr];
                    live = p < n && q < n;                              // else the bye of an odd n
                    if (p > q) { const int s = p; p = q; q = s; }
                }
                double* xp = Wc + (size_t)p * n;
                double* yp = Wc + (size_t)q * n;
                double x[4], y[4];
                double al = 0.0, be = 0.0, ga = 0.0;
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int e = sl + GW * u;
                    const bool in = live && e < n;
                    x[u] = in ? xp[e] : 0.0;
                    y[u] = in ? yp[e] : 0.0;
                    al += x[u] * x[u];
                    be += y[u] * y[u];
                    ga += x[u] * y[u];
                }
                al = jgroup_sum<GW>(al);
                be = jgroup_sum<GW>(be);
                ga = jgroup_sum<GW>(ga);
                // (|ga| > 1e-15 sqrt(al be), without the root; four special-function calls a rotation instead
                // of six: their dependent chain is most of what a round costs)
                if (live && al > 0.0 && be > 0.0 && ga * ga > 1.0e-30 * (al * be)) {
                    const double zeta = (be - al) / (2.0 * ga);
                    const double tt = copysign(1.0, zeta) / (fabs(zeta) + sqrt(1.0 + zeta * zeta));
                    const double cs = rsqrt(1.0 + tt * tt), sn = cs * tt;
                    double* vp = Vc + (size_t)p * n;
                    double* vq = Vc + (size_t)q * n;
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int e = sl + GW * u;
                        if (e < n) {
                            xp[e] = cs * x[u] - sn * y[u];
                            yp[e] = sn * x[u] + cs * y[u];
                            if (ACCV) {
                                const double vx = vp[e], vy = vq[e];
                                vp[e] = cs * vx - sn * vy;
                                vq[e] = sn * vx + cs * vy;
                            }
                        }
                    }
                    if (sl == 0) rotated = 1;
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
        s = jgroup_sum<64>(s);
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
        double scale = s > 0.0 ? (a.pw == 0.0 ? 1.0 : pow(s, a.pw)) : 0.0;
        if (!ACCV && s > 0.0) scale /= s;                   // v_j = the column of the rotated G over its norm
        for (int e = lane; e < n; e += 64) {
            if (a.Ws) a.Ws[(size_t)jj * n + e] = Wc[(size_t)j * n + e];
            if (a.Vs) a.Vs[(size_t)jj * n + e] = scale * (ACCV ? Vc[(size_t)j * n + e] : Wc[(size_t)j * n + e]);
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
    const bool in_lds = j.n <= (j.sym ? JLDS_SYM : JLDS);
    const size_t lds = in_lds ? (size_t)(j.sym ? 1 : 2) * j.n * j.n * sizeof(double) : 0;
    auto launch = [&](auto kern, int threads) {
        if (lds > 48 * 1024) {
            const hipError_t e = bwla_ensure_lds((const void*)kern, lds);
            if (e != hipSuccess) return e;
        }
        hipLaunchKernelGGL(kern, dim3(1), dim3(threads), lds, st, j);
        return hipGetLastError();
    };
    if (j.sym) {
        if (j.n <= 64) return launch(jacobi_kernel<16, true, false>, jacobi_threads(16));
        if (j.n <= 128) return launch(jacobi_kernel<32, true, false>, jacobi_threads(32));
        if (in_lds) return launch(jacobi_kernel<64, true, false>, jacobi_threads(64));
        return launch(jacobi_kernel<64, false, false>, jacobi_threads(64));
    }
    if (j.n <= 64) return launch(jacobi_kernel<16, true, true>, jacobi_threads(16));
    if (in_lds) return launch(jacobi_kernel<64, true, true>, jacobi_threads(64));
    return launch(jacobi_kernel<64, false, true>, jacobi_threads(64));
}
