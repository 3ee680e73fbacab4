// Row-wise steps of the offline quantizer (paper App. A.1 Algorithm 2; App. A.2.2 for the mixture,
// its EM updates and the MM targets; App. A.2.3 for the gradient behind the proximal step), fp64.
// One workgroup of 256 threads per weight row; a row is read from global memory once per pass
// (it stays in L2 between the passes of one kernel).  Sums are taken per thread in a fixed order,
// then over the wavefront by butterflies and over the four wavefronts in wavefront order, so that a
// result does not depend on the launch.
#include "quantizer_internal.h"

namespace {

constexpr int RT = 256;

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}
// sum over the workgroup, returned to every thread; `sh` holds 4 doubles
__device__ __forceinline__ double block_sum(double v, double* sh) {
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    return (sh[0] + sh[1]) + (sh[2] + sh[3]);
}

__global__ void convert_f32_f64_kernel(const float* src, double* dst, size_t count) {
    for (size_t e = (size_t)blockIdx.x * RT + threadIdx.x; e < count; e += (size_t)gridDim.x * RT) dst[e] = (double)src[e];
}
__global__ void convert_f64_f32_kernel(const double* src, float* dst, size_t count) {
    for (size_t e = (size_t)blockIdx.x * RT + threadIdx.x; e < count; e += (size_t)gridDim.x * RT) dst[e] = (float)src[e];
}

// X = Y H: the row mean taken out (Sec. 3.1, "Transformation Objectives")
__global__ __launch_bounds__(RT) void center_kernel(const double* Y, double* X, double* ybar, int m) {
    __shared__ double sh[4];
    const double* y = Y + (size_t)blockIdx.x * m;
    double* x = X + (size_t)blockIdx.x * m;
    double s = 0.0;
    for (int j = threadIdx.x; j < m; j += RT) s += y[j];
    const double mean = block_sum(s, sh) / m;
    if (X)
        for (int j = threadIdx.x; j < m; j += RT) x[j] = y[j] - mean;
    if (ybar && threadIdx.x == 0) ybar[blockIdx.x] = mean;
}

// Algorithm 2's empirical start: c = mean |x|, s^2 = mean (|x| - c)^2, floored
__global__ __launch_bounds__(RT) void init_theta_kernel(const double* X, int m, double s2_min, double* c, double* s2) {
    __shared__ double sh[4];
    const double* x = X + (size_t)blockIdx.x * m;
    double s = 0.0;
    for (int j = threadIdx.x; j < m; j += RT) s += fabs(x[j]);
    const double ci = block_sum(s, sh) / m;
    double q = 0.0;
    for (int j = threadIdx.x; j < m; j += RT) {
        const double d = fabs(x[j]) - ci;
        q += d * d;
    }
    const double v = block_sum(q, sh) / m;
    if (threadIdx.x == 0) {
        c[blockIdx.x] = ci;
        s2[blockIdx.x] = fmax(v, s2_min);
    }
}

// 2 r^+ - 1 = tanh(c x / s^2): the two densities' ratio is exp(2 c x / s^2) (App. A.2.2, E step)
__device__ __forceinline__ double signed_resp(double x, double c, double inv_s2) { return tanh(c * x * inv_s2); }

// one EM update of a row's mixture (App. A.2.2): c from the responsibilities at the old parameters,
// then s^2 with the new c
__global__ __launch_bounds__(RT) void em_kernel(const double* X, int m, double s2_min, double* c, double* s2) {
    __shared__ double sh[4];
    const double* x = X + (size_t)blockIdx.x * m;
    const double c0 = c[blockIdx.x], inv = 1.0 / s2[blockIdx.x];
    double s = 0.0;
    for (int j = threadIdx.x; j < m; j += RT) s += signed_resp(x[j], c0, inv) * x[j];
    const double c1 = block_sum(s, sh) / m;
    double q = 0.0;
    for (int j = threadIdx.x; j < m; j += RT) {
        const double r = 0.5 * (1.0 + signed_resp(x[j], c0, inv));
        const double dp = x[j] - c1, dm = x[j] + c1;
        q += r * dp * dp + (1.0 - r) * dm * dm;
    }
    const double v = block_sum(q, sh) / m;
    if (threadIdx.x == 0) {
        c[blockIdx.x] = c1;
        s2[blockIdx.x] = fmax(v, s2_min);
    }
}

// per-row sums of -log[ 1/2 phi(x; c, s^2) + 1/2 phi(x; -c, s^2) ], in log space
__global__ __launch_bounds__(RT) void nll_rows_kernel(const double* X, int m, const double* c, const double* s2, double* part) {
    __shared__ double sh[4];
    const double* x = X + (size_t)blockIdx.x * m;
    const double ci = c[blockIdx.x], v = s2[blockIdx.x];
    const double lognorm = -0.5 * log(2.0 * 3.14159265358979323846 * v), h = 0.5 / v;
    double s = 0.0;
    for (int j = threadIdx.x; j < m; j += RT) {
        const double dp = x[j] - ci, dm = x[j] + ci;
        const double lp = lognorm - dp * dp * h, lm = lognorm - dm * dm * h;
        const double hi = fmax(lp, lm), lo = fmin(lp, lm);
        s -= hi + log1p(exp(lo - hi)) + log(0.5);
    }
    const double tot = block_sum(s, sh);
    if (threadIdx.x == 0) part[blockIdx.x] = tot;
}
__global__ __launch_bounds__(RT) void sum_scale_kernel(const double* part, int n, double scale, double* out) {
    __shared__ double sh[4];
    double s = 0.0;
    for (int i = threadIdx.x; i < n; i += RT) s += part[i];
    const double tot = block_sum(s, sh);
    if (threadIdx.x == 0) out[0] = tot * scale;
}

// MM targets on the uncentered rotated rows (App. A.2.2, "MM Surrogate"): m_ij = (2 r_ij - 1) c_i at
// x = y - ybar; target H m_i + ybar_i 1 (the concave part of the centered objective majorized by its
// tangent); stored times lambda_i = 1 / s_i^2, the weight of the row in the Procrustes matrices
__global__ __launch_bounds__(RT) void targets_kernel(const double* Y, const double* ybar, const double* c, const double* s2,
                                                     int m, double* T) {
    __shared__ double sh[4];
    const double* y = Y + (size_t)blockIdx.x * m;
    double* tg = T + (size_t)blockIdx.x * m;
    const double yb = ybar[blockIdx.x], ci = c[blockIdx.x], lam = 1.0 / s2[blockIdx.x];
    double s = 0.0;
    for (int j = threadIdx.x; j < m; j += RT) s += ci * signed_resp(y[j] - yb, ci, lam);
    const double mbar = block_sum(s, sh) / m;
    for (int j = threadIdx.x; j < m; j += RT) tg[j] = lam * (ci * signed_resp(y[j] - yb, ci, lam) - mbar + yb);
}

__global__ __launch_bounds__(RT) void prox_factor_kernel(const double* s2, int n, double nm, double mu, double* fac) {
    __shared__ double sh[RT];
    double v = 1.0e300;
    for (int i = threadIdx.x; i < n; i += RT) v = fmin(v, s2[i]);
    sh[threadIdx.x] = v;
    __syncthreads();
    for (int o = RT / 2; o > 0; o >>= 1) {
        if (threadIdx.x < o) sh[threadIdx.x] = fmin(sh[threadIdx.x], sh[threadIdx.x + o]);
        __syncthreads();
    }
    if (threadIdx.x == 0) fac[0] = mu > 0.0 ? 1.0 / (nm * mu) : sh[0];
}

// fac * H[(x - m) lambda]: minus the gradient of L_GMM in the centered coordinates, over mu
// (App. A.2.2 for d L / d x_ij = (x_ij - m_ij) / (n m s_i^2); App. A.2.3 for the adjoint's H)
__global__ __launch_bounds__(RT) void gradx_kernel(const double* X, const double* c, const double* s2, const double* fac,
                                                   int m, double* GX) {
    __shared__ double sh[4];
    const double* x = X + (size_t)blockIdx.x * m;
    double* gx = GX + (size_t)blockIdx.x * m;
    const double ci = c[blockIdx.x], lam = 1.0 / s2[blockIdx.x], f = fac[0];
    double s = 0.0;
    for (int j = threadIdx.x; j < m; j += RT) s += (x[j] - ci * signed_resp(x[j], ci, lam)) * lam;
    const double gbar = block_sum(s, sh) / m;
    for (int j = threadIdx.x; j < m; j += RT) gx[j] = f * ((x[j] - ci * signed_resp(x[j], ci, lam)) * lam - gbar);
}

__device__ __forceinline__ uint32_t hash32(uint32_t x) {
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return x;
}
__global__ void fill_hash_kernel(double* Q, size_t count, uint32_t seed) {
    for (size_t e = (size_t)blockIdx.x * RT + threadIdx.x; e < count; e += (size_t)gridDim.x * RT) {
        const uint32_t h = hash32((uint32_t)e * 0x9e3779b9u + hash32(seed + (uint32_t)(e >> 32)));
        Q[e] = (double)h * (1.0 / 2147483648.0) - 1.0;
    }
}
__global__ void fill_identity_kernel(double* R, int n) {
    for (int e = blockIdx.x * RT + threadIdx.x; e < n * n; e += gridDim.x * RT) R[e] = (e / n == e % n) ? 1.0 : 0.0;
}
// X = C / ||C||_F, one workgroup (the start of the Newton-Schulz iteration for the polar factor:
// every singular value of X is at most 1); a zero matrix stays zero
__global__ __launch_bounds__(RT) void scale_inv_frob_kernel(const double* C, int count, double* X) {
    __shared__ double sh[4];
    double s = 0.0;
    for (int e = threadIdx.x; e < count; e += RT) s += C[e] * C[e];
    const double tot = block_sum(s, sh);
    const double inv = tot > 0.0 ? 1.0 / sqrt(tot) : 0.0;
    for (int e = threadIdx.x; e < count; e += RT) X[e] = C[e] * inv;
}
// out[0] = 1 / sqrt(largest absolute column sum of G): for G = X^T X that sum bounds sigma_max(X)^2
__global__ __launch_bounds__(RT) void gram_inv_norm_kernel(const double* G, int nn, double* out) {
    __shared__ double sh[RT];
    double worst = 0.0;
    for (int j = threadIdx.x; j < nn; j += RT) {
        double s = 0.0;
        for (int i = 0; i < nn; ++i) s += fabs(G[(size_t)i * nn + j]);
        worst = s > worst ? s : worst;
    }
    sh[threadIdx.x] = worst;
    __syncthreads();
    if (threadIdx.x == 0) {
        double w = 0.0;
        for (int i = 0; i < RT; ++i) w = sh[i] > w ? sh[i] : w;
        out[0] = w > 0.0 ? 1.0 / sqrt(w) : 0.0;
    }
}
__global__ void scale_by_kernel(double* X, size_t count, const double* s) {
    const double f = s[0];
    for (size_t e = (size_t)blockIdx.x * RT + threadIdx.x; e < count; e += (size_t)gridDim.x * RT) X[e] *= f;
}
// *done = 1 once max |G - I| <= tol (G nn x nn, one workgroup); never cleared here
__global__ __launch_bounds__(RT) void near_identity_kernel(const double* G, int nn, double tol, int* done) {
    __shared__ double sh[4];
    double worst = 0.0;
    for (int e = threadIdx.x; e < nn * nn; e += RT) {
        const double d = fabs(G[e] - (e / nn == e % nn ? 1.0 : 0.0));
        worst = d > worst || d != d ? d : worst;            // (a NaN stays)
    }
    // (the largest by way of the sum helper's layout: per wavefront, then over the four)
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const double o = __shfl_xor(worst, off, 64);
        worst = o > worst || o != o ? o : worst;
    }
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = worst;
    __syncthreads();
    if (threadIdx.x == 0) {
        double w = sh[0];
        for (int i = 1; i < 4; ++i) w = sh[i] > w || sh[i] != sh[i] ? sh[i] : w;
        if (w <= tol) *done = 1;
    }
}
__global__ void set_int_kernel(int* p, int v) { *p = v; }
__global__ void fill_value_kernel(double* p, size_t count, double v) {
    for (size_t e = (size_t)blockIdx.x * RT + threadIdx.x; e < count; e += (size_t)gridDim.x * RT) p[e] = v;
}
__global__ void pow_vec_kernel(const double* src, double pw, int count, double* dst) {
    for (int e = blockIdx.x * RT + threadIdx.x; e < count; e += gridDim.x * RT) dst[e] = src[e] > 0.0 ? pow(src[e], pw) : 0.0;
}

__global__ void scale_cols_f32_kernel(const double* src, const double* lam, double pw, int n, int k, float* dst) {
    for (size_t e = (size_t)blockIdx.x * RT + threadIdx.x; e < (size_t)n * k; e += (size_t)gridDim.x * RT) {
        const double l = lam[e % k];
        dst[e] = (float)(l > 0.0 ? src[e] * pow(l, pw) : 0.0);
    }
}

// Algorithm 2, "Final binarization": shift = row mean, scale = row mean of |y - shift|
__global__ __launch_bounds__(RT) void row_stats_kernel(const double* Y, int m, double* mean, double* absdev) {
    __shared__ double sh[4];
    const double* y = Y + (size_t)blockIdx.x * m;
    double s = 0.0;
    for (int j = threadIdx.x; j < m; j += RT) s += y[j];
    const double mu = block_sum(s, sh) / m;
    double a = 0.0;
    for (int j = threadIdx.x; j < m; j += RT) a += fabs(y[j] - mu);
    const double ad = block_sum(a, sh) / m;
    if (threadIdx.x == 0) {
        mean[blockIdx.x] = mu;
        absdev[blockIdx.x] = ad;
    }
}

inline int flat_blocks(size_t count) {
    const size_t b = (count + RT - 1) / RT;
    return (int)(b < 4096 ? (b ? b : 1) : 4096);
}

}  // namespace

hipError_t bwla_q_launch_convert_f32_f64(const float* src, double* dst, size_t count, hipStream_t st) {
    hipLaunchKernelGGL(convert_f32_f64_kernel, dim3(flat_blocks(count)), dim3(RT), 0, st, src, dst, count);
    return hipGetLastError();
}
hipError_t bwla_q_launch_convert_f64_f32(const double* src, float* dst, size_t count, hipStream_t st) {
    hipLaunchKernelGGL(convert_f64_f32_kernel, dim3(flat_blocks(count)), dim3(RT), 0, st, src, dst, count);
    return hipGetLastError();
}
hipError_t bwla_q_launch_center(const double* Y, double* X, double* ybar, int n, int m, hipStream_t st) {
    hipLaunchKernelGGL(center_kernel, dim3(n), dim3(RT), 0, st, Y, X, ybar, m);
    return hipGetLastError();
}
hipError_t bwla_q_launch_init_theta(const double* X, int n, int m, double s2_min, double* c, double* s2, hipStream_t st) {
    hipLaunchKernelGGL(init_theta_kernel, dim3(n), dim3(RT), 0, st, X, m, s2_min, c, s2);
    return hipGetLastError();
}
hipError_t bwla_q_launch_em(const double* X, int n, int m, double s2_min, double* c, double* s2, hipStream_t st) {
    hipLaunchKernelGGL(em_kernel, dim3(n), dim3(RT), 0, st, X, m, s2_min, c, s2);
    return hipGetLastError();
}
hipError_t bwla_q_launch_nll(const double* X, int n, int m, const double* c, const double* s2, double* row_part,
                             double* out, hipStream_t st) {
    hipLaunchKernelGGL(nll_rows_kernel, dim3(n), dim3(RT), 0, st, X, m, c, s2, row_part);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(sum_scale_kernel, dim3(1), dim3(RT), 0, st, row_part, n, 1.0 / ((double)n * m), out);
    return hipGetLastError();
}
hipError_t bwla_q_launch_targets(const double* Y, const double* ybar, const double* c, const double* s2, int n, int m,
                                 double* T, hipStream_t st) {
    hipLaunchKernelGGL(targets_kernel, dim3(n), dim3(RT), 0, st, Y, ybar, c, s2, m, T);
    return hipGetLastError();
}
hipError_t bwla_q_launch_prox_factor(const double* s2, int n, int m, double mu, double* fac, hipStream_t st) {
    hipLaunchKernelGGL(prox_factor_kernel, dim3(1), dim3(RT), 0, st, s2, n, (double)n * m, mu, fac);
    return hipGetLastError();
}
hipError_t bwla_q_launch_gradx(const double* X, const double* c, const double* s2, const double* fac, int n, int m,
                               double* GX, hipStream_t st) {
    hipLaunchKernelGGL(gradx_kernel, dim3(n), dim3(RT), 0, st, X, c, s2, fac, m, GX);
    return hipGetLastError();
}
hipError_t bwla_q_launch_fill_hash(double* Q, size_t count, uint32_t seed, hipStream_t st) {
    hipLaunchKernelGGL(fill_hash_kernel, dim3(flat_blocks(count)), dim3(RT), 0, st, Q, count, seed);
    return hipGetLastError();
}
hipError_t bwla_q_launch_fill_identity(double* R, int n, hipStream_t st) {
    hipLaunchKernelGGL(fill_identity_kernel, dim3(flat_blocks((size_t)n * n)), dim3(RT), 0, st, R, n);
    return hipGetLastError();
}
hipError_t bwla_q_launch_scale_inv_frob(const double* C, int count, double* X, hipStream_t st) {
    hipLaunchKernelGGL(scale_inv_frob_kernel, dim3(1), dim3(RT), 0, st, C, count, X);
    return hipGetLastError();
}
hipError_t bwla_q_launch_gram_inv_norm(const double* G, int nn, double* out, hipStream_t st) {
    hipLaunchKernelGGL(gram_inv_norm_kernel, dim3(1), dim3(RT), 0, st, G, nn, out);
    return hipGetLastError();
}
hipError_t bwla_q_launch_scale_by(double* X, size_t count, const double* s, hipStream_t st) {
    hipLaunchKernelGGL(scale_by_kernel, dim3(flat_blocks(count)), dim3(RT), 0, st, X, count, s);
    return hipGetLastError();
}
hipError_t bwla_q_launch_near_identity(const double* G, int nn, double tol, int* done, hipStream_t st) {
    hipLaunchKernelGGL(near_identity_kernel, dim3(1), dim3(RT), 0, st, G, nn, tol, done);
    return hipGetLastError();
}
hipError_t bwla_q_launch_set_int(int* p, int v, hipStream_t st) {
    hipLaunchKernelGGL(set_int_kernel, dim3(1), dim3(1), 0, st, p, v);
    return hipGetLastError();
}
hipError_t bwla_q_launch_fill_value(double* p, size_t count, double v, hipStream_t st) {
    hipLaunchKernelGGL(fill_value_kernel, dim3(flat_blocks(count)), dim3(RT), 0, st, p, count, v);
    return hipGetLastError();
}
hipError_t bwla_q_launch_pow_vec(const double* src, double pw, int count, double* dst, hipStream_t st) {
    hipLaunchKernelGGL(pow_vec_kernel, dim3(flat_blocks((size_t)count)), dim3(RT), 0, st, src, pw, count, dst);
    return hipGetLastError();
}
hipError_t bwla_q_launch_scale_cols_f32(const double* src, const double* lam, double pw, int n, int k, float* dst,
                                        hipStream_t st) {
    hipLaunchKernelGGL(scale_cols_f32_kernel, dim3(flat_blocks((size_t)n * k)), dim3(RT), 0, st, src, lam, pw, n, k, dst);
    return hipGetLastError();
}
hipError_t bwla_q_launch_row_stats(const double* Y, int n, int m, double* mean, double* absdev, hipStream_t st) {
    hipLaunchKernelGGL(row_stats_kernel, dim3(n), dim3(RT), 0, st, Y, m, mean, absdev);
    return hipGetLastError();
}
