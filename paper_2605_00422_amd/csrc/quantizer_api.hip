// C ABI of the offline quantizer (paper App. A.1 Algorithm 2): validation and scratch layout on the
// host, then the sequence of launches -- fp64 GEMMs on strided views (quantizer_gemm.hip), row-wise
// mixture kernels (quantizer_rows.hip), one-sided Jacobi SVDs (quantizer_jacobi.hip).  Nothing
// here allocates or synchronizes; a call is a chain of launches on the caller's stream.
#include <math.h>

#include "quantizer_internal.h"

namespace {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t al256(size_t x) { return (x + 255u) & ~(size_t)255; }
constexpr size_t PART_BYTES = (size_t)64 << 20;   // partial products of split contractions

// Scratch layout.  big[0..4]: W in fp64, W - M, the half-rotated rows (W - M) R2 viewed as
// (n n1) x n2, the rotated rows, and the centered rows / the MM targets.
struct QPlan {
    int n, m, n1, n2, k, p, jn;
    size_t big[5], R1, R2, C, A, Bt, A2, Bt2, c, s2, ybar, rowpart, scal, Q, Q2, Zs, G, Vs, Ws, sig, prev, lam,
        jwork, flags, partials, bytes;
};

bwla_status_t make_plan(int64_t n, int64_t m, int32_t n1, int32_t n2, int32_t k, QPlan& P) {
    if (n <= 0 || m <= 0 || n1 <= 0 || n2 <= 0 || k < 0) return BWLA_ERR_SHAPE;
    // n1 = n2 = 1 with m > 1 is the sizing of the calls that take no factors (bwla_q_truncate_rank)
    const bool no_factors = n1 == 1 && n2 == 1;
    if (!no_factors && (int64_t)n1 * n2 != m) return BWLA_ERR_SHAPE;
    if (k > n || k > m) return BWLA_ERR_SHAPE;
    if (n1 > 256 || n2 > 256 || k > 128 || n > 65535 || m > 65536) return BWLA_ERR_UNSUPPORTED;
    P.n = (int)n; P.m = (int)m; P.n1 = n1; P.n2 = n2; P.k = k;
    int p = k > 0 ? (2 * k > k + 16 ? 2 * k : k + 16) : 0;
    if (p > n) p = (int)n;
    if (p > m) p = (int)m;
    P.p = p;
    P.jn = p > n1 ? p : n1;
    if (n2 > P.jn) P.jn = n2;
    const size_t D = sizeof(double), nm = (size_t)n * m, jj = (size_t)P.jn * P.jn;
    size_t off = 0;
    auto take = [&](size_t bytes) { const size_t o = off; off = al256(off + bytes); return o; };
    for (int i = 0; i < 5; ++i) P.big[i] = take(nm * D);
    P.R1 = take((size_t)n1 * n1 * D); P.R2 = take((size_t)n2 * n2 * D); P.C = take(jj * D);
    P.A = take((size_t)n * k * D); P.Bt = take((size_t)m * k * D);
    P.A2 = take((size_t)n * k * D); P.Bt2 = take((size_t)m * k * D);
    P.c = take(n * D); P.s2 = take(n * D); P.ybar = take(n * D); P.rowpart = take(n * D);
    P.scal = take(64 * D);
    P.Q = take((size_t)m * p * D); P.Q2 = take((size_t)m * p * D); P.Zs = take((size_t)n * p * D);
    P.G = take(jj * D); P.Vs = take(jj * D); P.Ws = take(jj * D);
    P.sig = take(P.jn * D); P.prev = take(P.jn * D); P.lam = take(P.jn * D);
    P.jwork = take(2 * jj * D);
    P.flags = take(256);
    P.partials = take(PART_BYTES);
    P.bytes = off;
    return BWLA_OK;
}

struct Ctx {
    QPlan P; char* ws; hipStream_t st; hipError_t err = hipSuccess;
    double* d(size_t off) const { return reinterpret_cast<double*>(ws + off); }
    int* done() const { return reinterpret_cast<int*>(ws + P.flags); }
    void ck(hipError_t e) { if (err == hipSuccess && e != hipSuccess) err = e; }
};

// picks the split of the contraction: about 1024 workgroups, at least 256 of K per range, partial
// products within the scratch reserved for them
void gemm(Ctx& x, QGemm g, const int* skip = nullptr) {
    const long tiles = (long)((g.M + 63) / 64) * ((g.N + 63) / 64) * g.batch;
    long S = 1;
    if (tiles < 512) {
        S = 1024 / tiles;
        if (S > g.K / 256) S = g.K / 256;
        const long cap = (long)(PART_BYTES / ((size_t)g.batch * g.M * g.N * sizeof(double)));
        if (S > cap) S = cap;
        if (S > 256) S = 256;
        if (S < 2) S = 1;
    }
    g.ksplit = (int)S;
    g.partials = x.d(x.P.partials);
    g.skip = skip;
    x.ck(bwla_q_launch_gemm(g, x.st));
}

// dst rows = src rows times R1 (x) R2 (transposed = false) or times its transpose R1^T (x) R2^T;
// half = the (n n1) x n2 intermediate src_i R2.  src may equal dst; half must differ from both.
void rotate_rows(Ctx& x, const double* src, const double* R1, const double* R2, bool transposed, double* half,
                 double* dst) {
    const QPlan& P = x.P;
    QGemm a = qgemm_plain(src, R2, half, P.n * P.n1, P.n2, P.n2);
    if (transposed) { a.csB = P.n2; a.klB = 1; }
    gemm(x, a);
    QGemm b{};
    b.A = R1; b.B = half; b.C = dst; b.M = P.n1; b.N = P.n2; b.K = P.n1; b.batch = P.n;
    if (transposed) { b.rsA = P.n1; b.klA = 1; } else { b.rsA = 1; b.klA = P.n1; }
    b.bsA = 0; b.csB = 1; b.klB = P.n2; b.bsB = P.m; b.rsC = P.n2; b.bsC = P.m; b.alpha = 1.0; b.beta = 0.0;
    gemm(x, b);
}

// Wres = W - A Bt^T (returns W itself when k == 0)
const double* residual(Ctx& x, const double* W, const double* A, const double* Bt, double* Wres) {
    const QPlan& P = x.P;
    if (P.k == 0) return W;
    QGemm g{};
    g.A = A; g.B = Bt; g.C = Wres; g.C0 = W; g.M = P.n; g.N = P.m; g.K = P.k; g.batch = 1;
    g.rsA = P.k; g.klA = 1; g.csB = P.k; g.klB = 1; g.rsC = P.m; g.alpha = -1.0; g.beta = 1.0;
    gemm(x, g);
    return Wres;
}

// big[1] = W - M (when k > 0), big[2] = half-rotated, big[3] = Y = (W - M) R, X = Y H, ybar
const double* okt(Ctx& x, const double* W, const double* A, const double* Bt, const double* R1, const double* R2,
                  double* X, double* ybar) {
    const QPlan& P = x.P;
    const double* Wres = residual(x, W, A, Bt, x.d(P.big[1]));
    rotate_rows(x, Wres, R1, R2, false, x.d(P.big[2]), x.d(P.big[3]));
    x.ck(bwla_q_launch_center(x.d(P.big[3]), X, ybar, P.n, P.m, x.st));
    return Wres;
}

// Above this size the polar factor comes from the Newton-Schulz iteration (a few dozen small GEMMs on
// the matrix cores) instead of the one-workgroup Jacobi SVD, whose time grows with the cube of the size
// (86: 4 ms, 128: 11 ms, 256: 81 ms).
constexpr int POLAR_JACOBI_MAX = 64;
constexpr int POLAR_NS_PAIRS = 32;

// polar factor of the jn-sized scratch matrix C (nn x nn) into R
void polar(Ctx& x, int nn, double* R) {
    const QPlan& P = x.P;
    if (nn > POLAR_JACOBI_MAX) {
        // X <- X (3 I - X^T X) / 2 from X = C / ||C||_F: singular values in (0, 1] rise to 1 (by 3/2 per
        // step while small, then quadratically), the singular vectors stay: X -> U V^T.  Steps come in
        // pairs so that X is back in the same buffer after each; before a pair X^T X is compared with I,
        // and once it is within 1e-13 the remaining launches return at once.  A singular C never gets
        // there and leaves a finite matrix that is not orthogonal.
        double *Xa = x.d(P.Ws), *Xb = x.d(P.Vs), *G = x.d(P.G);
        int* done = x.done();
        x.ck(bwla_q_launch_set_int(done, 0, x.st));
        x.ck(bwla_q_launch_scale_inv_frob(x.d(P.C), nn * nn, Xa, x.st));
        auto step = [&](const double* src, double* dst) {
            QGemm g = qgemm_plain(src, src, G, nn, nn, nn);       // G = src^T src
            g.rsA = 1; g.klA = nn;
            gemm(x, g, done);
            QGemm u = qgemm_plain(src, G, dst, nn, nn, nn);       // dst = 1.5 src - 0.5 src G
            u.C0 = src; u.alpha = -0.5; u.beta = 1.5;
            gemm(x, u, done);
        };
        for (int it = 0; it < POLAR_NS_PAIRS; ++it) {
            if (it > 0) {
                QGemm g = qgemm_plain(Xa, Xa, G, nn, nn, nn);
                g.rsA = 1; g.klA = nn;
                gemm(x, g, done);
                x.ck(bwla_q_launch_near_identity(G, nn, 1.0e-13, done, x.st));
            }
            step(Xa, Xb);
            step(Xb, Xa);
        }
        x.ck(hipMemcpyAsync(R, Xa, (size_t)nn * nn * sizeof(double), hipMemcpyDeviceToDevice, x.st));
        return;
    }
    QJacobi j{};
    j.G = x.d(P.C); j.n = nn; j.pw = -1.0; j.sig = x.d(P.sig); j.Ws = x.d(P.Ws); j.Vs = x.d(P.Vs); j.work = x.d(P.jwork);
    x.ck(bwla_q_launch_jacobi(j, x.st));
    QGemm g = qgemm_plain(x.d(P.Ws), x.d(P.Vs), R, nn, nn, nn);
    g.rsA = 1; g.klA = nn;
    gemm(x, g);
}

// The Procrustes update of one factor at (Wres, R1, R2, c, s2); expects nothing of the scratch.
void procrustes(Ctx& x, int which, const double* Wres, const double* R1, const double* R2, const double* c,
                const double* s2, double* Rnew) {
    const QPlan& P = x.P;
    double *half = x.d(P.big[2]), *Y = x.d(P.big[3]), *T = x.d(P.big[4]), *ybar = x.d(P.ybar);
    rotate_rows(x, Wres, R1, R2, false, half, Y);
    x.ck(bwla_q_launch_center(Y, nullptr, ybar, P.n, P.m, x.st));
    x.ck(bwla_q_launch_targets(Y, ybar, c, s2, P.n, P.m, T, x.st));
    QGemm g{};
    g.batch = 1; g.alpha = 1.0; g.beta = 0.0; g.C = x.d(P.C);
    if (which == 1) {
        // C1[a][c] = sum_i sum_d (V_i R2)[a][d] (lambda_i T_i)[c][d]
        g.A = half; g.B = T; g.M = P.n1; g.N = P.n1; g.K = P.n * P.n2;
        g.rsA = P.n2; g.kdivA = P.n2; g.khA = P.m; g.klA = 1;
        g.csB = P.n2; g.kdivB = P.n2; g.khB = P.m; g.klB = 1;
        g.rsC = P.n1;
        gemm(x, g);
        polar(x, P.n1, Rnew);
    } else {
        // P_i = R1^T V_i into `half`, then C2[b][d] = sum_(i,c) P[(i,c)][b] (lambda_i T_i)[(i,c)][d]
        QGemm b{};
        b.A = R1; b.B = Wres; b.C = half; b.M = P.n1; b.N = P.n2; b.K = P.n1; b.batch = P.n;
        b.rsA = 1; b.klA = P.n1; b.csB = 1; b.klB = P.n2; b.bsB = P.m; b.rsC = P.n2; b.bsC = P.m; b.alpha = 1.0;
        gemm(x, b);
        g.A = half; g.B = T; g.M = P.n2; g.N = P.n2; g.K = P.n * P.n1;
        g.rsA = 1; g.klA = P.n2; g.csB = 1; g.klB = P.n2; g.rsC = P.n2;
        gemm(x, g);
        polar(x, P.n2, Rnew);
    }
}

// rank-k truncation of Y (n x m) into A2 (n x k), Bt2 (m x k); lam gets the k leading eigenvalues
// of Y^T Y restricted to the block (sigma^2)
void truncate(Ctx& x, const double* Y, int iters, double tol, double* A2, double* Bt2, double* lam) {
    const QPlan& P = x.P;
    const int n = P.n, m = P.m, p = P.p, k = P.k;
    double *Q = x.d(P.Q), *Q2 = x.d(P.Q2), *Zs = x.d(P.Zs), *G = x.d(P.G), *Vs = x.d(P.Vs);
    int* done = x.done();
    x.ck(bwla_q_launch_set_int(done, 0, x.st));
    x.ck(bwla_q_launch_fill_hash(x.d(P.prev), P.jn, 1u, x.st));        // any values: the first comparison only must not stop
    x.ck(bwla_q_launch_fill_hash(Q, (size_t)m * p, 12345u, x.st));
    auto gram = [&](const double* B, int rows, const int* skip) {      // G = B^T B, B rows x p
        QGemm g = qgemm_plain(B, B, G, p, p, rows);
        g.rsA = 1; g.klA = p;
        gemm(x, g, skip);
    };
    auto jac = [&](double pw, bool track, const int* skip) {
        QJacobi j{};
        j.G = G; j.n = p; j.pw = pw; j.sig = x.d(P.sig); j.Vs = Vs; j.Ws = nullptr; j.work = x.d(P.jwork);
        if (track) { j.prev_sig = x.d(P.prev); j.lead = k; j.tol = tol; j.done = done; }
        j.skip = skip;
        j.sym = true;                                       // a Gram matrix
        x.ck(bwla_q_launch_jacobi(j, x.st));
    };
    auto times_vs = [&](const double* B, int rows, int cols, double* out, const int* skip) {   // out = B Vs^T[:, :cols]
        QGemm g = qgemm_plain(B, Vs, out, rows, cols, p);
        g.csB = p; g.klB = 1;
        gemm(x, g, skip);
    };
    if (p > BWLA_Q_JACOBI_SYM_LDS) {
        // Blocks too wide for the one-workgroup eigensolver to hold in LDS (ranks above 68): the block is
        // orthonormalized by the Newton-Schulz iteration X <- X (3 I - X^T X) / 2 instead (tall GEMMs; it
        // converges to the orthogonal polar factor of the block, a basis of the same subspace), there are
        // no Ritz values along the way, so every one of the `iters` iterations runs, and the eigensolver is
        // called once, for the Rayleigh-Ritz step.
        auto ns_ortho = [&](double* src, double* dst) {                 // src is overwritten; result in dst
            x.ck(bwla_q_launch_set_int(done, 0, x.st));
            gram(src, m, nullptr);
            x.ck(bwla_q_launch_gram_inv_norm(G, p, x.d(P.scal), x.st));
            x.ck(bwla_q_launch_scale_by(src, (size_t)m * p, x.d(P.scal), x.st));
            auto step = [&](const double* a, double* b, const int* skip) {
                gram(a, m, skip);
                QGemm u = qgemm_plain(a, G, b, m, p, p);                  // b = 1.5 a - 0.5 a G
                u.C0 = a; u.alpha = -0.5; u.beta = 1.5;
                gemm(x, u, skip);
            };
            step(src, dst, nullptr);
            for (int pair = 0; pair < POLAR_NS_PAIRS; ++pair) {
                gram(dst, m, done);
                x.ck(bwla_q_launch_near_identity(G, p, 1.0e-13, done, x.st));
                step(dst, src, done);
                step(src, dst, done);
            }
        };
        ns_ortho(Q, Q2);
        double* cur = Q2; double* oth = Q;
        for (int it = 0; it < iters; ++it) {
            gemm(x, qgemm_plain(Y, cur, Zs, n, p, m));                   // Zs = Y Q
            QGemm t = qgemm_plain(Y, Zs, oth, m, p, n);                  // oth = Y^T Zs
            t.rsA = 1; t.klA = m;
            gemm(x, t);
            ns_ortho(oth, cur);
        }
        gemm(x, qgemm_plain(Y, cur, Zs, n, p, m));
        gram(Zs, n, nullptr);
        QJacobi j{};
        j.G = G; j.n = p; j.pw = 0.0; j.sig = lam; j.Vs = Vs; j.work = x.d(P.jwork);
        j.sym = true;
        x.ck(bwla_q_launch_jacobi(j, x.st));
        times_vs(Zs, n, k, A2, nullptr);
        times_vs(cur, m, k, Bt2, nullptr);
        return;
    }
    // the start, orthonormalized
    gram(Q, m, nullptr); jac(-0.5, false, nullptr); times_vs(Q, m, p, Q2, nullptr);
    double* cur = Q2; double* oth = Q;
    for (int it = 0; it < iters; ++it) {
        gemm(x, qgemm_plain(Y, cur, Zs, n, p, m), done);                 // Zs = Y Q
        QGemm t = qgemm_plain(Y, Zs, oth, m, p, n);                      // oth = Y^T Zs
        t.rsA = 1; t.klA = m;
        gemm(x, t, done);
        gram(oth, m, done);
        jac(-0.5, true, done);
        // cur <- oth Vs Lambda^(-1/2); when the iteration has converged in this Jacobi call the
        // product is skipped and cur stays the orthonormal block of the previous iteration
        times_vs(oth, m, p, cur, done);
    }
    // one more orthonormalization (the Gram matrix is close to I now), then Rayleigh-Ritz
    gram(cur, m, nullptr); jac(-0.5, false, nullptr); times_vs(cur, m, p, oth, nullptr);
    gemm(x, qgemm_plain(Y, oth, Zs, n, p, m));
    gram(Zs, n, nullptr);
    {
        QJacobi j{};
        j.G = G; j.n = p; j.pw = 0.0; j.sig = lam; j.Vs = Vs; j.work = x.d(P.jwork);
        j.sym = true;
        x.ck(bwla_q_launch_jacobi(j, x.st));
    }
    times_vs(Zs, n, k, A2, nullptr);
    times_vs(oth, m, k, Bt2, nullptr);
}

// M <- truncation of M - (1/mu) dL/dM; A, Bt in place.  Leaves the scratch's big arrays stale.
void psp(Ctx& x, const double* W, double* A, double* Bt, const double* R1, const double* R2, const double* c,
         const double* s2, double mu, int iters, double tol, double* lam) {
    const QPlan& P = x.P;
    double *half = x.d(P.big[2]), *Y = x.d(P.big[3]), *X = x.d(P.big[4]), *fac = x.d(P.scal);
    okt(x, W, A, Bt, R1, R2, X, nullptr);
    x.ck(bwla_q_launch_prox_factor(s2, P.n, P.m, mu, fac, x.st));
    x.ck(bwla_q_launch_gradx(X, c, s2, fac, P.n, P.m, Y, x.st));          // Y <- (G_X H) / mu, sign folded in
    rotate_rows(x, Y, R1, R2, true, half, Y);                             // back through R^T
    QGemm g{};                                                            // Y <- Y + A Bt^T: the proximal point
    g.A = A; g.B = Bt; g.C = Y; g.C0 = Y; g.M = P.n; g.N = P.m; g.K = P.k; g.batch = 1;
    g.rsA = P.k; g.klA = 1; g.csB = P.k; g.klB = 1; g.rsC = P.m; g.alpha = 1.0; g.beta = 1.0;
    gemm(x, g);
    truncate(x, Y, iters, tol, x.d(P.A2), x.d(P.Bt2), lam);
    x.ck(hipMemcpyAsync(A, x.d(P.A2), (size_t)P.n * P.k * sizeof(double), hipMemcpyDeviceToDevice, x.st));
    x.ck(hipMemcpyAsync(Bt, x.d(P.Bt2), (size_t)P.m * P.k * sizeof(double), hipMemcpyDeviceToDevice, x.st));
}

bwla_status_t open_ctx(Ctx& x, int64_t n, int64_t m, int32_t n1, int32_t n2, int32_t k, void* d_ws, size_t ws_bytes,
                       void* stream) {
    const bwla_status_t s = make_plan(n, m, n1, n2, k, x.P);
    if (s != BWLA_OK) return s;
    if (!d_ws) return BWLA_ERR_NULL;
    if (!aligned16(d_ws)) return BWLA_ERR_ALIGN;
    if (ws_bytes < x.P.bytes) return BWLA_ERR_BUFSIZE;
    x.ws = static_cast<char*>(d_ws);
    x.st = static_cast<hipStream_t>(stream);
    return BWLA_OK;
}
inline bwla_status_t finish(const Ctx& x) { return x.err == hipSuccess ? BWLA_OK : BWLA_ERR_HIP; }

}  // namespace

extern "C" {

bwla_status_t bwla_quantizer_workspace_size(int64_t n, int64_t m, int32_t n1, int32_t n2, int32_t k, size_t* bytes) {
    if (!bytes) return BWLA_ERR_NULL;
    QPlan P;
    const bwla_status_t s = make_plan(n, m, n1, n2, k, P);
    if (s != BWLA_OK) return s;
    *bytes = P.bytes;
    return BWLA_OK;
}

bwla_status_t bwla_q_okt_rows(const double* d_W, const double* d_A, const double* d_Bt, int32_t k, const double* d_R1,
                              const double* d_R2, int64_t n, int64_t m, int32_t n1, int32_t n2, double* d_X,
                              double* d_ybar, void* d_ws, size_t ws_bytes, void* stream) {
    if (!d_W || !d_R1 || !d_R2 || !d_X) return BWLA_ERR_NULL;
    if (k > 0 && (!d_A || !d_Bt)) return BWLA_ERR_NULL;
    if (!aligned16(d_W) || !aligned16(d_A) || !aligned16(d_Bt) || !aligned16(d_R1) || !aligned16(d_R2) ||
        !aligned16(d_X) || !aligned16(d_ybar))
        return BWLA_ERR_ALIGN;
    Ctx x;
    const bwla_status_t s = open_ctx(x, n, m, n1, n2, k, d_ws, ws_bytes, stream);
    if (s != BWLA_OK) return s;
    okt(x, d_W, d_A, d_Bt, d_R1, d_R2, d_X, d_ybar);
    return finish(x);
}

static bwla_status_t check_rows(const double* d_X, int64_t n, int64_t m, const double* d_c, const double* d_s2) {
    if (!d_X || !d_c || !d_s2) return BWLA_ERR_NULL;
    if (n <= 0 || m <= 0) return BWLA_ERR_SHAPE;
    if (n > 65535 || m > 65536) return BWLA_ERR_UNSUPPORTED;
    if (!aligned16(d_X) || !aligned16(d_c) || !aligned16(d_s2)) return BWLA_ERR_ALIGN;
    return BWLA_OK;
}

bwla_status_t bwla_q_init_theta(const double* d_X, int64_t n, int64_t m, double s2_min, double* d_c, double* d_s2,
                                void* stream) {
    const bwla_status_t s = check_rows(d_X, n, m, d_c, d_s2);
    if (s != BWLA_OK) return s;
    return bwla_q_launch_init_theta(d_X, (int)n, (int)m, s2_min, d_c, d_s2, static_cast<hipStream_t>(stream)) == hipSuccess
               ? BWLA_OK : BWLA_ERR_HIP;
}

bwla_status_t bwla_q_em_step(const double* d_X, int64_t n, int64_t m, double s2_min, double* d_c, double* d_s2,
                             void* stream) {
    const bwla_status_t s = check_rows(d_X, n, m, d_c, d_s2);
    if (s != BWLA_OK) return s;
    return bwla_q_launch_em(d_X, (int)n, (int)m, s2_min, d_c, d_s2, static_cast<hipStream_t>(stream)) == hipSuccess
               ? BWLA_OK : BWLA_ERR_HIP;
}

bwla_status_t bwla_q_gmm_nll(const double* d_X, int64_t n, int64_t m, const double* d_c, const double* d_s2,
                             double* d_out, void* d_ws, size_t ws_bytes, void* stream) {
    const bwla_status_t s = check_rows(d_X, n, m, d_c, d_s2);
    if (s != BWLA_OK) return s;
    if (!d_out || !d_ws) return BWLA_ERR_NULL;
    if (!aligned16(d_ws)) return BWLA_ERR_ALIGN;
    if (ws_bytes < (size_t)n * sizeof(double)) return BWLA_ERR_BUFSIZE;
    return bwla_q_launch_nll(d_X, (int)n, (int)m, d_c, d_s2, static_cast<double*>(d_ws), d_out,
                             static_cast<hipStream_t>(stream)) == hipSuccess ? BWLA_OK : BWLA_ERR_HIP;
}

bwla_status_t bwla_q_procrustes(int32_t which, const double* d_Wres, const double* d_R1, const double* d_R2,
                                const double* d_c, const double* d_s2, int64_t n, int64_t m, int32_t n1, int32_t n2,
                                double* d_Rnew, void* d_ws, size_t ws_bytes, void* stream) {
    if (!d_Wres || !d_R1 || !d_R2 || !d_c || !d_s2 || !d_Rnew) return BWLA_ERR_NULL;
    if (which != 1 && which != 2) return BWLA_ERR_SHAPE;
    if (!aligned16(d_Wres) || !aligned16(d_R1) || !aligned16(d_R2) || !aligned16(d_c) || !aligned16(d_s2) ||
        !aligned16(d_Rnew))
        return BWLA_ERR_ALIGN;
    Ctx x;
    const bwla_status_t s = open_ctx(x, n, m, n1, n2, 0, d_ws, ws_bytes, stream);
    if (s != BWLA_OK) return s;
    procrustes(x, which, d_Wres, d_R1, d_R2, d_c, d_s2, d_Rnew);
    return finish(x);
}

bwla_status_t bwla_q_svd_square(const double* d_G, int32_t nn, double* d_sig, double* d_Ut, double* d_Vt, void* d_ws,
                                size_t ws_bytes, void* stream) {
    if (!d_G || !d_ws) return BWLA_ERR_NULL;
    if (nn <= 0) return BWLA_ERR_SHAPE;
    if (nn > 256) return BWLA_ERR_UNSUPPORTED;
    if (!aligned16(d_G) || !aligned16(d_sig) || !aligned16(d_Ut) || !aligned16(d_Vt) || !aligned16(d_ws))
        return BWLA_ERR_ALIGN;
    if (ws_bytes < (size_t)2 * nn * nn * sizeof(double)) return BWLA_ERR_BUFSIZE;
    QJacobi j{};
    j.G = d_G; j.n = nn; j.pw = 0.0; j.sig = d_sig; j.Ws = d_Ut; j.Vs = d_Vt; j.work = static_cast<double*>(d_ws);
    return bwla_q_launch_jacobi(j, static_cast<hipStream_t>(stream)) == hipSuccess ? BWLA_OK : BWLA_ERR_HIP;
}

bwla_status_t bwla_q_truncate_rank(const double* d_Y, int64_t n, int64_t m, int32_t k, int32_t iters, double tol,
                                   double* d_A, double* d_Bt, double* d_sig, void* d_ws, size_t ws_bytes,
                                   void* stream) {
    if (!d_Y || !d_A || !d_Bt) return BWLA_ERR_NULL;
    if (k <= 0 || iters < 0) return BWLA_ERR_SHAPE;
    if (!aligned16(d_Y) || !aligned16(d_A) || !aligned16(d_Bt) || !aligned16(d_sig)) return BWLA_ERR_ALIGN;
    Ctx x;
    const bwla_status_t s = open_ctx(x, n, m, 1, 1, k, d_ws, ws_bytes, stream);   // no factors
    if (s != BWLA_OK) return s;
    truncate(x, d_Y, iters, tol, d_A, d_Bt, x.d(x.P.lam));
    if (d_sig) x.ck(bwla_q_launch_pow_vec(x.d(x.P.lam), 0.5, k, d_sig, x.st));
    return finish(x);
}

bwla_status_t bwla_q_psp_step(const double* d_W, double* d_A, double* d_Bt, int32_t k, const double* d_R1,
                              const double* d_R2, const double* d_c, const double* d_s2, int64_t n, int64_t m,
                              int32_t n1, int32_t n2, double mu, int32_t iters, double tol, void* d_ws, size_t ws_bytes,
                              void* stream) {
    if (!d_W || !d_A || !d_Bt || !d_R1 || !d_R2 || !d_c || !d_s2) return BWLA_ERR_NULL;
    if (k <= 0 || iters < 0) return BWLA_ERR_SHAPE;
    if (!aligned16(d_W) || !aligned16(d_A) || !aligned16(d_Bt) || !aligned16(d_R1) || !aligned16(d_R2) ||
        !aligned16(d_c) || !aligned16(d_s2))
        return BWLA_ERR_ALIGN;
    Ctx x;
    const bwla_status_t s = open_ctx(x, n, m, n1, n2, k, d_ws, ws_bytes, stream);
    if (s != BWLA_OK) return s;
    psp(x, d_W, d_A, d_Bt, d_R1, d_R2, d_c, d_s2, mu, iters, tol, x.d(x.P.lam));
    return finish(x);
}

bwla_status_t bwla_quantize_layer(const float* d_W, int64_t n, int64_t m, int32_t n1, int32_t n2, int32_t k,
                                  int32_t t_outer, double mu, double s2_min, int32_t svd_iters, double svd_tol,
                                  int32_t init_identity, float* d_R1, float* d_R2, float* d_W_rot, float* d_U,
                                  float* d_V, double* d_c, double* d_s2, double* d_hist, void* d_ws, size_t ws_bytes,
                                  void* stream) {
    if (!d_W || !d_R1 || !d_R2 || !d_W_rot) return BWLA_ERR_NULL;
    if (k > 0 && (!d_U || !d_V)) return BWLA_ERR_NULL;
    if (t_outer < 0 || svd_iters < 0 || !(s2_min > 0.0)) return BWLA_ERR_SHAPE;
    if (!aligned16(d_W) || !aligned16(d_R1) || !aligned16(d_R2) || !aligned16(d_W_rot) || !aligned16(d_U) ||
        !aligned16(d_V) || !aligned16(d_c) || !aligned16(d_s2) || !aligned16(d_hist))
        return BWLA_ERR_ALIGN;
    Ctx x;
    const bwla_status_t s = open_ctx(x, n, m, n1, n2, k, d_ws, ws_bytes, stream);
    if (s != BWLA_OK) return s;
    const QPlan& P = x.P;
    const size_t nm = (size_t)P.n * P.m;
    double *W = x.d(P.big[0]), *Y = x.d(P.big[3]), *X = x.d(P.big[4]);
    double *R1 = x.d(P.R1), *R2 = x.d(P.R2), *A = x.d(P.A), *Bt = x.d(P.Bt), *ybar = x.d(P.ybar);
    double* c = d_c ? d_c : x.d(P.c);
    double* s2 = d_s2 ? d_s2 : x.d(P.s2);
    double* lam = x.d(P.lam);
    double* rowpart = x.d(P.rowpart);
    double* hist_sink = x.d(P.scal) + 8;
    int hi = 0;
    auto record = [&]() {               // L_GMM of the centered rows in X
        x.ck(bwla_q_launch_nll(X, P.n, P.m, c, s2, rowpart, d_hist ? d_hist + hi : hist_sink, x.st));
        ++hi;
    };
    x.ck(bwla_q_launch_convert_f32_f64(d_W, W, nm, x.st));
    if (init_identity) {
        x.ck(bwla_q_launch_fill_identity(R1, n1, x.st));
        x.ck(bwla_q_launch_fill_identity(R2, n2, x.st));
    } else {
        x.ck(bwla_q_launch_convert_f32_f64(d_R1, R1, (size_t)n1 * n1, x.st));
        x.ck(bwla_q_launch_convert_f32_f64(d_R2, R2, (size_t)n2 * n2, x.st));
    }
    if (k > 0) {                        // M = 0
        x.ck(bwla_q_launch_fill_value(A, (size_t)P.n * k, 0.0, x.st));
        x.ck(bwla_q_launch_fill_value(Bt, (size_t)P.m * k, 0.0, x.st));
        x.ck(bwla_q_launch_fill_value(lam, k, 0.0, x.st));
    }
    const double* Wres = okt(x, W, A, Bt, R1, R2, X, ybar);
    x.ck(bwla_q_launch_init_theta(X, P.n, P.m, s2_min, c, s2, x.st));
    record();
    for (int t = 0; t < t_outer; ++t) {
        // X holds the centered rows at the current M, R1, R2
        x.ck(bwla_q_launch_em(X, P.n, P.m, s2_min, c, s2, x.st));
        record();
        if (k > 0) {
            psp(x, W, A, Bt, R1, R2, c, s2, mu, svd_iters, svd_tol, lam);
            Wres = okt(x, W, A, Bt, R1, R2, X, ybar);
        }
        record();
        procrustes(x, 1, Wres, R1, R2, c, s2, R1);
        procrustes(x, 2, Wres, R1, R2, c, s2, R2);
        Wres = okt(x, W, A, Bt, R1, R2, X, ybar);
        record();
    }
    // Y = (W - M)(R1 (x) R2) at the final factors
    x.ck(bwla_q_launch_convert_f64_f32(Y, d_W_rot, nm, x.st));
    x.ck(bwla_q_launch_convert_f64_f32(R1, d_R1, (size_t)n1 * n1, x.st));
    x.ck(bwla_q_launch_convert_f64_f32(R2, d_R2, (size_t)n2 * n2, x.st));
    if (k > 0) {
        // A = U_k S_k, Bt = V_k, lam = S_k^2: balanced factors V = U_k S_k^(1/2), U = V_k S_k^(1/2)
        x.ck(bwla_q_launch_scale_cols_f32(A, lam, -0.25, P.n, k, d_V, x.st));
        x.ck(bwla_q_launch_scale_cols_f32(Bt, lam, 0.25, P.m, k, d_U, x.st));
    }
    return finish(x);
}

}  // extern "C"
