/*
 * K-FAC preconditioner step: plain fp64 CPU oracle.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct statement
 * of what the K-FAC hot path computes, written from the paper (arXiv 2007.00784,
 * "Convolutional Neural Network Training with Distributed K-FAC").  It shares no
 * code with the HIP library and must never be linked into or called from the
 * product path; only tests, the smoke check and the benchmark's CPU-baseline leg
 * use it.
 *
 * Every routine works on row-major double arrays supplied by the caller.
 * OpenMP is used only to spread independent outputs over host cores; the
 * arithmetic of each output element is the plain definition.
 *
 * Parity pins (see tests): kron <- the paper's printed 2x2 (x) 3x2 example;
 * unfold <- direct convolution, adjoint identity, hand-computed cases;
 * gram/ema <- closed forms and invariants; eigh <- closed-form spectra,
 * constructed matrices, LAPACK cross-check; precondition <- brute-force
 * inversion of the damped Kronecker product and the undamped two-solve identity
 * of Sec. II-C.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>
#include <stdint.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------------
 * Kronecker product, Sec. II-C definition: (A (x) B) is the block matrix whose
 * (i,j) block is a_ij * B.  A is m x n, B is p x q, out is (m*p) x (n*q).
 * ---------------------------------------------------------------------- */
void oracle_kron(const double *A, int m, int n, const double *B, int p, int q, double *out)
{
    const int64_t ld = (int64_t)n * q;
    for (int i = 0; i < m; ++i)
        for (int j = 0; j < n; ++j)
            for (int k = 0; k < p; ++k)
                for (int l = 0; l < q; ++l)
                    out[((int64_t)i * p + k) * ld + ((int64_t)j * q + l)] = A[i * n + j] * B[k * q + l];
}

/* ------------------------------------------------------------------------
 * Unfold of a convolution input (the paper supports Conv2D layers, Sec. V, and
 * defers the construction to the Kronecker-factored-convolution work it cites):
 * every output location of every example becomes one sample row holding the
 * receptive field it sees.
 *   x : [N][C][H][W]
 *   P : [N*Ho*Wo][C*kh*kw], P[(n,ho,wo)][(c,ky,kx)] = x[n][c][ho*sh-ph+ky][wo*sw-pw+kx]
 * with zero outside the image.  Column order (c,ky,kx) is the row-major
 * flattening of a [C_out][C][kh][kw] weight, so the columns of the A factor
 * line up with the columns of the reshaped weight gradient.
 * ---------------------------------------------------------------------- */
void oracle_unfold(const double *x, int N, int C, int H, int W, int kh, int kw,
                   int sh, int sw, int ph, int pw, double *P)
{
    const int Ho = (H + 2 * ph - kh) / sh + 1;
    const int Wo = (W + 2 * pw - kw) / sw + 1;
    const int64_t d = (int64_t)C * kh * kw;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int ho = 0; ho < Ho; ++ho)
            for (int wo = 0; wo < Wo; ++wo) {
                double *row = P + (((int64_t)n * Ho + ho) * Wo + wo) * d;
                for (int c = 0; c < C; ++c)
                    for (int ky = 0; ky < kh; ++ky)
                        for (int kx = 0; kx < kw; ++kx) {
                            const int h = ho * sh - ph + ky;
                            const int w = wo * sw - pw + kx;
                            double v = 0.0;
                            if (h >= 0 && h < H && w >= 0 && w < W)
                                v = x[(((int64_t)n * C + c) * H + h) * W + w];
                            row[((int64_t)c * kh + ky) * kw + kx] = v;
                        }
            }
}

/* ------------------------------------------------------------------------
 * Kronecker factor of one mini-batch (Sec. II-C: A = a a^T, G = g g^T, taken
 * over the sample rows):
 *   Fb[i][j] = scale * sum_r Xt[r][i] * Xt[r][j],   Xt = [X | 1] if append_ones.
 *   X : [R][d] row-major.  Fb : [D][D], D = d + append_ones, full symmetric.
 * ---------------------------------------------------------------------- */
void oracle_gram(const double *X, int64_t R, int d, int append_ones, double scale, double *Fb)
{
    const int D = d + (append_ones ? 1 : 0);
    /* column-contiguous copy so that each entry is a plain dot product */
    double *cols = (double *)malloc(sizeof(double) * (size_t)D * (size_t)R);
    for (int i = 0; i < D; ++i)
        for (int64_t r = 0; r < R; ++r)
            cols[(int64_t)i * R + r] = (i < d) ? X[r * d + i] : 1.0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int i = 0; i < D; ++i)
        for (int j = 0; j <= i; ++j) {
            const double *a = cols + (int64_t)i * R, *b = cols + (int64_t)j * R;
            double s = 0.0;
#pragma omp simd reduction(+ : s)
            for (int64_t r = 0; r < R; ++r)
                s += a[r] * b[r];
            Fb[(int64_t)i * D + j] = scale * s;
            Fb[(int64_t)j * D + i] = scale * s;
        }
    free(cols);
}

/* One entry of the batch factor, for spot checks at sizes where the full
 * matrix is too slow: scale * sum_r Xt[r][i]*Xt[r][j]. */
double oracle_gram_entry(const double *X, int64_t R, int d, int append_ones, double scale, int i, int j)
{
    (void)append_ones;
    double s = 0.0;
    for (int64_t r = 0; r < R; ++r) {
        const double a = (i < d) ? X[r * d + i] : 1.0;
        const double b = (j < d) ? X[r * d + j] : 1.0;
        s += a * b;
    }
    return scale * s;
}

/* One entry of the batch A factor of a conv layer without materialising the patch matrix, for spot
 * checks at full size: scale * sum over examples and output locations of Pt[r][i] * Pt[r][j], where
 * Pt[r][c] is the unfold entry defined above for c < C*kh*kw and the constant 1 for c == C*kh*kw. */
static double patch_value(const double *x, int C, int H, int W, int kh, int kw, int sh, int sw, int ph, int pw,
                          int n, int ho, int wo, int col)
{
    if (col == C * kh * kw) return 1.0;
    const int c = col / (kh * kw), ky = (col / kw) % kh, kx = col % kw;
    const int h = ho * sh - ph + ky, w = wo * sw - pw + kx;
    if (h < 0 || h >= H || w < 0 || w >= W) return 0.0;
    return x[(((int64_t)n * C + c) * H + h) * W + w];
}

double oracle_conv_factor_entry(const double *x, int N, int C, int H, int W, int kh, int kw,
                                int sh, int sw, int ph, int pw, double scale, int i, int j)
{
    const int Ho = (H + 2 * ph - kh) / sh + 1;
    const int Wo = (W + 2 * pw - kw) / sw + 1;
    double s = 0.0;
    for (int n = 0; n < N; ++n)
        for (int ho = 0; ho < Ho; ++ho)
            for (int wo = 0; wo < Wo; ++wo)
                s += patch_value(x, C, H, W, kh, kw, sh, sw, ph, pw, n, ho, wo, i) *
                     patch_value(x, C, H, W, kh, kw, sh, sw, ph, pw, n, ho, wo, j);
    return scale * s;
}

/* ------------------------------------------------------------------------
 * Running average of a factor (Sec. IV-B): F <- xi * F + (1 - xi) * Fb,
 * xi the weight of the history (see the design notes for the reading of the
 * printed equation).  n = number of elements.
 * ---------------------------------------------------------------------- */
void oracle_ema(double *F, const double *Fb, int64_t n, double xi)
{
    for (int64_t i = 0; i < n; ++i)
        F[i] = xi * F[i] + (1.0 - xi) * Fb[i];
}

/* ------------------------------------------------------------------------
 * Symmetric eigendecomposition F = Q diag(lam) Q^T (Sec. IV-A), lam ascending,
 * eigenvectors in the columns of Q (row-major storage).  Two textbook methods.
 * ---------------------------------------------------------------------- */

static void sort_eigenpairs(int n, double *lam, const double *vec_rows, double *Q)
{
    /* vec_rows[k][:] is the eigenvector of lam[k]; selection sort by value,
     * then write vectors into the columns of Q. */
    int *idx = (int *)malloc(sizeof(int) * (size_t)n);
    double *tmp = (double *)malloc(sizeof(double) * (size_t)n);
    for (int i = 0; i < n; ++i) idx[i] = i;
    for (int i = 0; i < n; ++i) {
        int best = i;
        for (int j = i + 1; j < n; ++j)
            if (lam[idx[j]] < lam[idx[best]]) best = j;
        int t = idx[i]; idx[i] = idx[best]; idx[best] = t;
    }
    for (int i = 0; i < n; ++i) tmp[i] = lam[idx[i]];
    memcpy(lam, tmp, sizeof(double) * (size_t)n);
    for (int k = 0; k < n; ++k) {
        const double *v = vec_rows + (int64_t)idx[k] * n;
        for (int i = 0; i < n; ++i) Q[(int64_t)i * n + k] = v[i];
    }
    free(idx);
    free(tmp);
}

/* Cyclic two-sided Jacobi: repeatedly annihilate S[p][q] with a plane rotation
 * chosen from the 2x2 symmetric Schur decomposition, row-cyclic order, until
 * the off-diagonal Frobenius norm is below 1e-15 of the matrix norm.
 * Returns the number of sweeps used, or -1 if 60 sweeps did not suffice. */
int oracle_eigh_jacobi(const double *F, int n, double *Q, double *lam)
{
    double *S = (double *)malloc(sizeof(double) * (size_t)n * n);
    double *Vt = (double *)calloc((size_t)n * n, sizeof(double)); /* rows = vectors */
    memcpy(S, F, sizeof(double) * (size_t)n * n);
    for (int i = 0; i < n; ++i) Vt[(int64_t)i * n + i] = 1.0;
    double fro2 = 0.0;
    for (int64_t i = 0; i < (int64_t)n * n; ++i) fro2 += S[i] * S[i];
    int sweeps = -1;
    for (int sweep = 0; sweep < 60; ++sweep) {
        double off2 = 0.0;
        for (int i = 0; i < n; ++i)
            for (int j = 0; j < n; ++j)
                if (i != j) off2 += S[(int64_t)i * n + j] * S[(int64_t)i * n + j];
        if (off2 <= 1e-30 * fro2) { sweeps = sweep; break; }
        for (int p = 0; p < n - 1; ++p)
            for (int q = p + 1; q < n; ++q) {
                const double apq = S[(int64_t)p * n + q];
                if (apq == 0.0) continue;
                const double app = S[(int64_t)p * n + p], aqq = S[(int64_t)q * n + q];
                /* tan of the rotation angle: smaller root of t^2 + 2*theta*t - 1 = 0 */
                const double theta = (aqq - app) / (2.0 * apq);
                const double t = (theta >= 0.0 ? 1.0 : -1.0) / (fabs(theta) + sqrt(theta * theta + 1.0));
                const double c = 1.0 / sqrt(t * t + 1.0), s = t * c;
                /* S <- J^T S J with J = [[c, s], [-s, c]] in the (p,q) plane */
                for (int k = 0; k < n; ++k) { /* columns p,q */
                    const double skp = S[(int64_t)k * n + p], skq = S[(int64_t)k * n + q];
                    S[(int64_t)k * n + p] = c * skp - s * skq;
                    S[(int64_t)k * n + q] = s * skp + c * skq;
                }
                for (int k = 0; k < n; ++k) { /* rows p,q */
                    const double spk = S[(int64_t)p * n + k], sqk = S[(int64_t)q * n + k];
                    S[(int64_t)p * n + k] = c * spk - s * sqk;
                    S[(int64_t)q * n + k] = s * spk + c * sqk;
                }
                for (int k = 0; k < n; ++k) { /* V <- V J, stored transposed */
                    const double vp = Vt[(int64_t)p * n + k], vq = Vt[(int64_t)q * n + k];
                    Vt[(int64_t)p * n + k] = c * vp - s * vq;
                    Vt[(int64_t)q * n + k] = s * vp + c * vq;
                }
            }
    }
    for (int i = 0; i < n; ++i) lam[i] = S[(int64_t)i * n + i];
    sort_eigenpairs(n, lam, Vt, Q);
    free(S);
    free(Vt);
    return sweeps;
}

/* Householder reduction to tridiagonal form followed by the implicitly shifted
 * QR iteration (Wilkinson shift) on the tridiagonal matrix, with all
 * transformations accumulated.  Returns 0, or -1 if the iteration cap is hit. */
int oracle_eigh_tridiag(const double *F, int n, double *Q, double *lam)
{
    double *S = (double *)malloc(sizeof(double) * (size_t)n * n);
    double *Zt = (double *)calloc((size_t)n * n, sizeof(double)); /* rows = vectors */
    double *v = (double *)malloc(sizeof(double) * (size_t)n);
    double *p = (double *)malloc(sizeof(double) * (size_t)n);
    double *w = (double *)malloc(sizeof(double) * (size_t)n);
    double *dg = (double *)malloc(sizeof(double) * (size_t)n);
    double *e = (double *)calloc((size_t)n, sizeof(double));
    double *rc = (double *)malloc(sizeof(double) * (size_t)n);
    double *rs = (double *)malloc(sizeof(double) * (size_t)n);
    memcpy(S, F, sizeof(double) * (size_t)n * n);
    for (int i = 0; i < n; ++i) Zt[(int64_t)i * n + i] = 1.0;

    /* --- T = H_{n-3} ... H_0 S H_0 ... H_{n-3},  H_k = I - beta v v^T --- */
    for (int k = 0; k + 2 < n; ++k) {
        const int m = n - k - 1; /* length of the column below the diagonal */
        double sigma = 0.0;
        for (int i = 1; i < m; ++i) sigma += S[(int64_t)(k + 1 + i) * n + k] * S[(int64_t)(k + 1 + i) * n + k];
        const double x0 = S[(int64_t)(k + 1) * n + k];
        if (sigma == 0.0) continue; /* column already in tridiagonal form */
        const double norm = sqrt(x0 * x0 + sigma);
        const double alpha = (x0 > 0.0) ? -norm : norm; /* reflected value, sign avoids cancellation */
        v[0] = x0 - alpha;
        for (int i = 1; i < m; ++i) v[i] = S[(int64_t)(k + 1 + i) * n + k];
        double vtv = v[0] * v[0] + sigma;
        const double beta = 2.0 / vtv;
        /* p = beta * S22 v */
#pragma omp parallel for schedule(static)
        for (int i = 0; i < m; ++i) {
            const double *row = S + (int64_t)(k + 1 + i) * n + (k + 1);
            double s = 0.0;
            for (int j = 0; j < m; ++j) s += row[j] * v[j];
            p[i] = beta * s;
        }
        double ptv = 0.0;
        for (int i = 0; i < m; ++i) ptv += p[i] * v[i];
        for (int i = 0; i < m; ++i) w[i] = p[i] - 0.5 * beta * ptv * v[i];
        /* S22 <- S22 - v w^T - w v^T */
#pragma omp parallel for schedule(static)
        for (int i = 0; i < m; ++i) {
            double *row = S + (int64_t)(k + 1 + i) * n + (k + 1);
            for (int j = 0; j < m; ++j) row[j] -= v[i] * w[j] + w[i] * v[j];
        }
        S[(int64_t)(k + 1) * n + k] = alpha;
        S[(int64_t)k * n + (k + 1)] = alpha;
        for (int i = 1; i < m; ++i) {
            S[(int64_t)(k + 1 + i) * n + k] = 0.0;
            S[(int64_t)k * n + (k + 1 + i)] = 0.0;
        }
        /* Zt <- H_k Zt (rows k+1.. of Zt), so that finally Zt = (H_0 H_1 ...)^T */
#pragma omp parallel for schedule(static)
        for (int j = 0; j < n; ++j) {
            double s = 0.0;
            for (int i = 0; i < m; ++i) s += v[i] * Zt[(int64_t)(k + 1 + i) * n + j];
            s *= beta;
            for (int i = 0; i < m; ++i) Zt[(int64_t)(k + 1 + i) * n + j] -= v[i] * s;
        }
    }
    for (int i = 0; i < n; ++i) dg[i] = S[(int64_t)i * n + i];
    for (int i = 0; i + 1 < n; ++i) e[i] = S[(int64_t)i * n + i + 1];

    /* --- implicit QR on the tridiagonal (dg, e) --- */
    const double eps = 2.220446049250313e-16;
    int status = 0;
    int hi = n - 1;
    int64_t iter = 0;
    const int64_t iter_cap = 80LL * n + 100;
    while (hi > 0) {
        /* deflate negligible couplings */
        for (int i = 0; i < hi; ++i)
            if (fabs(e[i]) <= eps * (fabs(dg[i]) + fabs(dg[i + 1]))) e[i] = 0.0;
        if (e[hi - 1] == 0.0) { --hi; continue; }
        int lo = hi - 1;
        while (lo > 0 && e[lo - 1] != 0.0) --lo;
        if (++iter > iter_cap) { status = -1; break; }
        /* Wilkinson shift from the trailing 2x2 of the block [lo..hi] */
        const double delta = 0.5 * (dg[hi - 1] - dg[hi]);
        const double eh = e[hi - 1];
        const double denom = delta + (delta >= 0.0 ? 1.0 : -1.0) * sqrt(delta * delta + eh * eh);
        const double mu = dg[hi] - (denom != 0.0 ? eh * eh / denom : 0.0);
        double x = dg[lo] - mu, z = e[lo];
        int nrot = 0;
        for (int k = lo; k < hi; ++k) {
            /* rotation R = [[c,-s],[s,c]] in plane (k,k+1) with R^T [x;z] = [r;0] */
            const double r = hypot(x, z);
            double c = 1.0, s = 0.0;
            if (r != 0.0) { c = x / r; s = z / r; }
            if (k > lo) e[k - 1] = r;
            const double a = dg[k], b = e[k], g = dg[k + 1];
            dg[k] = c * c * a + 2.0 * c * s * b + s * s * g;
            dg[k + 1] = s * s * a - 2.0 * c * s * b + c * c * g;
            e[k] = (c * c - s * s) * b + c * s * (g - a);
            if (k + 1 < hi) {
                z = s * e[k + 1]; /* the bulge at (k, k+2) */
                e[k + 1] = c * e[k + 1];
                x = e[k];
            }
            rc[nrot] = c; rs[nrot] = s; ++nrot;
        }
        /* Z <- Z R_lo R_lo+1 ...  ==  rotate rows (k,k+1) of Zt in sequence */
#pragma omp parallel
        {
#ifdef _OPENMP
            const int nt = omp_get_num_threads(), tid = omp_get_thread_num();
#else
            const int nt = 1, tid = 0;
#endif
            const int j0 = (int)((int64_t)n * tid / nt), j1 = (int)((int64_t)n * (tid + 1) / nt);
            for (int t = 0; t < nrot; ++t) {
                double *ra = Zt + (int64_t)(lo + t) * n, *rb = ra + n;
                const double c = rc[t], s = rs[t];
                for (int j = j0; j < j1; ++j) {
                    const double za = ra[j], zb = rb[j];
                    ra[j] = c * za + s * zb;
                    rb[j] = -s * za + c * zb;
                }
            }
        }
    }
    for (int i = 0; i < n; ++i) lam[i] = dg[i];
    sort_eigenpairs(n, lam, Zt, Q);
    free(S); free(Zt); free(v); free(p); free(w); free(dg); free(e); free(rc); free(rs);
    return status;
}

/* Dispatcher used by the tests and the baseline: Jacobi for small factors,
 * tridiagonal QR above (Jacobi in plain CPU code is hours at d ~ 4600). */
int oracle_eigh(const double *F, int n, double *Q, double *lam)
{
    if (n <= 96) return oracle_eigh_jacobi(F, n, Q, lam) < 0 ? -1 : 0;
    return oracle_eigh_tridiag(F, n, Q, lam);
}

/* ------------------------------------------------------------------------
 * Eigenbasis preconditioning, Eqs. (v1), (v2), (kfac-eigen) of Sec. IV-A:
 *   V1 = QG^T grad QA;  V2 = V1 / (lamG lamA^T + gamma);  out = QG V2 QA^T.
 * grad, out: [dG][dA] row-major.  Eigenvalues of the PSD factors are clamped at
 * zero before use (a no-op in exact arithmetic).
 * ---------------------------------------------------------------------- */
void oracle_precondition(const double *QA, const double *lamA, int dA,
                         const double *QG, const double *lamG, int dG,
                         double gamma, const double *grad, double *out)
{
    double *T = (double *)malloc(sizeof(double) * (size_t)dG * dA);
    double *V = (double *)malloc(sizeof(double) * (size_t)dG * dA);
    /* T = QG^T grad */
#pragma omp parallel for schedule(static)
    for (int i = 0; i < dG; ++i)
        for (int j = 0; j < dA; ++j) {
            double s = 0.0;
            for (int k = 0; k < dG; ++k) s += QG[(int64_t)k * dG + i] * grad[(int64_t)k * dA + j];
            T[(int64_t)i * dA + j] = s;
        }
    /* V = (T QA) / (lamG lamA^T + gamma) */
#pragma omp parallel for schedule(static)
    for (int i = 0; i < dG; ++i)
        for (int j = 0; j < dA; ++j) {
            double s = 0.0;
            for (int k = 0; k < dA; ++k) s += T[(int64_t)i * dA + k] * QA[(int64_t)k * dA + j];
            const double lg = lamG[i] > 0.0 ? lamG[i] : 0.0, la = lamA[j] > 0.0 ? lamA[j] : 0.0;
            V[(int64_t)i * dA + j] = s / (lg * la + gamma);
        }
    /* T = QG V */
#pragma omp parallel for schedule(static)
    for (int i = 0; i < dG; ++i)
        for (int j = 0; j < dA; ++j) {
            double s = 0.0;
            for (int k = 0; k < dG; ++k) s += QG[(int64_t)i * dG + k] * V[(int64_t)k * dA + j];
            T[(int64_t)i * dA + j] = s;
        }
    /* out = T QA^T */
#pragma omp parallel for schedule(static)
    for (int i = 0; i < dG; ++i)
        for (int j = 0; j < dA; ++j) {
            double s = 0.0;
            for (int k = 0; k < dA; ++k) s += T[(int64_t)i * dA + k] * QA[(int64_t)j * dA + k];
            out[(int64_t)i * dA + j] = s;
        }
    free(T);
    free(V);
}

/* ------------------------------------------------------------------------
 * Brute force for tiny layers: y = (G (x) A + gamma I)^{-1} vec_r(grad), the
 * damped inverse the eigen expansion of Sec. IV-A is stated to equal, by
 * forming the Kronecker product densely and solving with a Cholesky
 * factorisation.  vec_r stacks the rows of grad ([dG][dA]), for which
 * (G (x) A) vec_r(X) = vec_r(G X A^T) = vec_r(G X A) with A symmetric.
 * Returns 0, or -1 if the matrix is not positive definite.
 * ---------------------------------------------------------------------- */
int oracle_bruteforce(const double *G, int dG, const double *A, int dA, double gamma,
                      const double *grad, double *out)
{
    const int64_t n = (int64_t)dG * dA;
    double *K = (double *)malloc(sizeof(double) * (size_t)n * n);
    oracle_kron(G, dG, dG, A, dA, dA, K);
    for (int64_t i = 0; i < n; ++i) K[i * n + i] += gamma;
    /* K = L L^T, L stored in the lower triangle */
    int status = 0;
    for (int64_t j = 0; j < n && status == 0; ++j) {
        double djj = K[j * n + j];
        for (int64_t k = 0; k < j; ++k) djj -= K[j * n + k] * K[j * n + k];
        if (!(djj > 0.0)) { status = -1; break; }
        const double ljj = sqrt(djj);
        K[j * n + j] = ljj;
#pragma omp parallel for schedule(static)
        for (int64_t i = j + 1; i < n; ++i) {
            double s = K[i * n + j];
            for (int64_t k = 0; k < j; ++k) s -= K[i * n + k] * K[j * n + k];
            K[i * n + j] = s / ljj;
        }
    }
    if (status == 0) {
        for (int64_t i = 0; i < n; ++i) { /* L z = b */
            double s = grad[i];
            for (int64_t k = 0; k < i; ++k) s -= K[i * n + k] * out[k];
            out[i] = s / K[i * n + i];
        }
        for (int64_t i = n - 1; i >= 0; --i) { /* L^T y = z */
            double s = out[i];
            for (int64_t k = i + 1; k < n; ++k) s -= K[k * n + i] * out[k];
            out[i] = s / K[i * n + i];
        }
    }
    free(K);
    return status;
}

/* Dense SPD solve A X = B (A n x n, B n x m) by Cholesky; used by the test of
 * the undamped identity  F^{-1} grad = G^{-1} grad A^{-1}  of Sec. II-C. */
int oracle_spd_solve(const double *A, int n, const double *B, int m, double *X)
{
    double *L = (double *)malloc(sizeof(double) * (size_t)n * n);
    memcpy(L, A, sizeof(double) * (size_t)n * n);
    for (int j = 0; j < n; ++j) {
        double djj = L[(int64_t)j * n + j];
        for (int k = 0; k < j; ++k) djj -= L[(int64_t)j * n + k] * L[(int64_t)j * n + k];
        if (!(djj > 0.0)) { free(L); return -1; }
        const double ljj = sqrt(djj);
        L[(int64_t)j * n + j] = ljj;
        for (int i = j + 1; i < n; ++i) {
            double s = L[(int64_t)i * n + j];
            for (int k = 0; k < j; ++k) s -= L[(int64_t)i * n + k] * L[(int64_t)j * n + k];
            L[(int64_t)i * n + j] = s / ljj;
        }
    }
    for (int c = 0; c < m; ++c) {
        for (int i = 0; i < n; ++i) {
            double s = B[(int64_t)i * m + c];
            for (int k = 0; k < i; ++k) s -= L[(int64_t)i * n + k] * X[(int64_t)k * m + c];
            X[(int64_t)i * m + c] = s / L[(int64_t)i * n + i];
        }
        for (int i = n - 1; i >= 0; --i) {
            double s = X[(int64_t)i * m + c];
            for (int k = i + 1; k < n; ++k) s -= L[(int64_t)k * n + i] * X[(int64_t)k * m + c];
            X[(int64_t)i * m + c] = s / L[(int64_t)i * n + i];
        }
    }
    free(L);
    return 0;
}

/* ------------------------------------------------------------------------
 * Update-decoupled schedule (Sec. IV-C, Sec. V-C): at iteration k the factors
 * are refreshed every f_fac iterations, the eigendecompositions every f_eig,
 * the gradient is preconditioned every iteration.
 * ---------------------------------------------------------------------- */
void oracle_schedule(int64_t k, int f_fac, int f_eig, int *do_factors, int *do_eig)
{
    *do_factors = (k % f_fac) == 0;
    *do_eig = (k % f_eig) == 0;
}

/* ------------------------------------------------------------------------
 * Gradient scaling (Sec. V-C, "K-FAC Hyper-Parameters", the equation for nu): after preconditioning, every layer's gradient is multiplied by
 *     nu = min(1, sqrt(kappa / (alpha^2 * sum_i |<P_i, g_i>|)))
 * where P_i is the preconditioned and g_i the original gradient of layer i, <.,.> the sum of the elementwise
 * products, kappa a user constant and alpha the learning rate.  The layers are given back to back in two
 * flat arrays; sizes[i] elements belong to layer i.  A zero sum gives nu = 1.
 * ---------------------------------------------------------------------- */
double oracle_grad_scale(int nlayers, const int64_t *sizes, const double *precond, const double *grad,
                         double kappa, double alpha)
{
    double total = 0.0;
    int64_t off = 0;
    for (int i = 0; i < nlayers; ++i) {
        double dot = 0.0;
        for (int64_t e = 0; e < sizes[i]; ++e) dot += precond[off + e] * grad[off + e];
        total += fabs(dot);
        off += sizes[i];
    }
    if (!(total > 0.0)) return 1.0;
    const double nu = sqrt(kappa / (alpha * alpha * total));
    return nu < 1.0 ? nu : 1.0;
}

/* ------------------------------------------------------------------------
 * The explicit-inverse method (Sec. II-C, Eq. (kfac-damped) and the update step below it): the damping
 * is added to each Kronecker factor and the step is
 *     out = (G + gamma I)^{-1} grad (A + gamma I)^{-1}
 * Computed here with no eigendecomposition at all: two Cholesky solves.  grad, out: dG x dA row-major.
 * Returns 0, or -1 if a damped factor is not positive definite.
 * ---------------------------------------------------------------------- */
int oracle_precondition_inverse(const double *G, int dG, const double *A, int dA, double gamma,
                                const double *grad, double *out)
{
    int rc = -1;
    double *Gd = (double *)malloc(sizeof(double) * (size_t)dG * dG);
    double *Ad = (double *)malloc(sizeof(double) * (size_t)dA * dA);
    double *Y = (double *)malloc(sizeof(double) * (size_t)dG * dA);    /* (G + gamma I)^{-1} grad          */
    double *Yt = (double *)malloc(sizeof(double) * (size_t)dG * dA);   /* its transpose, dA x dG            */
    double *Zt = (double *)malloc(sizeof(double) * (size_t)dG * dA);   /* (A + gamma I)^{-1} Y^T = out^T    */
    if (Gd && Ad && Y && Yt && Zt) {
        for (int64_t i = 0; i < (int64_t)dG * dG; ++i) Gd[i] = G[i];
        for (int i = 0; i < dG; ++i) Gd[(int64_t)i * dG + i] += gamma;
        for (int64_t i = 0; i < (int64_t)dA * dA; ++i) Ad[i] = A[i];
        for (int i = 0; i < dA; ++i) Ad[(int64_t)i * dA + i] += gamma;
        if (oracle_spd_solve(Gd, dG, grad, dA, Y) == 0) {
            for (int i = 0; i < dG; ++i)
                for (int j = 0; j < dA; ++j) Yt[(int64_t)j * dG + i] = Y[(int64_t)i * dA + j];
            if (oracle_spd_solve(Ad, dA, Yt, dG, Zt) == 0) {      /* A symmetric: Y A^{-1} = (A^{-1} Y^T)^T */
                for (int i = 0; i < dG; ++i)
                    for (int j = 0; j < dA; ++j) out[(int64_t)i * dA + j] = Zt[(int64_t)j * dG + i];
                rc = 0;
            }
        }
    }
    free(Gd); free(Ad); free(Y); free(Yt); free(Zt);
    return rc;
}
