/*
 * gvq_oracle.c -- float64 CPU oracle for the GradiVeQ slice-wise linear PCA codec.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the HIP
 * library is checked against.  It shares no code, header, table or helper with the
 * HIP path, and nothing in the product package may load it.  Only tests, the smoke
 * check and the benchmark's CPU-baseline leg call it.
 *
 * What it computes (GradiVeQ, Section 2, "Description of GradiVeQ"):
 *   - a flattened gradient of M numbers is cut into slices of d adjacent numbers
 *     (the paper's slice size K); a last partial slice is zero-padded;
 *   - PCA paragraph after Eq. (4): the whitening vector mu is the mean of the sample
 *     slices, C is their covariance, the eigen-decomposition of C sorted by
 *     decreasing eigenvalue gives U, and the compressor is the first k columns
 *     (the paper's d);
 *   - Eq. (2)  compress:    y_n = U^T (x_n - mu/N)
 *   - Eq. (3)  aggregate:   Y   = sum_n y_n   ( = U^T (sum_n x_n - mu) )
 *   - Eq. (4)  decompress:  xhat = U Y + mu
 *
 * Readings where the paper is silent (they are the library's documented contract):
 *   - sample set of one basis = every full slice that lies in the basis' slice range,
 *     from each of the L fit gradients (the partial tail slice is not a sample);
 *   - covariance normalised by 1/n, computed two-pass (subtract the mean first);
 *   - "SVD" of the symmetric PSD covariance = its symmetric eigendecomposition, done
 *     here by the classical cyclic Jacobi rotation method run to convergence;
 *   - each kept eigenvector is negated if needed so that its entry of largest
 *     magnitude (lowest index on ties) is positive;
 *   - one mu and one U per basis, shared by all slices of the basis' range;
 *   - a basis with no sample (its range holds only the partial tail slice) has mu = 0,
 *     eigenvalues 0 and the first k unit vectors as U.
 *
 * Every floating-point value is widened to double on load (fp32 and bf16 widen
 * exactly) and every operation is done in double.  Loops over slices are split over
 * OpenMP threads; nothing else is blocked, fused or reordered.
 *
 * Pins (tests/test_oracle_*.py): closed forms for mean/covariance on hand-made data,
 * numpy's eigh on small matrices, 2x2 closed-form eigenpairs, exact round trip at
 * k = d, Eq. (3) linearity, the eigenvalue-mass identity of Eq. (5) on the fit set.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { GO_F32 = 0, GO_BF16 = 1 };
#define ORACLE_MAX_D 1024 /* largest slice length (size of the per-slice stack buffers) */

/* Widen element idx of a stored gradient to double. bf16 is the upper half of an fp32. */
static double load_elem(const void *g, int dtype, int64_t idx)
{
    if (dtype == GO_F32)
        return (double)((const float *)g)[idx];
    uint32_t bits = (uint32_t)((const uint16_t *)g)[idx] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/* Slice j of a gradient of M elements, zero-padded past M (Section 2: slices of K
 * adjacent gradients; padding is this build's reading for M not divisible by d). */
static void load_slice(const void *g, int dtype, int64_t M, int d, int64_t j, double *x)
{
    for (int e = 0; e < d; ++e) {
        int64_t idx = j * (int64_t)d + e;
        x[e] = idx < M ? load_elem(g, dtype, idx) : 0.0;
    }
}

int gvq_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void gvq_oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* ------------------------------------------------------------------------------------
 * Symmetric eigendecomposition by cyclic Jacobi rotations.
 * A (n x n, row-major, symmetric) is overwritten; on return its diagonal holds the
 * eigenvalues (unsorted) and V (n x n) holds the eigenvectors as columns, A_in = V D V^T.
 * Each rotation zeroes one off-diagonal pair (p,q): with theta = (a_qq - a_pp)/(2 a_pq),
 * t = sign(theta)/(|theta| + sqrt(theta^2+1)) is the smaller root of t^2 + 2 theta t - 1 = 0,
 * c = 1/sqrt(1+t^2), s = t c, and A <- J^T A J, V <- V J with J the plane rotation
 * [[c, s], [-s, c]] in the (p,q) plane.
 * Sweeps continue until the off-diagonal Frobenius norm is <= tol * ||A||_F.
 * Returns the number of sweeps used, or -1 if max_sweeps was not enough.
 * ---------------------------------------------------------------------------------- */
int gvq_oracle_jacobi_eig(double *A, double *V, int n, double tol, int max_sweeps)
{
    for (int i = 0; i < n; ++i)
        for (int j = 0; j < n; ++j)
            V[i * n + j] = (i == j) ? 1.0 : 0.0;

    double fro2 = 0.0;
    for (int i = 0; i < n * n; ++i) fro2 += A[i] * A[i];
    if (fro2 == 0.0) return 0;

    for (int sweep = 0; sweep <= max_sweeps; ++sweep) {
        double off2 = 0.0;
        for (int i = 0; i < n; ++i)
            for (int j = 0; j < n; ++j)
                if (i != j) off2 += A[i * n + j] * A[i * n + j];
        if (off2 <= tol * tol * fro2) return sweep;
        if (sweep == max_sweeps) break;

        for (int p = 0; p < n - 1; ++p) {
            for (int q = p + 1; q < n; ++q) {
                double apq = A[p * n + q];
                if (apq == 0.0) continue;
                double app = A[p * n + p], aqq = A[q * n + q];
                double theta = (aqq - app) / (2.0 * apq);
                double t = (theta >= 0.0 ? 1.0 : -1.0) / (fabs(theta) + sqrt(theta * theta + 1.0));
                double c = 1.0 / sqrt(1.0 + t * t);
                double s = t * c;
                /* columns p and q of A: A <- A J */
                for (int r = 0; r < n; ++r) {
                    double arp = A[r * n + p], arq = A[r * n + q];
                    A[r * n + p] = c * arp - s * arq;
                    A[r * n + q] = s * arp + c * arq;
                }
                /* rows p and q of A: A <- J^T A */
                for (int r = 0; r < n; ++r) {
                    double apr = A[p * n + r], aqr = A[q * n + r];
                    A[p * n + r] = c * apr - s * aqr;
                    A[q * n + r] = s * apr + c * aqr;
                }
                /* the rotated pair is zero by construction; remove the rounding residue */
                A[p * n + q] = 0.0;
                A[q * n + p] = 0.0;
                /* V <- V J */
                for (int r = 0; r < n; ++r) {
                    double vrp = V[r * n + p], vrq = V[r * n + q];
                    V[r * n + p] = c * vrp - s * vrq;
                    V[r * n + q] = s * vrp + c * vrq;
                }
            }
        }
    }
    return -1;
}

/* ------------------------------------------------------------------------------------
 * Sample mean and covariance of one basis (PCA paragraph of Section 2).
 * Samples: every full slice j in [s0, s1) (j*d + d <= M) of each of the L gradients.
 * mu[d], C[d*d] row-major, normaliser 1/n.  Returns the sample count n.
 * ---------------------------------------------------------------------------------- */
int64_t gvq_oracle_moments(const void *const *grads, int L, int64_t M, int d, int dtype,
                           int64_t s0, int64_t s1, double *mu, double *C)
{
    int64_t full = M / d;           /* number of full slices in a gradient */
    if (s1 > full) s1 = full;
    int64_t per = s1 > s0 ? s1 - s0 : 0;
    int64_t n = per * (int64_t)L;
    for (int e = 0; e < d; ++e) mu[e] = 0.0;
    for (int i = 0; i < d * d; ++i) C[i] = 0.0;
    if (n == 0) return 0;

    int nt = gvq_oracle_num_threads();
    double *part = (double *)calloc((size_t)nt * (size_t)(d * d), sizeof(double));

    /* pass 1: mean */
#pragma omp parallel num_threads(nt)
    {
#ifdef _OPENMP
        int t = omp_get_thread_num();
#else
        int t = 0;
#endif
        double *acc = part + (size_t)t * (size_t)(d * d);
        double x[ORACLE_MAX_D];
        for (int l = 0; l < L; ++l) {
#pragma omp for schedule(static)
            for (int64_t j = s0; j < s1; ++j) {
                load_slice(grads[l], dtype, M, d, j, x);
                for (int e = 0; e < d; ++e) acc[e] += x[e];
            }
        }
    }
    for (int t = 0; t < nt; ++t)
        for (int e = 0; e < d; ++e) mu[e] += part[(size_t)t * (size_t)(d * d) + e];
    for (int e = 0; e < d; ++e) mu[e] /= (double)n;

    /* pass 2: covariance of the centred samples */
    memset(part, 0, (size_t)nt * (size_t)(d * d) * sizeof(double));
#pragma omp parallel num_threads(nt)
    {
#ifdef _OPENMP
        int t = omp_get_thread_num();
#else
        int t = 0;
#endif
        double *acc = part + (size_t)t * (size_t)(d * d);
        double x[ORACLE_MAX_D];
        for (int l = 0; l < L; ++l) {
#pragma omp for schedule(static)
            for (int64_t j = s0; j < s1; ++j) {
                load_slice(grads[l], dtype, M, d, j, x);
                for (int e = 0; e < d; ++e) x[e] -= mu[e];
                for (int a = 0; a < d; ++a) {
                    double xa = x[a];
                    double *row = acc + (size_t)a * d;
                    for (int b = a; b < d; ++b) row[b] += xa * x[b];
                }
            }
        }
    }
    for (int t = 0; t < nt; ++t)
        for (int a = 0; a < d; ++a)
            for (int b = a; b < d; ++b)
                C[a * d + b] += part[(size_t)t * (size_t)(d * d) + a * d + b];
    for (int a = 0; a < d; ++a)
        for (int b = a; b < d; ++b) {
            C[a * d + b] /= (double)n;
            C[b * d + a] = C[a * d + b];
        }
    free(part);
    return n;
}

/* The sample mean alone (the "whitening vector" of the PCA paragraph of Section 2) over the same
 * sample set as gvq_oracle_moments: every full slice [s0, s1) of each of the L gradients.  For
 * checks at sizes where the whole covariance is too slow.  Returns the number of samples. */
int64_t gvq_oracle_mean(const void *const *grads, int L, int64_t M, int d, int dtype, int64_t s0,
                        int64_t s1, double *mu)
{
    int64_t full = M / d;
    if (s1 > full) s1 = full;
    int64_t per = s1 > s0 ? s1 - s0 : 0;
    int64_t n = per * (int64_t)L;
    for (int e = 0; e < d; ++e) {
        double acc = 0.0;
        for (int l = 0; l < L; ++l) {
#pragma omp parallel for schedule(static) reduction(+ : acc)
            for (int64_t j = s0; j < s1; ++j) acc += load_elem(grads[l], dtype, j * d + e);
        }
        mu[e] = n > 0 ? acc / (double)n : 0.0;
    }
    return n;
}

/* One entry (a,b) of the covariance above, computed on its own (for spot checks at
 * sizes where the whole matrix is too slow): two passes over the samples. */
double gvq_oracle_cov_entry(const void *const *grads, int L, int64_t M, int d, int dtype,
                            int64_t s0, int64_t s1, int a, int b)
{
    int64_t full = M / d;
    if (s1 > full) s1 = full;
    int64_t per = s1 > s0 ? s1 - s0 : 0;
    int64_t n = per * (int64_t)L;
    if (n == 0) return 0.0;
    double sa = 0.0, sb = 0.0;
    for (int l = 0; l < L; ++l) {
#pragma omp parallel for schedule(static) reduction(+ : sa, sb)
        for (int64_t j = s0; j < s1; ++j) {
            sa += load_elem(grads[l], dtype, j * d + a);
            sb += load_elem(grads[l], dtype, j * d + b);
        }
    }
    double ma = sa / (double)n, mb = sb / (double)n, acc = 0.0;
    for (int l = 0; l < L; ++l) {
#pragma omp parallel for schedule(static) reduction(+ : acc)
        for (int64_t j = s0; j < s1; ++j)
            acc += (load_elem(grads[l], dtype, j * d + a) - ma) *
                   (load_elem(grads[l], dtype, j * d + b) - mb);
    }
    return acc / (double)n;
}

/* ------------------------------------------------------------------------------------
 * From a covariance matrix to the compressor: eigendecompose, sort eigenvalues in
 * decreasing order, keep the first k eigenvectors, fix their signs.
 * C[d*d] is not modified.  U[d*k] row-major (U[e*k + i] = entry e of eigenvector i),
 * eig[d] all eigenvalues, descending.  Returns Jacobi's sweep count or -1.
 * ---------------------------------------------------------------------------------- */
int gvq_oracle_basis_from_cov(const double *C, int d, int k, double *U, double *eig)
{
    double *A = (double *)malloc(sizeof(double) * d * d);
    double *V = (double *)malloc(sizeof(double) * d * d);
    int *order = (int *)malloc(sizeof(int) * d);
    memcpy(A, C, sizeof(double) * d * d);
    int sweeps = gvq_oracle_jacobi_eig(A, V, d, 1e-15, 100);

    /* stable selection sort of indices by decreasing eigenvalue */
    for (int i = 0; i < d; ++i) order[i] = i;
    for (int i = 0; i < d; ++i) {
        int best = i;
        for (int j = i + 1; j < d; ++j)
            if (A[order[j] * d + order[j]] > A[order[best] * d + order[best]]) best = j;
        int tmp = order[best];
        for (int j = best; j > i; --j) order[j] = order[j - 1];
        order[i] = tmp;
    }
    for (int i = 0; i < d; ++i) eig[i] = A[order[i] * d + order[i]];
    for (int i = 0; i < k; ++i) {
        int col = order[i];
        int arg = 0;
        double big = -1.0;
        for (int e = 0; e < d; ++e) {
            double m = fabs(V[e * d + col]);
            if (m > big) { big = m; arg = e; }
        }
        double sign = V[arg * d + col] < 0.0 ? -1.0 : 1.0;
        for (int e = 0; e < d; ++e) U[e * k + i] = sign * V[e * d + col];
    }
    free(A); free(V); free(order);
    return sweeps;
}

/* ------------------------------------------------------------------------------------
 * Basis refresh for every block: block b covers slices [offs[b], offs[b+1]).
 * U[B][d][k], mu[B][d], eig[B][d], optional C_out[B][d][d] (may be NULL).
 * A block whose range holds no full slice has no sample: its mean and covariance are
 * taken as zero, so its eigenvectors are the unit vectors and U is the first k of them.
 * Returns 0, or -1 if an eigensolve did not converge.
 * ---------------------------------------------------------------------------------- */
int gvq_oracle_fit(const void *const *grads, int L, int64_t M, int d, int k, int dtype,
                   int n_blocks, const int64_t *offs, int first_slice_only, double *U, double *mu,
                   double *eig, double *C_out)
{
    double *C = (double *)malloc(sizeof(double) * d * d);
    int rc = 0;
    for (int b = 0; b < n_blocks; ++b) {
        /* Section 3, "compressor reuse": with first_slice_only the compressor of a group of
         * slices is computed from the group's first slice alone (its L time samples) */
        int64_t s1 = first_slice_only ? offs[b] + 1 : offs[b + 1];
        gvq_oracle_moments(grads, L, M, d, dtype, offs[b], s1, mu + (size_t)b * d, C);
        if (C_out) memcpy(C_out + (size_t)b * d * d, C, sizeof(double) * d * d);
        int sw = gvq_oracle_basis_from_cov(C, d, k, U + (size_t)b * d * k, eig + (size_t)b * d);
        if (sw < 0 && rc == 0) rc = -1;
    }
    free(C);
    return rc;
}

/* block that slice j belongs to (offs increasing, offs[0] = 0, offs[B] = S) */
static int block_of(int64_t j, int n_blocks, const int64_t *offs)
{
    int b = 0;
    while (b + 1 < n_blocks && j >= offs[b + 1]) ++b;
    return b;
}

/* ------------------------------------------------------------------------------------
 * Eq. (2): y_j = U^T (x_j - mu/N) for slices j in [j0, j1).  out[(j-j0)*k + i].
 * ---------------------------------------------------------------------------------- */
void gvq_oracle_compress(const void *grad, int64_t M, int d, int k, int dtype, int n_blocks,
                         const int64_t *offs, const double *U, const double *mu,
                         int n_workers, int64_t j0, int64_t j1, double *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t j = j0; j < j1; ++j) {
        double x[ORACLE_MAX_D];
        int b = block_of(j, n_blocks, offs);
        const double *Ub = U + (size_t)b * d * k, *mub = mu + (size_t)b * d;
        load_slice(grad, dtype, M, d, j, x);
        for (int e = 0; e < d; ++e) x[e] -= mub[e] / (double)n_workers;
        for (int i = 0; i < k; ++i) {
            double acc = 0.0;
            for (int e = 0; e < d; ++e) acc += Ub[e * k + i] * x[e];
            out[(j - j0) * k + i] = acc;
        }
    }
}

/* Eq. (3): out = sum over the N compressed vectors, each of len numbers. */
void gvq_oracle_aggregate(const double *const *comps, int N, int64_t len, double *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < len; ++i) {
        double acc = 0.0;
        for (int n = 0; n < N; ++n) acc += comps[n][i];
        out[i] = acc;
    }
}

/* ------------------------------------------------------------------------------------
 * Eq. (4): xhat_j = U Y_j + mu for slices j in [j0, j1); Y holds those slices only
 * (Y[(j-j0)*k + i]); out[(j-j0)*d + e], every slice written in full (d numbers), the
 * caller drops what lies past M.
 * ---------------------------------------------------------------------------------- */
void gvq_oracle_decompress(const double *Y, int d, int k, int n_blocks, const int64_t *offs,
                           const double *U, const double *mu, int64_t j0, int64_t j1,
                           double *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t j = j0; j < j1; ++j) {
        int b = block_of(j, n_blocks, offs);
        const double *Ub = U + (size_t)b * d * k, *mub = mu + (size_t)b * d;
        const double *y = Y + (j - j0) * k;
        for (int e = 0; e < d; ++e) {
            double acc = 0.0;
            for (int i = 0; i < k; ++i) acc += Ub[e * k + i] * y[i];
            out[(j - j0) * d + e] = acc + mub[e];
        }
    }
}

/* ------------------------------------------------------------------------------------
 * Section 3, "Compressor dimension" (Eq. 5): the smallest k such that
 *     (eig[0] + ... + eig[k-1]) / (eig[0] + ... + eig[d-1]) >= 1 - lambda,
 * eig in decreasing order, 0 <= lambda < 1.  Partial sums are taken from the largest
 * eigenvalue down, in double.  If the total is not positive (no sample, or all-zero
 * data) there is nothing to lose and the answer is 1.
 * ---------------------------------------------------------------------------------- */
int gvq_oracle_select_k(const double *eig, int d, double lambda)
{
    double total = 0.0;
    for (int i = 0; i < d; ++i) total += eig[i];
    if (!(total > 0.0)) return 1;
    double cum = 0.0;
    for (int k = 1; k <= d; ++k) {
        cum += eig[k - 1];
        if (cum / total >= 1.0 - lambda) return k;
    }
    return d;
}

/* ------------------------------------------------------------------------------------
 * Section 3, "Number of compressed iterations" (Eq. 6): the local compression loss of one
 * worker,  || g_n - (U g'_n + mu/N) ||^2  with g'_n = U^T (g_n - mu/N)  (Eq. 2),
 * summed per basis over the slices of its range.  The tail slice is compressed
 * zero-padded like everywhere else, but only its real elements (index < M) are part of
 * g_n and enter the norm.  loss[n_blocks].
 * ---------------------------------------------------------------------------------- */
void gvq_oracle_local_loss(const void *grad, int64_t M, int d, int k, int dtype, int n_blocks,
                           const int64_t *offs, const double *U, const double *mu,
                           int n_workers, double *loss)
{
    int64_t S = (M + d - 1) / d;
    for (int b = 0; b < n_blocks; ++b) {
        const double *Ub = U + (size_t)b * d * k, *mub = mu + (size_t)b * d;
        double acc = 0.0;
        int64_t j0 = offs[b], j1 = offs[b + 1] < S ? offs[b + 1] : S;
#pragma omp parallel for schedule(static) reduction(+ : acc)
        for (int64_t j = j0; j < j1; ++j) {
            double x[ORACLE_MAX_D], y[ORACLE_MAX_D];
            load_slice(grad, dtype, M, d, j, x);
            for (int e = 0; e < d; ++e) x[e] -= mub[e] / (double)n_workers;
            for (int i = 0; i < k; ++i) {
                double a = 0.0;
                for (int e = 0; e < d; ++e) a += Ub[e * k + i] * x[e];
                y[i] = a;
            }
            for (int e = 0; e < d; ++e) {
                if (j * (int64_t)d + e >= M) break;
                double r = x[e];            /* (g - mu/N) - U y  ==  g - (U y + mu/N) */
                for (int i = 0; i < k; ++i) r -= Ub[e * k + i] * y[i];
                acc += r * r;
            }
        }
        loss[b] = acc;
    }
}
