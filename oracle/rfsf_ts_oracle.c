/*
 * CPU oracle for the tensor-sketched Random Fourier Signature Features map
 * (RFSF-TS) and the linear Gram of its features.
 *
 * THIS IS TEST INFRASTRUCTURE. It is a plain, slow, fp64 statement of what the
 * method computes, written from the paper's definitions. It shares no code with
 * the HIP library, is never called by the product path, and is used only by the
 * tests, the smoke check and the CPU-baseline leg of the benchmark.
 *
 * What is computed (order p = 1, truncation level M), per sequence x_0..x_{L-1}
 * (L time points, T = L-1 increments), in the paper's order of steps:
 *
 *   1. Random Fourier features per level m (Sec. 3.1, eq. (rff); appendix class
 *      RandomFourierFeatures, W = Z / bandwidth):
 *        theta = (x_t . W_m[:,a]) / lengthscale
 *        phi_m(x_t) = F^{-1/2} ( cos(theta_0..F-1) , sin(theta_0..F-1) )   in R^{2F}
 *      with an independent W_m per level (Sec. 3.2, "independent RFF maps").
 *   2. Time increments (Sec. 2.1, the difference operator; Sec. 3.2, eq. (rfsf)):
 *        delta_m[k] = phi_m(x_k) - phi_m(x_{k-1}),  k = 1..T
 *   3. CountSketch per level (Sec. 3.5, eq. (cs)):
 *        c_m[k][j] = sum over a with hash_m[a] == j of sign_m[a] * delta_m[k][a]
 *   4. Level recursion (Sec. 3.5, eq. (ts_rec) with p = 1, convolution form):
 *        R_1[k] = c_1[k]
 *        R_m[k] = P_{m-1}[k] (*) c_m[k],   P_{m-1}[k] = sum_{k' < k} R_{m-1}[k']
 *        Phi_m  = sum_k R_m[k]
 *      where (*) is circular convolution modulo D (eq. (ts_def)), evaluated
 *      directly in O(D^2) -- no FFT anywhere in this file.
 *   5. Output row: ( 1 , Phi_1 , ... , Phi_M ), 1 + M*D numbers (Sec. 1, remark on
 *      primal features: shape (N, M D + 1); the level-0 term of eq. (ksig finite)
 *      is the constant 1).
 *   6. Gram of features: K[i][j] = <PhiX[i], PhiY[j]> (Sec. 1, P_X P_X^T).
 *   7. Optional level-wise normalisation (appendix, class SignatureBase: every level divided by
 *      its own norm, the M+1 levels averaged), as a map on feature rows:
 *        Phi_m <- Phi_m / (|Phi_m| sqrt(M+1)),  level 0 (the constant 1) <- 1 / sqrt(M+1),
 *      so that <row_i, row_j> = 1/(M+1) sum_m k_m(i,j) / sqrt(k_m(i,i) k_m(j,j)). A level whose
 *      block is exactly zero (more levels than increments) stays zero.
 *
 * Inputs are the float32 / int32 arrays the GPU library receives, widened to
 * double on read. OpenMP is used over sequences only (they are independent).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int rfsf_ts_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Steps 1-2 for one sequence: delta[m][k][a], m < M, k < T, a < 2F (k is 0-based:
 * delta[m][k] = phi_m(x_{k+1}) - phi_m(x_k)). phi is scratch of 2 * 2F doubles. */
static void increments_one(int64_t L, int d, int M, int F,
                           const float *x, const float *W, double lengthscale,
                           double *delta, double *phi)
{
    const int64_t T = L - 1;
    const int twoF = 2 * F;
    const double scale = 1.0 / sqrt((double)F);
    for (int m = 0; m < M; ++m) {
        double *prev = phi, *cur = phi + twoF;
        for (int64_t t = 0; t < L; ++t) {
            for (int a = 0; a < F; ++a) {
                double dot = 0.0;
                for (int c = 0; c < d; ++c)
                    dot += (double)x[t * d + c] * (double)W[((int64_t)m * d + c) * F + a];
                const double theta = dot / lengthscale;
                cur[a] = scale * cos(theta);
                cur[F + a] = scale * sin(theta);
            }
            if (t > 0) {
                double *dst = delta + ((int64_t)m * T + (t - 1)) * twoF;
                for (int a = 0; a < twoF; ++a)
                    dst[a] = cur[a] - prev[a];
            }
            double *tmp = prev; prev = cur; cur = tmp;
        }
    }
}

/* delta[N][T][M][2F] (double) -- steps 1-2 only, for stage-wise checks. */
int rfsf_ts_oracle_increments(int64_t N, int64_t L, int d, int M, int F,
                              const float *X, const float *W, double lengthscale,
                              double *dphi)
{
    if (N < 0 || L < 1 || d < 1 || M < 1 || F < 1 || !(lengthscale > 0.0)) return -1;
    const int64_t T = L - 1;
    const int twoF = 2 * F;
    int fail = 0;
#pragma omp parallel for schedule(dynamic)
    for (int64_t n = 0; n < N; ++n) {
        double *delta = (double *)malloc(sizeof(double) * (size_t)(M * (T > 0 ? T : 1)) * twoF);
        double *phi = (double *)malloc(sizeof(double) * 2 * twoF);
        if (!delta || !phi) {
#pragma omp atomic write
            fail = 1;
            free(delta); free(phi); continue;
        }
        increments_one(L, d, M, F, X + n * L * d, W, lengthscale, delta, phi);
        for (int64_t k = 0; k < T; ++k)
            for (int m = 0; m < M; ++m)
                memcpy(dphi + ((n * T + k) * M + m) * twoF,
                       delta + ((int64_t)m * T + k) * twoF, sizeof(double) * twoF);
        free(delta); free(phi);
    }
    return fail ? -2 : 0;
}

/* out[N][ld_out] (double), columns 0 .. M*D written. */
int rfsf_ts_oracle_features(int64_t N, int64_t L, int d, int M, int F, int D,
                            const float *X, const float *W,
                            const int32_t *hash, const float *sign,
                            double lengthscale, double *out, int64_t ld_out)
{
    if (N < 0 || L < 1 || d < 1 || M < 1 || F < 1 || D < 1) return -1;
    if (!(lengthscale > 0.0) || ld_out < 1 + (int64_t)M * D) return -1;
    const int64_t T = L - 1;
    const int twoF = 2 * F;
    for (int64_t i = 0; i < (int64_t)M * twoF; ++i)
        if (hash[i] < 0 || hash[i] >= D) return -3;
    int fail = 0;
#pragma omp parallel for schedule(dynamic)
    for (int64_t n = 0; n < N; ++n) {
        double *row = out + n * ld_out;
        row[0] = 1.0;                                   /* level 0 */
        for (int64_t j = 0; j < (int64_t)M * D; ++j) row[1 + j] = 0.0;
        if (T == 0) continue;                           /* no increments: empty sums */

        double *delta = (double *)malloc(sizeof(double) * (size_t)M * T * twoF);
        double *phi = (double *)malloc(sizeof(double) * 2 * twoF);
        double *c = (double *)calloc((size_t)M * T * D, sizeof(double));
        double *Rprev = (double *)malloc(sizeof(double) * (size_t)T * D);
        double *Rcur = (double *)malloc(sizeof(double) * (size_t)T * D);
        double *P = (double *)malloc(sizeof(double) * D);
        if (!delta || !phi || !c || !Rprev || !Rcur || !P) {
#pragma omp atomic write
            fail = 1;
            free(delta); free(phi); free(c); free(Rprev); free(Rcur); free(P);
            continue;
        }
        /* steps 1-2 */
        increments_one(L, d, M, F, X + n * L * d, W, lengthscale, delta, phi);
        /* step 3: CountSketch of every increment with the level's own hash/sign */
        for (int m = 0; m < M; ++m)
            for (int64_t k = 0; k < T; ++k) {
                const double *dl = delta + ((int64_t)m * T + k) * twoF;
                double *ck = c + ((int64_t)m * T + k) * D;
                for (int a = 0; a < twoF; ++a)
                    ck[hash[m * twoF + a]] += (double)sign[m * twoF + a] * dl[a];
            }
        /* step 4: level 1 */
        memcpy(Rprev, c, sizeof(double) * (size_t)T * D);
        for (int64_t k = 0; k < T; ++k)
            for (int j = 0; j < D; ++j)
                row[1 + j] += Rprev[k * D + j];
        /* step 4: levels 2..M */
        for (int m = 1; m < M; ++m) {
            for (int j = 0; j < D; ++j) P[j] = 0.0;     /* exclusive prefix of level m-1 */
            for (int64_t k = 0; k < T; ++k) {
                const double *ck = c + ((int64_t)m * T + k) * D;
                double *r = Rcur + k * D;
                for (int j = 0; j < D; ++j) {
                    double acc = 0.0;
                    for (int q = 0; q < D; ++q) {
                        int idx = j - q;
                        if (idx < 0) idx += D;
                        acc += P[q] * ck[idx];
                    }
                    r[j] = acc;
                }
                for (int j = 0; j < D; ++j) P[j] += Rprev[k * D + j];   /* after use */
            }
            double *blk = row + 1 + (int64_t)m * D;
            for (int64_t k = 0; k < T; ++k)
                for (int j = 0; j < D; ++j)
                    blk[j] += Rcur[k * D + j];
            double *tmp = Rprev; Rprev = Rcur; Rcur = tmp;
        }
        free(delta); free(phi); free(c); free(Rprev); free(Rcur); free(P);
    }
    return fail ? -2 : 0;
}

/* K[Nx][ldk] = PhiX[Nx][ldx] . PhiY[Ny][ldy]^T over the first ncols columns. */
int rfsf_ts_oracle_gram(const double *PhiX, int64_t Nx, int64_t ldx,
                        const double *PhiY, int64_t Ny, int64_t ldy,
                        int64_t ncols, double *K, int64_t ldk)
{
    if (Nx < 0 || Ny < 0 || ncols < 0 || ldx < ncols || ldy < ncols || ldk < Ny) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < Nx; ++i)
        for (int64_t j = 0; j < Ny; ++j) {
            double acc = 0.0;
            for (int64_t c = 0; c < ncols; ++c)
                acc += PhiX[i * ldx + c] * PhiY[j * ldy + c];
            K[i * ldk + j] = acc;
        }
    return 0;
}

/* Step 7, in place on Phi[N][ld] (columns 0 .. M*D). */
int rfsf_ts_oracle_normalize(double *Phi, int64_t N, int64_t ld, int M, int D)
{
    if (N < 0 || M < 1 || D < 1 || ld < 1 + (int64_t)M * D) return -1;
    const double w = 1.0 / sqrt((double)(M + 1));
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        double *row = Phi + n * ld;
        row[0] = row[0] * w;                      /* level 0 has norm |1| = 1 */
        for (int m = 0; m < M; ++m) {
            double *blk = row + 1 + (int64_t)m * D;
            double ss = 0.0;
            for (int j = 0; j < D; ++j) ss += blk[j] * blk[j];
            if (ss > 0.0) {
                const double f = w / sqrt(ss);
                for (int j = 0; j < D; ++j) blk[j] *= f;
            }
        }
    }
    return 0;
}

/*
 * Sibling variant RFSF-DP-1D (Sec. 3.3, eq. (dp1d); static map of Sec. 3.1, eq. (rff_1d), with the
 * appendix scale of class RandomFourierFeatures1D; appendix class DiagonalProjection with
 * internal size 1): F independent copies of a size-1 one-dimensional random Fourier signature
 * feature map, per level m = 1..M and component i < F
 *     phi_m(x)[i]   = sqrt(2) cos( (x . W_m[:, i]) / lengthscale + bias_m[i] )
 *     u_m[k][i]     = phi_m(x_k)[i] - phi_m(x_{k-1})[i]
 *     Phi_m[i]      = F^{-1/2} sum_{k_1 < ... < k_m} u_1[k_1][i] ... u_m[k_m][i]
 * evaluated with the recursion of eq. (rfsf_rec), p = 1, component by component:
 *     A_m <- A_m + A_{m-1}(before this step) * u_m[k],  A_0 = 1.
 * out[N][ld_out]: column 0 is 1, columns 1 + (m-1) F + i hold Phi_m[i].
 */
int rfsf_dp1d_oracle_features(int64_t N, int64_t L, int d, int M, int F,
                              const float *X, const float *W, const float *bias,
                              double lengthscale, double *out, int64_t ld_out)
{
    if (N < 0 || L < 1 || d < 1 || M < 1 || F < 1) return -1;
    if (!(lengthscale > 0.0) || ld_out < 1 + (int64_t)M * F) return -1;
    const double root2 = sqrt(2.0), scale = 1.0 / sqrt((double)F);
    int fail = 0;
#pragma omp parallel for schedule(dynamic)
    for (int64_t n = 0; n < N; ++n) {
        double *row = out + n * ld_out;
        double *A = (double *)calloc((size_t)M * F, sizeof(double));
        double *prev = (double *)malloc(sizeof(double) * (size_t)M * F);
        double *cur = (double *)malloc(sizeof(double) * (size_t)M * F);
        if (!A || !prev || !cur) {
#pragma omp atomic write
            fail = 1;
            free(A); free(prev); free(cur);
            continue;
        }
        const float *x = X + n * L * d;
        for (int64_t t = 0; t < L; ++t) {
            for (int m = 0; m < M; ++m)
                for (int i = 0; i < F; ++i) {
                    double dot = 0.0;
                    for (int c = 0; c < d; ++c)
                        dot += (double)x[t * d + c] * (double)W[((int64_t)m * d + c) * F + i];
                    cur[m * F + i] = root2 * cos(dot / lengthscale + (double)bias[m * F + i]);
                }
            if (t > 0) {
                for (int m = M - 1; m >= 0; --m)          /* descending: A_{m-1} is still the old value */
                    for (int i = 0; i < F; ++i) {
                        const double u = cur[m * F + i] - prev[m * F + i];
                        A[m * F + i] += (m == 0 ? 1.0 : A[(m - 1) * F + i]) * u;
                    }
            }
            double *tmp = prev; prev = cur; cur = tmp;
        }
        row[0] = 1.0;
        for (int64_t j = 0; j < (int64_t)M * F; ++j) row[1 + j] = scale * A[j];
        free(A); free(prev); free(cur);
    }
    return fail ? -2 : 0;
}

/*
 * Sibling variant RFSF-TRP (Sec. 3.4, eqs. (trp_def), (trp), (trp_rec) read with kappa for k; appendix
 * class TensorizedRandomProjection): the random Fourier increments of steps 1-2 above are projected
 * per level by an independent Gaussian matrix and combined by Hadamard products,
 *     p_m[k]   = Z_m delta_m[k]                  Z_m [Q x 2F], i.i.d. N(0, 1)
 *     A_m     <- A_m + A_{m-1}(before this step) (.) p_m[k],   A_0 = 1 (all ones)
 *     Phi_m    = Q^{-1/2} A_m   =  Q^{-1/2} sum_{k_1<...<k_m} p_1[k_1] (.) ... (.) p_m[k_m].
 * Z is stored [M][Q][2F] (each projection vector contiguous). out[N][ld_out]: column 0 is 1,
 * columns 1 + (m-1) Q + q hold Phi_m[q].
 */
int rfsf_trp_oracle_features(int64_t N, int64_t L, int d, int M, int F, int Q,
                             const float *X, const float *W, const float *Z,
                             double lengthscale, double *out, int64_t ld_out)
{
    if (N < 0 || L < 1 || d < 1 || M < 1 || F < 1 || Q < 1) return -1;
    if (!(lengthscale > 0.0) || ld_out < 1 + (int64_t)M * Q) return -1;
    const int64_t T = L - 1;
    const int twoF = 2 * F;
    const double scale = 1.0 / sqrt((double)Q);
    int fail = 0;
#pragma omp parallel for schedule(dynamic)
    for (int64_t n = 0; n < N; ++n) {
        double *row = out + n * ld_out;
        row[0] = 1.0;
        for (int64_t j = 0; j < (int64_t)M * Q; ++j) row[1 + j] = 0.0;
        if (T == 0) continue;
        double *delta = (double *)malloc(sizeof(double) * (size_t)M * T * twoF);
        double *phi = (double *)malloc(sizeof(double) * 2 * twoF);
        double *A = (double *)calloc((size_t)M * Q, sizeof(double));
        if (!delta || !phi || !A) {
#pragma omp atomic write
            fail = 1;
            free(delta); free(phi); free(A);
            continue;
        }
        increments_one(L, d, M, F, X + n * L * d, W, lengthscale, delta, phi);
        for (int64_t k = 0; k < T; ++k)
            for (int m = M - 1; m >= 0; --m) {            /* descending: A_{m-1} is still the old value */
                const double *dl = delta + ((int64_t)m * T + k) * twoF;
                for (int q = 0; q < Q; ++q) {
                    const float *z = Z + ((int64_t)m * Q + q) * twoF;
                    double p = 0.0;
                    for (int a = 0; a < twoF; ++a) p += (double)z[a] * dl[a];
                    A[m * Q + q] += (m == 0 ? 1.0 : A[(m - 1) * Q + q]) * p;
                }
            }
        for (int64_t j = 0; j < (int64_t)M * Q; ++j) row[1 + j] = scale * A[j];
        free(delta); free(phi); free(A);
    }
    return fail ? -2 : 0;
}

/* out[j] = sum_q a[q] * b[(j - q) mod D]: circular convolution, the direct O(D^2) way. */
static void circular_convolution(int D, const double *a, const double *b, double *out)
{
    for (int j = 0; j < D; ++j) {
        double acc = 0.0;
        for (int q = 0; q < D; ++q) {
            int idx = j - q;
            if (idx < 0) idx += D;
            acc += a[q] * b[idx];
        }
        out[j] = acc;
    }
}

/*
 * RFSF-TS with signature order p >= 1 (Sec. 2.1, the factor 1 / i!^(p); Sec. 3.5, eq. (ts_rec) with the
 * sum over q = 1..p): a time step may be used up to p times in a row, a run of q equal time indices
 * weighs 1/q!,
 *     R_m[k] = sum_{q=1}^{min(p,m)} (1/q!)  P_{m-q}[k] (*) c_{m-q+1}[k] (*) ... (*) c_m[k],
 *     P_j[k] = sum_{k' < k} R_j[k']  (exclusive prefix over time),  P_0 = unit impulse at bucket 0,
 *     Phi_m  = sum_k R_m[k].
 * order = 1 is rfsf_ts_oracle_features (kept as a separate, simpler function). Same arguments otherwise.
 */
int rfsf_ts_oracle_features_order(int64_t N, int64_t L, int d, int M, int F, int D, int order,
                                  const float *X, const float *W,
                                  const int32_t *hash, const float *sign,
                                  double lengthscale, double *out, int64_t ld_out)
{
    if (N < 0 || L < 1 || d < 1 || M < 1 || F < 1 || D < 1 || order < 1) return -1;
    if (!(lengthscale > 0.0) || ld_out < 1 + (int64_t)M * D) return -1;
    const int64_t T = L - 1;
    const int twoF = 2 * F;
    for (int64_t i = 0; i < (int64_t)M * twoF; ++i)
        if (hash[i] < 0 || hash[i] >= D) return -3;
    int fail = 0;
#pragma omp parallel for schedule(dynamic)
    for (int64_t n = 0; n < N; ++n) {
        double *row = out + n * ld_out;
        row[0] = 1.0;
        for (int64_t j = 0; j < (int64_t)M * D; ++j) row[1 + j] = 0.0;
        if (T == 0) continue;
        double *delta = (double *)malloc(sizeof(double) * (size_t)M * T * twoF);
        double *phi = (double *)malloc(sizeof(double) * 2 * twoF);
        double *c = (double *)calloc((size_t)M * T * D, sizeof(double));
        double *P = (double *)calloc((size_t)(M + 1) * D, sizeof(double));   /* P[j]: prefix of level j, j = 0..M */
        double *R = (double *)malloc(sizeof(double) * (size_t)(M + 1) * D);
        double *v = (double *)malloc(sizeof(double) * D), *w = (double *)malloc(sizeof(double) * D);
        if (!delta || !phi || !c || !P || !R || !v || !w) {
#pragma omp atomic write
            fail = 1;
            free(delta); free(phi); free(c); free(P); free(R); free(v); free(w);
            continue;
        }
        increments_one(L, d, M, F, X + n * L * d, W, lengthscale, delta, phi);
        for (int m = 0; m < M; ++m)
            for (int64_t k = 0; k < T; ++k) {
                const double *dl = delta + ((int64_t)m * T + k) * twoF;
                double *ck = c + ((int64_t)m * T + k) * D;
                for (int a = 0; a < twoF; ++a)
                    ck[hash[m * twoF + a]] += (double)sign[m * twoF + a] * dl[a];
            }
        P[0] = 1.0;                                     /* level 0: the unit of the convolution */
        for (int64_t k = 0; k < T; ++k) {
            for (int m = 1; m <= M; ++m) {              /* R_m[k] from the prefixes before step k */
                double *Rm = R + (int64_t)m * D;
                for (int j = 0; j < D; ++j) Rm[j] = 0.0;
                double fact = 1.0;
                for (int q = 1; q <= order && q <= m; ++q) {
                    fact *= (double)q;
                    memcpy(v, P + (int64_t)(m - q) * D, sizeof(double) * D);
                    for (int j = m - q + 1; j <= m; ++j) {
                        circular_convolution(D, v, c + ((int64_t)(j - 1) * T + k) * D, w);
                        double *t = v; v = w; w = t;
                    }
                    for (int j = 0; j < D; ++j) Rm[j] += v[j] / fact;
                }
            }
            for (int m = 1; m <= M; ++m)                /* after use: the prefixes now include step k */
                for (int j = 0; j < D; ++j) P[(int64_t)m * D + j] += R[(int64_t)m * D + j];
        }
        for (int m = 1; m <= M; ++m)
            for (int j = 0; j < D; ++j) row[1 + (int64_t)(m - 1) * D + j] = P[(int64_t)m * D + j];
        free(delta); free(phi); free(c); free(P); free(R); free(v); free(w);
    }
    return fail ? -2 : 0;
}
