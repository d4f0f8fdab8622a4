/*
 * fp64 CPU oracle for linear attention with kernel f(x) = a + b*x.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path (the HIP library and
 * its Python binding) may include, link or call this file.  Only the tests,
 * the smoke check and the benchmark's cpu_baseline leg use it.  It shares no
 * code with the HIP kernels.
 *
 * Layout: every tensor is dense row-major [BH, N, D] (D contiguous), which is
 * the paper's "[B x H, N, D]" storage (Sec. 4; Alg. 1-4 input lines).  G is
 * [BH, N].  All arithmetic is double precision.  Index i runs 0..N-1 here; the
 * paper is 1-based, so its "a*i" (Eq. xy, y^(1)) is a*(i+1) below.
 *
 * Attended set A(i): {0..i} with the causal mask, {0..N-1} without it
 * (Sec. 2.2; the causal form is the one whose sums stop at i, as in Eq. div).
 *
 * Two independent evaluations of every quantity are provided so that the
 * tests can cross-check them:
 *   *_def : the plain definition, O(N^2 D)   (Sec. 2.2, Eq. div / fijgi;
 *           gradients from Eq. bound and the chain rule of Sec. 3.2)
 *   *_rec : the running-sum factorisation, O(N D^2)
 *           (Eq. fglast / xy for the forward; Eq. back1 / back2 / endd for the
 *           backward; the state is the RNN form of App. B.1: S = sum k v^T,
 *           z = sum k)
 *
 * Parallelism: OpenMP over the independent (batch*head) index only.
 */
#include <stddef.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

int la_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static double dot(const double *x, const double *y, int D)
{
    double s = 0.0;
    for (int m = 0; m < D; ++m) s += x[m] * y[m];
    return s;
}

/* ------------------------------------------------------------------------ */
/* Forward, definition (Sec. 2.2; Eq. div, fijgi):                           */
/*   w_in = a + b q_i.k_n ; g_i = sum_{n in A(i)} w_in ;                     */
/*   o_i  = sum_{n in A(i)} w_in v_n / g_i                                   */
/* ------------------------------------------------------------------------ */
void la_oracle_forward_def(const double *Q, const double *K, const double *V,
                           double *O, double *G,
                           long BH, long N, int D, double a, double b, int causal)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (long bh = 0; bh < BH; ++bh) {
        const double *q = Q + bh * N * D, *k = K + bh * N * D, *v = V + bh * N * D;
        double *o = O + bh * N * D, *g = G + bh * N;
        double *f = (double *)malloc(sizeof(double) * (size_t)D);
        for (long i = 0; i < N; ++i) {
            long last = causal ? i : N - 1;
            double gi = 0.0;
            for (int j = 0; j < D; ++j) f[j] = 0.0;
            for (long n = 0; n <= last; ++n) {
                double w = a + b * dot(q + i * D, k + n * D, D);
                gi += w;
                for (int j = 0; j < D; ++j) f[j] += w * v[n * D + j];
            }
            g[i] = gi;
            for (int j = 0; j < D; ++j) o[i * D + j] = f[j] / gi;
        }
        free(f);
    }
}

/* Definition evaluated only at selected rows of one (batch*head) slice:
 * rows[r] in [0, N).  q,k,v point at that slice ([N, D]).  O(rows * N * D). */
void la_oracle_forward_def_rows(const double *q, const double *k, const double *v,
                                const long *rows, long nrows,
                                double *o_rows, double *g_rows,
                                long N, int D, double a, double b, int causal)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (long r = 0; r < nrows; ++r) {
        long i = rows[r];
        long last = causal ? i : N - 1;
        double gi = 0.0;
        double *f = o_rows + r * D;
        for (int j = 0; j < D; ++j) f[j] = 0.0;
        for (long n = 0; n <= last; ++n) {
            double w = a + b * dot(q + i * D, k + n * D, D);
            gi += w;
            for (int j = 0; j < D; ++j) f[j] += w * v[n * D + j];
        }
        g_rows[r] = gi;
        for (int j = 0; j < D; ++j) f[j] /= gi;
    }
}

/* ------------------------------------------------------------------------ */
/* Forward, running sums (Eq. fglast, xy; App. B.1).  State per slice:       */
/*   S[m][j] = sum k_nm v_nj, z[m] = sum k_nm, p[j] = sum v_nj, cnt = |A|    */
/* so that x^(1) = a p, x^(2) = b S, y^(1) = a cnt, y^(2) = b z.             */
/* Causal: row i is added to the state before it is read out (the sums in    */
/* Eq. xy include n = i).  Non-causal: all rows are added first.             */
/* ------------------------------------------------------------------------ */
static void state_add_row(double *S, double *z, double *p,
                          const double *k, const double *v, int D)
{
    for (int m = 0; m < D; ++m) {
        z[m] += k[m];
        for (int j = 0; j < D; ++j) S[m * D + j] += k[m] * v[j];
    }
    for (int j = 0; j < D; ++j) p[j] += v[j];
}

static void readout_row(const double *S, const double *z, const double *p, double cnt,
                        const double *q, double *o, double *g, int D, double a, double b)
{
    double gi = a * cnt + b * dot(q, z, D);
    for (int j = 0; j < D; ++j) {
        double lin = 0.0;
        for (int m = 0; m < D; ++m) lin += q[m] * S[m * D + j];
        o[j] = (a * p[j] + b * lin) / gi;
    }
    *g = gi;
}

void la_oracle_forward_rec(const double *Q, const double *K, const double *V,
                           double *O, double *G,
                           long BH, long N, int D, double a, double b, int causal)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (long bh = 0; bh < BH; ++bh) {
        const double *q = Q + bh * N * D, *k = K + bh * N * D, *v = V + bh * N * D;
        double *o = O + bh * N * D, *g = G + bh * N;
        double *S = (double *)calloc((size_t)D * D + 2 * (size_t)D, sizeof(double));
        double *z = S + (size_t)D * D, *p = z + D;
        if (causal) {
            for (long i = 0; i < N; ++i) {
                state_add_row(S, z, p, k + i * D, v + i * D, D);
                readout_row(S, z, p, (double)(i + 1), q + i * D, o + i * D, g + i, D, a, b);
            }
        } else {
            for (long i = 0; i < N; ++i) state_add_row(S, z, p, k + i * D, v + i * D, D);
            for (long i = 0; i < N; ++i)
                readout_row(S, z, p, (double)N, q + i * D, o + i * D, g + i, D, a, b);
        }
        free(S);
    }
}

/* ------------------------------------------------------------------------ */
/* Backward, definition.  With L = sum_ij o_ij Omega_ij (Omega = dO):        */
/*   dL/dw_in = sum_j Omega_ij (v_nj - o_ij) / g_i        (Eq. bound, / b)   */
/*            = OmegaHat_i . v_n - delta_i,  OmegaHat = Omega / g (Eq. back2),*/
/*              delta_i = o_i . OmegaHat_i                                    */
/*   dq_i += b c_in k_n ; dk_n += b c_in q_i ; dv_n += w_in OmegaHat_i        */
/* for every pair (i, n in A(i)); key/value n receives from the rows i that   */
/* attend to it (i >= n under the causal mask).  O and G are recomputed here  */
/* from the definition.                                                       */
/* ------------------------------------------------------------------------ */
void la_oracle_backward_def(const double *Q, const double *K, const double *V,
                            const double *dO, double *dQ, double *dK, double *dV,
                            long BH, long N, int D, double a, double b, int causal)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (long bh = 0; bh < BH; ++bh) {
        const double *q = Q + bh * N * D, *k = K + bh * N * D, *v = V + bh * N * D;
        const double *om = dO + bh * N * D;
        double *dq = dQ + bh * N * D, *dk = dK + bh * N * D, *dv = dV + bh * N * D;
        double *w = (double *)malloc(sizeof(double) * (size_t)(N + 2 * D));
        double *oi = w + N, *oh = oi + D;
        memset(dq, 0, sizeof(double) * (size_t)N * D);
        memset(dk, 0, sizeof(double) * (size_t)N * D);
        memset(dv, 0, sizeof(double) * (size_t)N * D);
        for (long i = 0; i < N; ++i) {
            long last = causal ? i : N - 1;
            double gi = 0.0;
            for (int j = 0; j < D; ++j) oi[j] = 0.0;
            for (long n = 0; n <= last; ++n) {
                w[n] = a + b * dot(q + i * D, k + n * D, D);
                gi += w[n];
                for (int j = 0; j < D; ++j) oi[j] += w[n] * v[n * D + j];
            }
            double delta = 0.0;
            for (int j = 0; j < D; ++j) {
                oi[j] /= gi;
                oh[j] = om[i * D + j] / gi;
                delta += oi[j] * oh[j];
            }
            for (long n = 0; n <= last; ++n) {
                double c = dot(oh, v + n * D, D) - delta;
                for (int r = 0; r < D; ++r) {
                    dq[i * D + r] += b * c * k[n * D + r];
                    dk[n * D + r] += b * c * q[i * D + r];
                }
                for (int j = 0; j < D; ++j) dv[n * D + j] += w[n] * oh[j];
            }
        }
        free(w);
    }
}

/* ------------------------------------------------------------------------ */
/* Backward, running sums (Eq. back1, back2, endd), with the stored set       */
/* {Q, K, V, O, g} of Sec. 3.2.  In state form:                               */
/*   alpha^Q = b S, beta^Q = b z          (forward-running, rows n <= i)      */
/*   alpha^K = beta^V = b R, R = sum q_m OmegaHat_m^T                         */
/*   sum_j beta^K = b u,   u = sum delta_m q_m                                */
/*   alpha^V = a w,        w = sum OmegaHat_m     (reverse-running, m >= i)   */
/*   dq_i = b (S_i OmegaHat_i - delta_i z_i)                                  */
/*   dk_i = b (R_i v_i - u_i)                                                 */
/*   dv_i = a w_i + b R_i^T k_i                                               */
/* Row i enters the running state before it is used (both sweeps include i).  */
/* Without the mask every state is the sum over all rows.                     */
/* ------------------------------------------------------------------------ */
void la_oracle_backward_rec(const double *Q, const double *K, const double *V,
                            const double *O, const double *G, const double *dO,
                            double *dQ, double *dK, double *dV,
                            long BH, long N, int D, double a, double b, int causal)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (long bh = 0; bh < BH; ++bh) {
        const double *q = Q + bh * N * D, *k = K + bh * N * D, *v = V + bh * N * D;
        const double *o = O + bh * N * D, *g = G + bh * N, *om = dO + bh * N * D;
        double *dq = dQ + bh * N * D, *dk = dK + bh * N * D, *dv = dV + bh * N * D;
        size_t DD = (size_t)D * D;
        double *S = (double *)calloc(2 * DD + 5 * (size_t)D, sizeof(double));
        double *R = S + DD, *z = R + DD, *p = z + D, *u = p + D, *wv = u + D, *oh = wv + D;

        /* forward-running sweep: dQ */
        if (!causal)
            for (long i = 0; i < N; ++i) state_add_row(S, z, p, k + i * D, v + i * D, D);
        for (long i = 0; i < N; ++i) {
            if (causal) state_add_row(S, z, p, k + i * D, v + i * D, D);
            double delta = 0.0;
            for (int j = 0; j < D; ++j) {
                oh[j] = om[i * D + j] / g[i];
                delta += o[i * D + j] * oh[j];
            }
            for (int r = 0; r < D; ++r)
                dq[i * D + r] = b * (dot(S + (size_t)r * D, oh, D) - delta * z[r]);
        }

        /* reverse-running sweep: dK, dV */
        if (!causal) {
            for (long i = 0; i < N; ++i) {
                double delta = 0.0;
                for (int j = 0; j < D; ++j) {
                    oh[j] = om[i * D + j] / g[i];
                    delta += o[i * D + j] * oh[j];
                }
                for (int r = 0; r < D; ++r) {
                    u[r] += delta * q[i * D + r];
                    for (int j = 0; j < D; ++j) R[(size_t)r * D + j] += q[i * D + r] * oh[j];
                }
                for (int j = 0; j < D; ++j) wv[j] += oh[j];
            }
        }
        for (long i = N - 1; i >= 0; --i) {
            if (causal) {
                double delta = 0.0;
                for (int j = 0; j < D; ++j) {
                    oh[j] = om[i * D + j] / g[i];
                    delta += o[i * D + j] * oh[j];
                }
                for (int r = 0; r < D; ++r) {
                    u[r] += delta * q[i * D + r];
                    for (int j = 0; j < D; ++j) R[(size_t)r * D + j] += q[i * D + r] * oh[j];
                }
                for (int j = 0; j < D; ++j) wv[j] += oh[j];
            }
            for (int r = 0; r < D; ++r)
                dk[i * D + r] = b * (dot(R + (size_t)r * D, v + i * D, D) - u[r]);
            for (int j = 0; j < D; ++j) {
                double s = 0.0;
                for (int r = 0; r < D; ++r) s += R[(size_t)r * D + j] * k[i * D + r];
                dv[i * D + j] = a * wv[j] + b * s;
            }
        }
        free(S);
    }
}

/* ------------------------------------------------------------------------ */
/* Incremental (decode) form: the recurrence of App. B.1 (Table 3, row 2)    */
/* with the state carried by the caller.  state = [S (D*D) | z (D) | p (D) | */
/* cnt (1)] per slice, the sums of Eq. xy over every row seen so far (zeros   */
/* for an empty prefix).  Each of the T new rows is added to the state, then  */
/* read out: o_t = (a p + b S^T q_t) / g_t, g_t = a cnt + b q_t.z (Eq. fglast,*/
/* div).  Always causal: a new row sees the prefix and itself.                */
/* ------------------------------------------------------------------------ */
void la_oracle_decode(const double *Q, const double *K, const double *V,
                      double *O, double *G, double *state,
                      long BH, long T, int D, double a, double b)
{
    const size_t SF = (size_t)D * D + 2 * (size_t)D + 1;
#pragma omp parallel for schedule(dynamic, 1)
    for (long bh = 0; bh < BH; ++bh) {
        const double *q = Q + bh * T * D, *k = K + bh * T * D, *v = V + bh * T * D;
        double *o = O + bh * T * D, *g = G + bh * T;
        double *S = state + (size_t)bh * SF, *z = S + (size_t)D * D, *p = z + D, *cnt = p + D;
        for (long t = 0; t < T; ++t) {
            state_add_row(S, z, p, k + t * D, v + t * D, D);
            *cnt += 1.0;
            readout_row(S, z, p, *cnt, q + t * D, o + t * D, g + t, D, a, b);
        }
    }
}

/* ------------------------------------------------------------------------ */
/* Gradients of L = sum_ij o_ij Omega_ij with respect to the kernel's own     */
/* coefficients (Sec. 2.2 allows a, b to be learnable), by the definition:    */
/* with w_in = a + b s_in, s_in = q_i.k_n, dw/da = 1 and dw/db = s_in, and    */
/* dL/dw_in = OmegaHat_i . v_n - delta_i as above,                            */
/*   dL/da = sum_{i, n in A(i)} (OmegaHat_i . v_n - delta_i)                  */
/*   dL/db = sum_{i, n in A(i)} (OmegaHat_i . v_n - delta_i) s_in             */
/* dab[0] = dL/da, dab[1] = dL/db, summed over all slices.  O(N^2 D).         */
/* ------------------------------------------------------------------------ */
void la_oracle_grad_ab_def(const double *Q, const double *K, const double *V,
                           const double *dO, double *dab,
                           long BH, long N, int D, double a, double b, int causal)
{
    double da = 0.0, db = 0.0;
#pragma omp parallel for schedule(dynamic, 1) reduction(+ : da, db)
    for (long bh = 0; bh < BH; ++bh) {
        const double *q = Q + bh * N * D, *k = K + bh * N * D, *v = V + bh * N * D;
        const double *om = dO + bh * N * D;
        double *s = (double *)malloc(sizeof(double) * (size_t)(N + 2 * D));
        double *oi = s + N, *oh = oi + D;
        for (long i = 0; i < N; ++i) {
            long last = causal ? i : N - 1;
            double gi = 0.0;
            for (int j = 0; j < D; ++j) oi[j] = 0.0;
            for (long n = 0; n <= last; ++n) {
                s[n] = dot(q + i * D, k + n * D, D);
                double w = a + b * s[n];
                gi += w;
                for (int j = 0; j < D; ++j) oi[j] += w * v[n * D + j];
            }
            double delta = 0.0;
            for (int j = 0; j < D; ++j) {
                oi[j] /= gi;
                oh[j] = om[i * D + j] / gi;
                delta += oi[j] * oh[j];
            }
            for (long n = 0; n <= last; ++n) {
                double c = dot(oh, v + n * D, D) - delta;
                da += c;
                db += c * s[n];
            }
        }
        free(s);
    }
    dab[0] = da;
    dab[1] = db;
}

/* ------------------------------------------------------------------------ */
/* Row normalisation of Q and K before the attention (Sec. 3.3): every row    */
/* x is replaced by xhat = x / ||x||_2.  Backward of that map for one row:    */
/* with the gradient dxhat with respect to xhat,                              */
/*   dx = (dxhat - xhat (xhat . dxhat)) / ||x||                               */
/* (the Jacobian of x / ||x|| is (I - xhat xhat^T) / ||x||).                  */
/* X, Y: [rows, D].                                                           */
/* ------------------------------------------------------------------------ */
void la_oracle_normalise_rows(const double *X, double *Xhat, long rows, int D)
{
#pragma omp parallel for schedule(static)
    for (long i = 0; i < rows; ++i) {
        const double *x = X + i * D;
        double nrm = 0.0;
        for (int m = 0; m < D; ++m) nrm += x[m] * x[m];
        nrm = __builtin_sqrt(nrm);
        for (int m = 0; m < D; ++m) Xhat[i * D + m] = x[m] / nrm;
    }
}

void la_oracle_normalise_rows_backward(const double *X, const double *dXhat, double *dX,
                                       long rows, int D)
{
#pragma omp parallel for schedule(static)
    for (long i = 0; i < rows; ++i) {
        const double *x = X + i * D, *dh = dXhat + i * D;
        double nrm = 0.0, proj = 0.0;
        for (int m = 0; m < D; ++m) nrm += x[m] * x[m];
        nrm = __builtin_sqrt(nrm);
        for (int m = 0; m < D; ++m) proj += (x[m] / nrm) * dh[m];
        for (int m = 0; m < D; ++m) dX[i * D + m] = (dh[m] - (x[m] / nrm) * proj) / nrm;
    }
}
