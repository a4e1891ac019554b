/*
 * fp64 CPU oracle for signatures of piecewise-linear paths.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing on the product path may call, link or
 * import this file; it exists so that the GPU library has something
 * independent to be compared with.  It shares no code with the GPU library.
 *
 * Two routes, both plain and slow on purpose:
 *
 *   dense  - the signature as an element of the truncated tensor algebra
 *            T_{<=N}(R^d) (Section 2.1): per segment the tensor exponential
 *            exp(dX) (Proposition 3.1) is built level by level and multiplied
 *            on the right with the truncated Cauchy product (Definition of the
 *            product in Section 2.1, Chen's relation, Theorem 3.2 / eq. 2).
 *   words  - eq. 3 evaluated word by word over a prefix-closed set, with the
 *            word-indexed exponential coefficients of Section 3 multiplied
 *            out explicitly for every prefix/suffix split.
 *
 * The backward functions are ordinary reverse-mode differentiation of those
 * two forward routes with every intermediate signature S_{0,t_j} kept in
 * memory (no reconstruction), followed by the increments-to-points chain
 * rule of Section 4.1.
 *
 * Inputs are the fp32 points the GPU also receives, widened to double here.
 * OpenMP is used only as "one path per thread".
 */
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int sig_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* pw[n] = d^n, off[n] = sum_{k<n} d^k (level 0 sits at offset 0), total = off[N+1] */
static void level_layout(int d, int N, size_t *pw, size_t *off)
{
    pw[0] = 1;
    off[0] = 0;
    for (int n = 1; n <= N + 1; ++n) {
        pw[n] = pw[n - 1] * (size_t)d;
        off[n] = off[n - 1] + pw[n - 1];
    }
}

/* E_0 = 1, E_n = E_{n-1} (x) dx / n   (Proposition 3.1: level n of exp(dx) is dx^{(x)n}/n!) */
static void tensor_exp(int d, int N, const size_t *pw, const size_t *off, const double *dx, double *E)
{
    E[0] = 1.0;
    for (int n = 1; n <= N; ++n)
        for (size_t v = 0; v < pw[n - 1]; ++v)
            for (int i = 0; i < d; ++i)
                E[off[n] + v * (size_t)d + (size_t)i] = E[off[n - 1] + v] * dx[i] / (double)n;
}

/* C = A (x) B truncated at level N:  c_n = sum_{k=0..n} a_k (x) b_{n-k} */
static void cauchy_product(int N, const size_t *pw, const size_t *off, const double *A, const double *B, double *C)
{
    for (int n = 0; n <= N; ++n) {
        double *c = C + off[n];
        for (size_t t = 0; t < pw[n]; ++t) c[t] = 0.0;
        for (int k = 0; k <= n; ++k) {
            const double *a = A + off[k];
            const double *b = B + off[n - k];
            for (size_t u = 0; u < pw[k]; ++u)
                for (size_t v = 0; v < pw[n - k]; ++v)
                    c[u * pw[n - k] + v] += a[u] * b[v];
        }
    }
}

size_t sig_oracle_dense_size(int d, int N)
{
    size_t pw[66], off[66];
    if (N > 63) return 0;
    level_layout(d, N, pw, off);
    return off[N + 1];
}

/* Exposed so that tests can check Chen's relation and the inverse property with the
 * oracle's own product:  C = A (x) B, each laid out [level 0 | level 1 | ... | level N]. */
void sig_oracle_tensor_product(int d, int N, const double *A, const double *B, double *C)
{
    size_t pw[66], off[66];
    level_layout(d, N, pw, off);
    cauchy_product(N, pw, off, A, B, C);
}

/*
 * Dense forward.  path: float [B, P, d] (P = L+1 points).  out: double [B, total]
 * INCLUDING level 0 (= 1) at index 0; the caller drops it.
 */
int sig_oracle_forward_dense(const float *path, int64_t B, int64_t P, int d, int N, double *out)
{
    size_t pw[66], off[66];
    if (d < 1 || N < 0 || N > 63 || P < 1) return -1;
    level_layout(d, N, pw, off);
    const size_t tot = off[N + 1];
    int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t b = 0; b < B; ++b) {
        double *S = (double *)malloc(tot * sizeof(double));
        double *T = (double *)malloc(tot * sizeof(double));
        double *E = (double *)malloc(tot * sizeof(double));
        double *dx = (double *)malloc((size_t)d * sizeof(double));
        if (!S || !T || !E || !dx) { fail = 1; free(S); free(T); free(E); free(dx); continue; }
        memset(S, 0, tot * sizeof(double));
        S[0] = 1.0;                                   /* S_{0,0} = 1 */
        const float *X = path + (size_t)b * (size_t)P * (size_t)d;
        for (int64_t j = 1; j < P; ++j) {
            for (int i = 0; i < d; ++i)
                dx[i] = (double)X[(size_t)j * d + i] - (double)X[(size_t)(j - 1) * d + i];
            tensor_exp(d, N, pw, off, dx, E);
            cauchy_product(N, pw, off, S, E, T);      /* S_{0,t_j} = S_{0,t_{j-1}} (x) exp(dX_j) */
            double *tmp = S; S = T; T = tmp;
        }
        memcpy(out + (size_t)b * tot, S, tot * sizeof(double));
        free(S); free(T); free(E); free(dx);
    }
    return fail ? -2 : 0;
}

/*
 * Dense backward.  grad: double [B, total] = dLoss/dS_{0,T} per dense entry (entry 0,
 * the level-0 slot, is ignored).  grad_path: double [B, P, d].
 * Keeps all P intermediate signatures of one path in memory.
 */
int sig_oracle_backward_dense(const float *path, const double *grad, int64_t B, int64_t P, int d, int N,
                              double *grad_path)
{
    size_t pw[66], off[66];
    if (d < 1 || N < 0 || N > 63 || P < 1) return -1;
    level_layout(d, N, pw, off);
    const size_t tot = off[N + 1];
    int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t b = 0; b < B; ++b) {
        double *Sall = (double *)malloc((size_t)P * tot * sizeof(double));   /* S_{0,t_j}, j = 0..L */
        double *E = (double *)malloc(tot * sizeof(double));
        double *Ebar = (double *)malloc(tot * sizeof(double));
        double *Sbar = (double *)malloc(tot * sizeof(double));
        double *Sbar_prev = (double *)malloc(tot * sizeof(double));
        double *dxbar = (double *)malloc((size_t)P * d * sizeof(double));    /* row j: dLoss/d dX_j, row 0 unused */
        double *dx = (double *)malloc((size_t)d * sizeof(double));
        if (!Sall || !E || !Ebar || !Sbar || !Sbar_prev || !dxbar || !dx) {
            fail = 1;
            free(Sall); free(E); free(Ebar); free(Sbar); free(Sbar_prev); free(dxbar); free(dx);
            continue;
        }
        const float *X = path + (size_t)b * (size_t)P * (size_t)d;
        memset(Sall, 0, tot * sizeof(double));
        Sall[0] = 1.0;
        for (int64_t j = 1; j < P; ++j) {
            for (int i = 0; i < d; ++i)
                dx[i] = (double)X[(size_t)j * d + i] - (double)X[(size_t)(j - 1) * d + i];
            tensor_exp(d, N, pw, off, dx, E);
            cauchy_product(N, pw, off, Sall + (size_t)(j - 1) * tot, E, Sall + (size_t)j * tot);
        }
        memcpy(Sbar, grad + (size_t)b * tot, tot * sizeof(double));
        Sbar[0] = 0.0;
        memset(dxbar, 0, (size_t)P * d * sizeof(double));
        for (int64_t j = P - 1; j >= 1; --j) {
            const double *Sp = Sall + (size_t)(j - 1) * tot;      /* S_{0,t_{j-1}} */
            for (int i = 0; i < d; ++i)
                dx[i] = (double)X[(size_t)j * d + i] - (double)X[(size_t)(j - 1) * d + i];
            tensor_exp(d, N, pw, off, dx, E);
            /* forward was  S'_n[u v] = sum_k S_k[u] E_{n-k}[v].  Reverse it: */
            memset(Sbar_prev, 0, tot * sizeof(double));
            memset(Ebar, 0, tot * sizeof(double));
            for (int n = 0; n <= N; ++n)
                for (int k = 0; k <= n; ++k)
                    for (size_t u = 0; u < pw[k]; ++u)
                        for (size_t v = 0; v < pw[n - k]; ++v) {
                            const double g = Sbar[off[n] + u * pw[n - k] + v];
                            Sbar_prev[off[k] + u] += g * E[off[n - k] + v];
                            Ebar[off[n - k] + v] += g * Sp[off[k] + u];
                        }
            /* forward was  E_m[v i] = E_{m-1}[v] dx[i] / m.  Reverse it from the top level down: */
            double *row = dxbar + (size_t)j * d;
            for (int m = N; m >= 1; --m)
                for (size_t v = 0; v < pw[m - 1]; ++v)
                    for (int i = 0; i < d; ++i) {
                        const double g = Ebar[off[m] + v * (size_t)d + (size_t)i];
                        Ebar[off[m - 1] + v] += g * dx[i] / (double)m;
                        row[i] += g * E[off[m - 1] + v] / (double)m;
                    }
            double *tmp = Sbar; Sbar = Sbar_prev; Sbar_prev = tmp;
        }
        /* dX_j = X_j - X_{j-1}  =>  dLoss/dX_j = dLoss/d dX_j - dLoss/d dX_{j+1}  (Section 4.1) */
        double *gp = grad_path + (size_t)b * (size_t)P * (size_t)d;
        for (int64_t j = 0; j < P; ++j)
            for (int i = 0; i < d; ++i) {
                const double here = (j >= 1) ? dxbar[(size_t)j * d + i] : 0.0;
                const double next = (j + 1 < P) ? dxbar[(size_t)(j + 1) * d + i] : 0.0;
                gp[(size_t)j * d + i] = here - next;
            }
        free(Sall); free(E); free(Ebar); free(Sbar); free(Sbar_prev); free(dxbar); free(dx);
    }
    return fail ? -2 : 0;
}

/*
 * Word route.  The prefix-closed set W has nw words; word w has letters
 * letters[offs[w] .. offs[w+1]) and prefix_idx[offs[w] + k - 1] is the index in W of
 * its prefix of length k (k = 1..n; the last entry is w itself).  The empty word
 * is not in W; its coefficient is the constant 1.
 *
 * eq. 3:  S_j(w) = sum_{k=0..n} S_{j-1}(w_[k]) * prod_{r=k+1..n} dX_j^{(w_r)} / (n-k)!
 */
static double inv_factorial(int m)
{
    double f = 1.0;
    for (int q = 2; q <= m; ++q) f *= (double)q;
    return 1.0 / f;
}

static void words_step(int64_t nw, const int32_t *letters, const int64_t *offs, const int64_t *prefix_idx,
                       const double *dx, const double *Sold, double *Snew)
{
    for (int64_t w = 0; w < nw; ++w) {
        const int64_t o = offs[w];
        const int n = (int)(offs[w + 1] - o);
        double acc = 0.0;
        for (int k = 0; k <= n; ++k) {
            const double left = (k == 0) ? 1.0 : Sold[prefix_idx[o + k - 1]];
            double e = inv_factorial(n - k);
            for (int r = k; r < n; ++r) e *= dx[letters[o + r]];
            acc += left * e;
        }
        Snew[w] = acc;
    }
}

int sig_oracle_forward_words(const float *path, int64_t B, int64_t P, int d, int64_t nw, const int32_t *letters,
                             const int64_t *offs, const int64_t *prefix_idx, double *out)
{
    if (d < 1 || P < 1 || nw < 0) return -1;
    int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t b = 0; b < B; ++b) {
        double *S = (double *)calloc((size_t)(nw ? nw : 1), sizeof(double));
        double *T = (double *)calloc((size_t)(nw ? nw : 1), sizeof(double));
        double *dx = (double *)malloc((size_t)d * sizeof(double));
        if (!S || !T || !dx) { fail = 1; free(S); free(T); free(dx); continue; }
        const float *X = path + (size_t)b * (size_t)P * (size_t)d;
        for (int64_t j = 1; j < P; ++j) {
            for (int i = 0; i < d; ++i)
                dx[i] = (double)X[(size_t)j * d + i] - (double)X[(size_t)(j - 1) * d + i];
            words_step(nw, letters, offs, prefix_idx, dx, S, T);
            double *tmp = S; S = T; T = tmp;
        }
        memcpy(out + (size_t)b * (size_t)nw, S, (size_t)nw * sizeof(double));
        free(S); free(T); free(dx);
    }
    return fail ? -2 : 0;
}

int sig_oracle_backward_words(const float *path, const double *grad, int64_t B, int64_t P, int d, int64_t nw,
                              const int32_t *letters, const int64_t *offs, const int64_t *prefix_idx,
                              double *grad_path)
{
    if (d < 1 || P < 1 || nw < 0) return -1;
    int fail = 0;
    const size_t W = (size_t)(nw ? nw : 1);
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t b = 0; b < B; ++b) {
        double *Sall = (double *)calloc((size_t)P * W, sizeof(double));
        double *Sbar = (double *)malloc(W * sizeof(double));
        double *Sbar_prev = (double *)malloc(W * sizeof(double));
        double *dxbar = (double *)calloc((size_t)P * d, sizeof(double));
        double *dx = (double *)malloc((size_t)d * sizeof(double));
        if (!Sall || !Sbar || !Sbar_prev || !dxbar || !dx) {
            fail = 1;
            free(Sall); free(Sbar); free(Sbar_prev); free(dxbar); free(dx);
            continue;
        }
        const float *X = path + (size_t)b * (size_t)P * (size_t)d;
        for (int64_t j = 1; j < P; ++j) {
            for (int i = 0; i < d; ++i)
                dx[i] = (double)X[(size_t)j * d + i] - (double)X[(size_t)(j - 1) * d + i];
            words_step(nw, letters, offs, prefix_idx, dx, Sall + (size_t)(j - 1) * W, Sall + (size_t)j * W);
        }
        for (int64_t w = 0; w < nw; ++w) Sbar[w] = grad[(size_t)b * (size_t)nw + (size_t)w];
        for (int64_t j = P - 1; j >= 1; --j) {
            const double *Sp = Sall + (size_t)(j - 1) * W;
            double *row = dxbar + (size_t)j * d;
            for (int i = 0; i < d; ++i)
                dx[i] = (double)X[(size_t)j * d + i] - (double)X[(size_t)(j - 1) * d + i];
            memset(Sbar_prev, 0, W * sizeof(double));
            for (int64_t w = 0; w < nw; ++w) {
                const int64_t o = offs[w];
                const int n = (int)(offs[w + 1] - o);
                const double g = Sbar[w];
                for (int k = 0; k <= n; ++k) {
                    const double left = (k == 0) ? 1.0 : Sp[prefix_idx[o + k - 1]];
                    const double c = inv_factorial(n - k);
                    double e = c;
                    for (int r = k; r < n; ++r) e *= dx[letters[o + r]];
                    if (k >= 1) Sbar_prev[prefix_idx[o + k - 1]] += g * e;
                    /* derivative of the product of increments: drop one factor at a time */
                    for (int r = k; r < n; ++r) {
                        double rest = c;
                        for (int q = k; q < n; ++q)
                            if (q != r) rest *= dx[letters[o + q]];
                        row[letters[o + r]] += g * left * rest;
                    }
                }
            }
            double *tmp = Sbar; Sbar = Sbar_prev; Sbar_prev = tmp;
        }
        double *gp = grad_path + (size_t)b * (size_t)P * (size_t)d;
        for (int64_t j = 0; j < P; ++j)
            for (int i = 0; i < d; ++i) {
                const double here = (j >= 1) ? dxbar[(size_t)j * d + i] : 0.0;
                const double next = (j + 1 < P) ? dxbar[(size_t)(j + 1) * d + i] : 0.0;
                gp[(size_t)j * d + i] = here - next;
            }
        free(Sall); free(Sbar); free(Sbar_prev); free(dxbar); free(dx);
    }
    return fail ? -2 : 0;
}

void sig_oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n >= 1) omp_set_num_threads(n);
#else
    (void)n;
#endif
}
