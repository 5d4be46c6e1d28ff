/*
 * xkv_oracle.c -- plain, slow, double-precision CPU oracle for xKV Selective
 * Reconstruction (SR) decode attention over a cross-layer factorized KV cache.
 *
 * THIS IS TEST INFRASTRUCTURE.  It exists to check the GPU library and to be
 * timed as a CPU baseline.  It shares no code with the GPU path, is never
 * called by it, and is "obviously correct" on purpose: straight loops in the
 * paper's notation, no blocking, no fusion, no reordering.
 *
 * Notation (paper, Sec. 2.1 "Notation", Sec. 3.1 Eq. 1-2, App. C.6 "Setup"):
 *   L      tokens in the compressed context
 *   H_kv   KV heads, H_q query heads, d_h per-head width, d = H_kv*d_h
 *   rho(h) GQA map, contiguous groups: rho(h) = h / (H_q/H_kv)
 *   A^K    [L][r_K]  shared key token basis of one layer group (A = U*Sigma)
 *   A^V    [L][r_V]  shared value token basis
 *   B^K_l  [r_K][d]  key reconstruction matrix of layer l, head block g is
 *                    columns g*d_h .. g*d_h+d_h-1 (Eq. 2)
 *   B^V_l  [r_V][d]
 *   q      [H_q][d_h] the decode-step queries of layer l
 *
 * All matrices are row-major double.  Callers widen fp32 / bf16 inputs to
 * double exactly before calling; nothing in here rounds an intermediate.
 * The one place where single precision appears is selection: the pooled
 * score is rounded once to fp32 and ordered by its fp32 bit pattern, because
 * that decision is taken in the kernel's precision on both sides.
 *
 * Parity pins (tests/test_oracle_pins.py): every function below is pinned by
 * an identity, a brute force or a library routine that is not this file.
 * No numeric SR output is printed anywhere in the paper, so the end-to-end
 * numbers themselves are "parity unpinned by a printed value"; they are
 * pinned by the k = L identity (SR equals dense attention on K = A B) and by
 * brute force on tiny inputs.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_API __attribute__((visibility("default")))

/* number of threads an OpenMP region of this library will use */
ORACLE_API int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------ */
/* Step 1 -- project the queries into the rank space.                  */
/* p_h = B^K_{l,rho(h)} q_h  in R^{r_K}.  Follows from Eq. 3 by        */
/* associativity: q_h . (A[t,:] B_{l,g}) = A[t,:] . (B_{l,g} q_h).      */
/* ------------------------------------------------------------------ */
ORACLE_API void oracle_project(const double *B_k, /* [r_k][d] */
                               const double *q,   /* [H_q][d_h] */
                               int r_k, int H_kv, int H_q, int d_h,
                               double *p /* [H_q][r_k] */)
{
    const int d = H_kv * d_h;
    const int n_rep = H_q / H_kv;
    for (int h = 0; h < H_q; ++h) {
        const int g = h / n_rep;
        for (int i = 0; i < r_k; ++i) {
            double acc = 0.0;
            for (int j = 0; j < d_h; ++j)
                acc += B_k[(size_t)i * d + (size_t)g * d_h + j] * q[(size_t)h * d_h + j];
            p[(size_t)h * r_k + i] = acc;
        }
    }
}

/* ------------------------------------------------------------------ */
/* Step 2 -- low-rank scores of every token.                           */
/* s[h,t] = scale * A^K[t,:] . p_h     (scale = 1/sqrt(d_h), Alg. 2    */
/* "scores" step; here applied per token to the factors).              */
/* ------------------------------------------------------------------ */
ORACLE_API void oracle_scores(const double *A_k, /* [L][r_k] */
                              const double *p,   /* [H_q][r_k] */
                              int L, int r_k, int H_q, double scale,
                              double *s /* [H_q][L] */)
{
#pragma omp parallel for schedule(static)
    for (int h = 0; h < H_q; ++h) {
        for (int t = 0; t < L; ++t) {
            double acc = 0.0;
            for (int i = 0; i < r_k; ++i)
                acc += A_k[(size_t)t * r_k + i] * p[(size_t)h * r_k + i];
            s[(size_t)h * L + t] = scale * acc;
        }
    }
}

/* ------------------------------------------------------------------ */
/* Step 3 -- pool from query heads to KV heads (Alg. 2, GQA pooling):  */
/* S[g,t] = max over h with rho(h) = g of s[h,t].                      */
/* ------------------------------------------------------------------ */
ORACLE_API void oracle_pool(const double *s, /* [H_q][L] */
                            int L, int H_kv, int H_q,
                            double *S /* [H_kv][L] */)
{
    const int n_rep = H_q / H_kv;
    for (int g = 0; g < H_kv; ++g) {
        for (int t = 0; t < L; ++t) {
            double m = s[(size_t)(g * n_rep) * L + t];
            for (int h = g * n_rep + 1; h < (g + 1) * n_rep; ++h) {
                const double v = s[(size_t)h * L + t];
                if (v > m) m = v;
            }
            S[(size_t)g * L + t] = m;
        }
    }
}

/* ------------------------------------------------------------------ */
/* Step 4 -- ArgTopK per KV head (Alg. 2, top-k step) by full sort.    */
/* Total order: fp32 value descending, ties (equal bit-order key) by   */
/* index ascending.  The key is the usual monotone unsigned image of   */
/* the IEEE-754 single bit pattern, so -0.0 < +0.0; no NaNs by         */
/* contract.  Output: the k selected indices in ascending index order. */
/* ------------------------------------------------------------------ */
static uint32_t order_key_f32(float x)
{
    uint32_t u;
    memcpy(&u, &x, sizeof u);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

typedef struct {
    uint32_t key;
    int32_t idx;
} keyed_t;

static int cmp_key_desc_idx_asc(const void *a, const void *b)
{
    const keyed_t *x = (const keyed_t *)a, *y = (const keyed_t *)b;
    if (x->key != y->key) return (x->key > y->key) ? -1 : 1;
    if (x->idx != y->idx) return (x->idx < y->idx) ? -1 : 1;
    return 0;
}

static int cmp_i32_asc(const void *a, const void *b)
{
    const int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

ORACLE_API int oracle_select(const float *S_row, /* [L] */
                             int L, int k,
                             int32_t *idx /* [k], ascending */)
{
    if (k < 0 || k > L) return -1;
    keyed_t *e = (keyed_t *)malloc((size_t)(L > 0 ? L : 1) * sizeof *e);
    if (!e) return -2;
    for (int t = 0; t < L; ++t) {
        e[t].key = order_key_f32(S_row[t]);
        e[t].idx = t;
    }
    qsort(e, (size_t)L, sizeof *e, cmp_key_desc_idx_asc);
    for (int m = 0; m < k; ++m) idx[m] = e[m].idx;
    qsort(idx, (size_t)k, sizeof *idx, cmp_i32_asc);
    free(e);
    return 0;
}

/* ------------------------------------------------------------------ */
/* Dense reconstruction X^_l = A B_l for all L tokens (Sec. 3.2).      */
/* ------------------------------------------------------------------ */
ORACLE_API void oracle_reconstruct(const double *A, /* [L][r] */
                                   const double *B, /* [r][d] */
                                   int L, int r, int d,
                                   double *X /* [L][d] */)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < L; ++t) {
        for (int j = 0; j < d; ++j) {
            double acc = 0.0;
            for (int i = 0; i < r; ++i)
                acc += A[(size_t)t * r + i] * B[(size_t)i * d + j];
            X[(size_t)t * d + j] = acc;
        }
    }
}

/* ------------------------------------------------------------------ */
/* Steps 5-6 -- selective reconstruction (Eq. 3) and softmax attention */
/* over the selected rows, for every KV head g and every query head h  */
/* with rho(h) = g:                                                    */
/*   K^_g[m,:] = A^K[I_g[m],:] B^K_{l,g},  V^_g likewise,              */
/*   z_m = scale * K^_g[m,:] . q_h,  w = softmax(z),  o_h = w^T V^_g.   */
/* Softmax is max-subtracted, natural exp, no mask.                    */
/* ------------------------------------------------------------------ */
ORACLE_API int oracle_gather_attend(const double *A_k, /* [L][r_k] */
                                    const double *A_v, /* [L][r_v] */
                                    const double *B_k, /* [r_k][d] */
                                    const double *B_v, /* [r_v][d] */
                                    const double *q,   /* [H_q][d_h] */
                                    const int32_t *idx, /* [H_kv][k] */
                                    int L, int r_k, int r_v, int H_kv, int H_q, int d_h,
                                    int k, double scale,
                                    double *out /* [H_q][d_h] */)
{
    const int d = H_kv * d_h;
    const int n_rep = H_q / H_kv;
    int bad = 0;
#pragma omp parallel for schedule(static)
    for (int g = 0; g < H_kv; ++g) {
        double *Khat = (double *)malloc((size_t)k * d_h * sizeof(double));
        double *Vhat = (double *)malloc((size_t)k * d_h * sizeof(double));
        double *z = (double *)malloc((size_t)k * sizeof(double));
        if (!Khat || !Vhat || !z) {
            bad = 1;
            free(Khat); free(Vhat); free(z);
            continue;
        }
        /* Eq. 3, one selected row at a time */
        for (int m = 0; m < k; ++m) {
            const int t = idx[(size_t)g * k + m];
            if (t < 0 || t >= L) { bad = 1; continue; }
            for (int j = 0; j < d_h; ++j) {
                double ak = 0.0, av = 0.0;
                for (int i = 0; i < r_k; ++i)
                    ak += A_k[(size_t)t * r_k + i] * B_k[(size_t)i * d + (size_t)g * d_h + j];
                for (int i = 0; i < r_v; ++i)
                    av += A_v[(size_t)t * r_v + i] * B_v[(size_t)i * d + (size_t)g * d_h + j];
                Khat[(size_t)m * d_h + j] = ak;
                Vhat[(size_t)m * d_h + j] = av;
            }
        }
        for (int h = g * n_rep; h < (g + 1) * n_rep; ++h) {
            double zmax = -INFINITY;
            for (int m = 0; m < k; ++m) {
                double acc = 0.0;
                for (int j = 0; j < d_h; ++j)
                    acc += Khat[(size_t)m * d_h + j] * q[(size_t)h * d_h + j];
                z[m] = scale * acc;
                if (z[m] > zmax) zmax = z[m];
            }
            double denom = 0.0;
            for (int m = 0; m < k; ++m) {
                z[m] = exp(z[m] - zmax);
                denom += z[m];
            }
            for (int j = 0; j < d_h; ++j) {
                double acc = 0.0;
                for (int m = 0; m < k; ++m)
                    acc += z[m] * Vhat[(size_t)m * d_h + j];
                out[(size_t)h * d_h + j] = acc / denom;
            }
        }
        free(Khat); free(Vhat); free(z);
    }
    return bad ? -1 : 0;
}

/* ------------------------------------------------------------------ */
/* Textbook dense decode attention on given K, V (the speedup          */
/* baseline's definition): o_h = softmax(scale * K_{rho(h)} q_h)^T V.   */
/* K, V are [L][d] with head g in columns g*d_h..                       */
/* ------------------------------------------------------------------ */
ORACLE_API int oracle_dense(const double *K, /* [L][d] */
                            const double *V, /* [L][d] */
                            const double *q, /* [H_q][d_h] */
                            int L, int H_kv, int H_q, int d_h, double scale,
                            double *out /* [H_q][d_h] */)
{
    const int d = H_kv * d_h;
    const int n_rep = H_q / H_kv;
    int bad = 0;
#pragma omp parallel for schedule(static)
    for (int h = 0; h < H_q; ++h) {
        const int g = h / n_rep;
        double *z = (double *)malloc((size_t)L * sizeof(double));
        if (!z) { bad = 1; continue; }
        double zmax = -INFINITY;
        for (int t = 0; t < L; ++t) {
            double acc = 0.0;
            for (int j = 0; j < d_h; ++j)
                acc += K[(size_t)t * d + (size_t)g * d_h + j] * q[(size_t)h * d_h + j];
            z[t] = scale * acc;
            if (z[t] > zmax) zmax = z[t];
        }
        double denom = 0.0;
        for (int t = 0; t < L; ++t) {
            z[t] = exp(z[t] - zmax);
            denom += z[t];
        }
        for (int j = 0; j < d_h; ++j) {
            double acc = 0.0;
            for (int t = 0; t < L; ++t)
                acc += z[t] * V[(size_t)t * d + (size_t)g * d_h + j];
            out[(size_t)h * d_h + j] = acc / denom;
        }
        free(z);
    }
    return bad ? -1 : 0;
}

/* ------------------------------------------------------------------ */
/* The whole SR decode step for one layer of one sequence, steps 1-6   */
/* in order.  Optional outputs: S_out [H_kv][L] pooled scores as the   */
/* fp32 values the selection saw, idx_out [H_kv][k] ascending.         */
/* ------------------------------------------------------------------ */
ORACLE_API int oracle_sr_decode(const double *A_k, const double *A_v,
                                const double *B_k, const double *B_v,
                                const double *q,
                                int L, int r_k, int r_v, int H_kv, int H_q, int d_h,
                                int k, double scale,
                                double *out,      /* [H_q][d_h] */
                                int32_t *idx_out, /* nullable [H_kv][k] */
                                float *S_out /* nullable [H_kv][L] */)
{
    if (H_kv <= 0 || H_q % H_kv != 0 || k < 1 || k > L) return -1;
    double *p = (double *)malloc((size_t)H_q * r_k * sizeof(double));
    double *s = (double *)malloc((size_t)H_q * L * sizeof(double));
    double *S = (double *)malloc((size_t)H_kv * L * sizeof(double));
    float *S32 = (float *)malloc((size_t)H_kv * L * sizeof(float));
    int32_t *idx = (int32_t *)malloc((size_t)H_kv * k * sizeof(int32_t));
    int rc = -2;
    if (p && s && S && S32 && idx) {
        oracle_project(B_k, q, r_k, H_kv, H_q, d_h, p);
        oracle_scores(A_k, p, L, r_k, H_q, scale, s);
        oracle_pool(s, L, H_kv, H_q, S);
        for (size_t e = 0; e < (size_t)H_kv * L; ++e) S32[e] = (float)S[e];
        rc = 0;
        for (int g = 0; g < H_kv && rc == 0; ++g)
            rc = oracle_select(S32 + (size_t)g * L, L, k, idx + (size_t)g * k);
        if (rc == 0)
            rc = oracle_gather_attend(A_k, A_v, B_k, B_v, q, idx, L, r_k, r_v,
                                      H_kv, H_q, d_h, k, scale, out);
        if (rc == 0 && idx_out) memcpy(idx_out, idx, (size_t)H_kv * k * sizeof(int32_t));
        if (rc == 0 && S_out) memcpy(S_out, S32, (size_t)H_kv * L * sizeof(float));
    }
    free(p); free(s); free(S); free(S32); free(idx);
    return rc;
}

/* ------------------------------------------------------------------ */
/* Cross-Layer Factorization (Eq. 1): exact rank-r truncated SVD of    */
/* X_cat [L][n], n = G*d, written as A = U Sigma [L][r] and            */
/* B = V_r^T [r][n] (layer l's B_l is columns l*d .. l*d+d-1).          */
/* Route: cyclic Jacobi eigen-decomposition of the n x n Gram matrix   */
/* X^T X = V Lambda V^T, eigenvalues sorted descending, A = X V_r.      */
/* Meant for small n only (tests).                                     */
/* ------------------------------------------------------------------ */
ORACLE_API int oracle_factorize(const double *X, /* [L][n] */
                                int L, int n, int r,
                                double *A, /* [L][r] */
                                double *B, /* [r][n] */
                                double *sigma /* nullable [n], all singular values desc */)
{
    if (r < 1 || r > n) return -1;
    double *Gm = (double *)calloc((size_t)n * n, sizeof(double));
    double *Vm = (double *)calloc((size_t)n * n, sizeof(double));
    int *order = (int *)malloc((size_t)n * sizeof(int));
    if (!Gm || !Vm || !order) { free(Gm); free(Vm); free(order); return -2; }
    for (int a = 0; a < n; ++a)
        for (int b = a; b < n; ++b) {
            double acc = 0.0;
            for (int t = 0; t < L; ++t) acc += X[(size_t)t * n + a] * X[(size_t)t * n + b];
            Gm[(size_t)a * n + b] = acc;
            Gm[(size_t)b * n + a] = acc;
        }
    for (int a = 0; a < n; ++a) Vm[(size_t)a * n + a] = 1.0;
    /* cyclic Jacobi sweeps: rotate away each off-diagonal pair in turn */
    for (int sweep = 0; sweep < 100; ++sweep) {
        double off = 0.0, diag = 0.0;
        for (int a = 0; a < n; ++a) {
            diag += Gm[(size_t)a * n + a] * Gm[(size_t)a * n + a];
            for (int b = a + 1; b < n; ++b) off += Gm[(size_t)a * n + b] * Gm[(size_t)a * n + b];
        }
        if (off <= 1e-30 * (diag + 1e-300)) break;
        for (int a = 0; a < n - 1; ++a)
            for (int b = a + 1; b < n; ++b) {
                const double gab = Gm[(size_t)a * n + b];
                if (gab == 0.0) continue;
                const double gaa = Gm[(size_t)a * n + a], gbb = Gm[(size_t)b * n + b];
                const double theta = (gbb - gaa) / (2.0 * gab);
                const double tt = (theta >= 0.0 ? 1.0 : -1.0) / (fabs(theta) + sqrt(theta * theta + 1.0));
                const double c = 1.0 / sqrt(tt * tt + 1.0), sn = tt * c;
                for (int m = 0; m < n; ++m) { /* columns a,b of G */
                    const double x = Gm[(size_t)m * n + a], y = Gm[(size_t)m * n + b];
                    Gm[(size_t)m * n + a] = c * x - sn * y;
                    Gm[(size_t)m * n + b] = sn * x + c * y;
                }
                for (int m = 0; m < n; ++m) { /* rows a,b of G */
                    const double x = Gm[(size_t)a * n + m], y = Gm[(size_t)b * n + m];
                    Gm[(size_t)a * n + m] = c * x - sn * y;
                    Gm[(size_t)b * n + m] = sn * x + c * y;
                }
                for (int m = 0; m < n; ++m) { /* accumulate eigenvectors */
                    const double x = Vm[(size_t)m * n + a], y = Vm[(size_t)m * n + b];
                    Vm[(size_t)m * n + a] = c * x - sn * y;
                    Vm[(size_t)m * n + b] = sn * x + c * y;
                }
            }
    }
    /* sort eigenpairs by eigenvalue descending (selection sort on an index) */
    for (int a = 0; a < n; ++a) order[a] = a;
    for (int a = 0; a < n - 1; ++a) {
        int best = a;
        for (int b = a + 1; b < n; ++b)
            if (Gm[(size_t)order[b] * n + order[b]] > Gm[(size_t)order[best] * n + order[best]]) best = b;
        const int tmp = order[a]; order[a] = order[best]; order[best] = tmp;
    }
    if (sigma)
        for (int a = 0; a < n; ++a) {
            const double lam = Gm[(size_t)order[a] * n + order[a]];
            sigma[a] = lam > 0.0 ? sqrt(lam) : 0.0;
        }
    for (int i = 0; i < r; ++i)
        for (int c = 0; c < n; ++c) B[(size_t)i * n + c] = Vm[(size_t)c * n + order[i]];
    for (int t = 0; t < L; ++t)
        for (int i = 0; i < r; ++i) {
            double acc = 0.0;
            for (int c = 0; c < n; ++c) acc += X[(size_t)t * n + c] * B[(size_t)i * n + c];
            A[(size_t)t * r + i] = acc;
        }
    free(Gm); free(Vm); free(order);
    return 0;
}

/* ------------------------------------------------------------------ */
/* Memory model and compression ratios (App. C.6, "Compressed-cache    */
/* memory" and "How we compute KV-Cache compression ratios").          */
/* N layers, W layers per window, n_win = ceil(N/W) windows, per-layer  */
/* KV width d, context L, landmark chunk c (alpha = 1/c).              */
/* which: 0 = C_K (factor-only, keys), 1 = C_V, 2 = xKV (keys and       */
/* values compressed, no landmarks) = 2/(1/C_K + 1/C_V),               */
/* 3 = xK-SR GPU = 2/(1/C_K + alpha), 4 = xK-SR total =                */
/* 2/(1/C_K + alpha + 1), 5 = xKV-SR = 2/(1/C_K + 1/C_V + alpha).       */
/* ------------------------------------------------------------------ */
ORACLE_API double oracle_compression_ratio(int which, int N, int W, int d, double L,
                                           int r_k, int r_v, int c)
{
    const int n_win = (N + W - 1) / W;
    const double full = (double)N * L * d;
    const double CK = full / ((double)n_win * L * r_k + (double)N * r_k * d);
    const double CV = r_v > 0 ? full / ((double)n_win * L * r_v + (double)N * r_v * d) : 0.0;
    const double alpha = c > 0 ? 1.0 / (double)c : 0.0;
    switch (which) {
    case 0: return CK;
    case 1: return CV;
    case 2: return 2.0 / (1.0 / CK + 1.0 / CV);
    case 3: return 2.0 / (1.0 / CK + alpha);
    case 4: return 2.0 / (1.0 / CK + alpha + 1.0);
    case 5: return 2.0 / (1.0 / CK + 1.0 / CV + alpha);
    default: return -1.0;
    }
}
