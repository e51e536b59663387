/* Plain fp64 CPU oracle for the marginalized graph kernel, C edition.
 * TEST INFRASTRUCTURE: linked only by the tests, the smoke entry and the
 * CPU-baseline leg of the benchmark.  Shares no code with the HIP path.
 *
 * Tier 0 (dense): assembles the N x N system of paper Eq. 1 (Section II-B),
 *     S = D_x V_x^{-1} - A_x (.) E_x,  b = D_x q_x,  K = p_x^T S^{-1} b,
 *   entry by entry, and solves it by an unblocked Cholesky factorisation
 *   (S is SPD, Section II-B); a non-positive pivot is reported as an error.
 * Tier 1 (matrix-free): applies the same S edge pair by edge pair (the double
 *   loop of Alg. 2 with the A_ij A'_i'j' factor of the appendix listings) and
 *   runs plain conjugate gradients in fp64 to a relative residual of 1e-13;
 *   for sizes where S cannot be stored.
 *
 * Readings: product index (i,i') -> i*n'+i'; d_i = sum_j A_ij + q; q_i = q;
 * p_i = 1/n unless given; kappa_v = 1 if labels equal else h;
 * kappa_e = exp(-(e-e')^2 / (2 l^2)), or one of the other examples of Appendix B
 * chosen with mgk_oracle_set_edge_kernel (compact polynomial, Kronecker product
 * of square exponentials over label attributes, R-convolution over label parts).
 *
 * Parallelism (OpenMP) is over pairs in tier 0 and over rows of G inside a
 * pair in tier 1; it changes no arithmetic of a single pair in tier 0.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Edge base kernel in force (process-wide; the callers are single-threaded at this
 * level).  kind 0: square exponential with the length scale each call passes.
 * kind 1: compact polynomial, par = {rho, number of coefficients, c0, c1, ...}:
 *   sum_i c_i r^i for r = |e-e'|/rho < 1, else 0.
 * kind 2: product over dim attributes of exp(-(e_a-e'_a)^2/(2 l_a^2)), par = {l_0, ...}.
 * kind 3: (1/dim^2) sum_a sum_b exp(-(e_a-e'_b)^2/(2 l^2)), par = {l}. */
typedef struct { int kind, dim; double par[16]; } okern;
static okern g_kern = {0, 1, {0}};

int mgk_oracle_set_edge_kernel(int32_t kind, int32_t dim, const double* par, int32_t n_par) {
    if (kind < 0 || kind > 3 || dim < 1 || dim > 8 || n_par < 0 || n_par > 16) return -5;
    if (kind < 2 && dim != 1) return -5;
    g_kern.kind = kind; g_kern.dim = dim;
    for (int i = 0; i < 16; ++i) g_kern.par[i] = i < n_par ? par[i] : 0.0;
    return 0;
}

typedef struct {
    int n;           /* vertices */
    int z;           /* directed (stored) nonzeros = 2 * edges */
    const int32_t* label;
    const double* start; /* may be NULL */
    int* rowptr;     /* [n+1] CSR over directed edges */
    int* col;        /* [z] */
    double* w;       /* [z] */
    double* e;       /* [z][dim]: dim label attributes per nonzero */
    double* deg;     /* [n], sum_j A_ij + q */
} ograph;

static int build_graph(ograph* g, int n, const int32_t* label, const double* start,
                       int m, const int32_t* src, const int32_t* dst,
                       const float* weight, const float* elabel, double q) {
    g->n = n; g->z = 2 * m; g->label = label; g->start = start;
    g->rowptr = (int*)calloc((size_t)n + 1, sizeof(int));
    g->col = (int*)malloc(sizeof(int) * (size_t)(2 * m + 1));
    g->w = (double*)malloc(sizeof(double) * (size_t)(2 * m + 1));
    const int dim = g_kern.dim;
    g->e = (double*)malloc(sizeof(double) * (size_t)(2 * m + 1) * (size_t)dim);
    g->deg = (double*)malloc(sizeof(double) * (size_t)(n + 1));
    if (!g->rowptr || !g->col || !g->w || !g->e || !g->deg) return -1;
    for (int k = 0; k < m; ++k) {
        if (src[k] < 0 || src[k] >= n || dst[k] < 0 || dst[k] >= n || src[k] == dst[k]) return -2;
        g->rowptr[src[k] + 1]++; g->rowptr[dst[k] + 1]++;
    }
    for (int i = 0; i < n; ++i) g->rowptr[i + 1] += g->rowptr[i];
    int* cur = (int*)malloc(sizeof(int) * (size_t)(n + 1));
    if (!cur) return -1;
    memcpy(cur, g->rowptr, sizeof(int) * (size_t)n);
    for (int k = 0; k < m; ++k) {
        int a = src[k], b = dst[k];
        int pa = cur[a]++, pb = cur[b]++;
        g->col[pa] = b; g->w[pa] = (double)weight[k];
        g->col[pb] = a; g->w[pb] = (double)weight[k];
        for (int t = 0; t < dim; ++t) {
            g->e[(size_t)pa * dim + t] = (double)elabel[(size_t)k * dim + t];
            g->e[(size_t)pb * dim + t] = (double)elabel[(size_t)k * dim + t];
        }
    }
    free(cur);
    for (int i = 0; i < n; ++i) {
        double s = 0.0;
        for (int k = g->rowptr[i]; k < g->rowptr[i + 1]; ++k) s += g->w[k];
        g->deg[i] = s + q;
    }
    return 0;
}

static void free_graph(ograph* g) {
    free(g->rowptr); free(g->col); free(g->w); free(g->e); free(g->deg);
}

static double kv(int a, int b, double h) { return a == b ? 1.0 : h; }
/* kappa_e of two labels (dim attributes each); alpha = 1/(2 l^2) of the call for kind 0 */
static double ke(const double* e1, const double* e2, double alpha) {
    const okern* kn = &g_kern;
    if (kn->kind == 0) { double d = e1[0] - e2[0]; return exp(-alpha * d * d); }
    if (kn->kind == 1) {
        double r = fabs(e1[0] - e2[0]) / kn->par[0];
        if (!(r < 1.0)) return 0.0;
        int nc = (int)kn->par[1];
        double v = 0.0, rp = 1.0;
        for (int i = 0; i < nc; ++i) { v += kn->par[2 + i] * rp; rp *= r; }
        return v;
    }
    if (kn->kind == 2) {
        double v = 1.0;
        for (int a = 0; a < kn->dim; ++a) {
            double d = e1[a] - e2[a], l = kn->par[a];
            v *= exp(-d * d / (2.0 * l * l));
        }
        return v;
    }
    double v = 0.0, l = kn->par[0];
    for (int a = 0; a < kn->dim; ++a)
        for (int b = 0; b < kn->dim; ++b) {
            double d = e1[a] - e2[b];
            v += exp(-d * d / (2.0 * l * l));
        }
    return v / (double)(kn->dim * kn->dim);
}
static double pstart(const ograph* g, int i) { return g->start ? g->start[i] : 1.0 / (double)g->n; }

/* ---- tier 0: dense assemble + Cholesky ---------------------------------- */
static int pair_dense(const ograph* g1, const ograph* g2, double q, double h, double alpha,
                      double* K_out, double* x_out /* may be NULL, [N] */) {
    const int n1 = g1->n, n2 = g2->n;
    const size_t N = (size_t)n1 * (size_t)n2;
    double* S = (double*)calloc(N * N, sizeof(double));
    double* x = (double*)malloc(sizeof(double) * N);
    if (!S || !x) { free(S); free(x); return -1; }
    for (int i = 0; i < n1; ++i)
        for (int ip = 0; ip < n2; ++ip) {
            size_t row = (size_t)i * n2 + ip;
            S[row * N + row] = g1->deg[i] * g2->deg[ip] / kv(g1->label[i], g2->label[ip], h);
            for (int k = g1->rowptr[i]; k < g1->rowptr[i + 1]; ++k)
                for (int kp = g2->rowptr[ip]; kp < g2->rowptr[ip + 1]; ++kp) {
                    size_t colx = (size_t)g1->col[k] * n2 + g2->col[kp];
                    S[row * N + colx] = -g1->w[k] * g2->w[kp] * ke(g1->e + (size_t)k * g_kern.dim, g2->e + (size_t)kp * g_kern.dim, alpha);
                }
            x[row] = g1->deg[i] * g2->deg[ip] * q * q;   /* b = D_x q_x */
        }
    /* Cholesky S = L L^T, lower triangle in place, row by row */
    for (size_t i = 0; i < N; ++i) {
        double* Li = S + i * N;
        for (size_t j = 0; j <= i; ++j) {
            const double* Lj = S + j * N;
            double s = Li[j];
            for (size_t k = 0; k < j; ++k) s -= Li[k] * Lj[k];
            if (j == i) {
                if (!(s > 0.0)) { free(S); free(x); return -3; }
                Li[i] = sqrt(s);
            } else {
                Li[j] = s / Lj[j];
            }
        }
    }
    for (size_t i = 0; i < N; ++i) {           /* L y = b */
        double s = x[i];
        const double* Li = S + i * N;
        for (size_t k = 0; k < i; ++k) s -= Li[k] * x[k];
        x[i] = s / Li[i];
    }
    for (size_t ii = N; ii-- > 0;) {           /* L^T x = y */
        double s = x[ii];
        for (size_t k = ii + 1; k < N; ++k) s -= S[k * N + ii] * x[k];
        x[ii] = s / S[ii * N + ii];
    }
    double K = 0.0;
    for (int i = 0; i < n1; ++i)
        for (int ip = 0; ip < n2; ++ip)
            K += pstart(g1, i) * pstart(g2, ip) * x[(size_t)i * n2 + ip];
    *K_out = K;
    if (x_out) memcpy(x_out, x, sizeof(double) * N);
    free(S); free(x);
    return 0;
}

/* ---- tier 1: matrix-free operator + CG ---------------------------------- */
static void apply_S(const ograph* g1, const ograph* g2, double h, double alpha,
                    const double* u, double* out) {
    const int n1 = g1->n, n2 = g2->n;
#pragma omp parallel for schedule(dynamic, 4)
    for (int i = 0; i < n1; ++i)
        for (int ip = 0; ip < n2; ++ip) {
            size_t row = (size_t)i * n2 + ip;
            double s = g1->deg[i] * g2->deg[ip] / kv(g1->label[i], g2->label[ip], h) * u[row];
            for (int k = g1->rowptr[i]; k < g1->rowptr[i + 1]; ++k) {
                const double* urow = u + (size_t)g1->col[k] * n2;
                for (int kp = g2->rowptr[ip]; kp < g2->rowptr[ip + 1]; ++kp)
                    s -= g1->w[k] * g2->w[kp] * ke(g1->e + (size_t)k * g_kern.dim, g2->e + (size_t)kp * g_kern.dim, alpha) * urow[g2->col[kp]];
            }
            out[row] = s;
        }
}

static double dotp(const double* a, const double* b, size_t N) {
    double s = 0.0;
    for (size_t i = 0; i < N; ++i) s += a[i] * b[i];
    return s;
}

static int pair_matrix_free(const ograph* g1, const ograph* g2, double q, double h, double alpha,
                            double rtol, int max_iter, double* K_out, int* iters_out,
                            double* x_out) {
    const int n1 = g1->n, n2 = g2->n;
    const size_t N = (size_t)n1 * (size_t)n2;
    double* x = (double*)calloc(N, sizeof(double));
    double* r = (double*)malloc(sizeof(double) * N);
    double* p = (double*)malloc(sizeof(double) * N);
    double* a = (double*)malloc(sizeof(double) * N);
    if (!x || !r || !p || !a) { free(x); free(r); free(p); free(a); return -1; }
    for (int i = 0; i < n1; ++i)
        for (int ip = 0; ip < n2; ++ip)
            r[(size_t)i * n2 + ip] = g1->deg[i] * g2->deg[ip] * q * q;
    memcpy(p, r, sizeof(double) * N);
    double rr = dotp(r, r, N), bb = rr;
    int it = 0;
    for (; it < max_iter && rr > rtol * rtol * bb; ++it) {
        apply_S(g1, g2, h, alpha, p, a);
        double al = rr / dotp(p, a, N);
        for (size_t i = 0; i < N; ++i) { x[i] += al * p[i]; r[i] -= al * a[i]; }
        double rr2 = dotp(r, r, N);
        double be = rr2 / rr;
        for (size_t i = 0; i < N; ++i) p[i] = r[i] + be * p[i];
        rr = rr2;
    }
    double K = 0.0;
    for (int i = 0; i < n1; ++i)
        for (int ip = 0; ip < n2; ++ip)
            K += pstart(g1, i) * pstart(g2, ip) * x[(size_t)i * n2 + ip];
    *K_out = K;
    if (iters_out) *iters_out = it;
    if (x_out) memcpy(x_out, x, sizeof(double) * N);
    free(x); free(r); free(p); free(a);
    return rr <= rtol * rtol * bb ? 0 : -4;
}

/* ---- exported ------------------------------------------------------------ */
/* Kernel values for n_pairs pairs (pi[k], pj[k]) of a batch given in the flat
 * form: vtx_off[G+1], vtx_label, start_prob (NULL -> 1/n), edge_off[G+1],
 * src/dst (local ids, each undirected edge once), weight, edge_label (dim floats
 * per edge for the kernel in force; length_scale is used by kind 0 only).
 * tier 0 = dense Cholesky, 1 = matrix-free CG.  Returns 0, or the first
 * negative error (-1 memory, -2 bad edge, -3 not SPD, -4 CG not converged). */
int mgk_oracle_pairs(int32_t n_graphs, const int64_t* vtx_off, const int32_t* vtx_label,
                     const double* start_prob, const int64_t* edge_off,
                     const int32_t* src, const int32_t* dst,
                     const float* weight, const float* edge_label,
                     double q, double h, double length_scale,
                     int64_t n_pairs, const int32_t* pi, const int32_t* pj,
                     int32_t tier, int32_t n_threads, double* K_out) {
    const double alpha = 1.0 / (2.0 * length_scale * length_scale);
    ograph* gs = (ograph*)calloc((size_t)n_graphs, sizeof(ograph));
    if (!gs) return -1;
    int err = 0;
    for (int g = 0; g < n_graphs; ++g) {
        int64_t v0 = vtx_off[g], e0 = edge_off[g];
        int rc = build_graph(&gs[g], (int)(vtx_off[g + 1] - v0), vtx_label + v0,
                             start_prob ? start_prob + v0 : NULL, (int)(edge_off[g + 1] - e0),
                             src + e0, dst + e0, weight + e0, edge_label + e0 * g_kern.dim, q);
        if (rc && !err) err = rc;
    }
    if (!err) {
#ifdef _OPENMP
        if (n_threads > 0) omp_set_num_threads(n_threads);
#endif
        if (tier == 0) {
#pragma omp parallel for schedule(dynamic, 1)
            for (int64_t k = 0; k < n_pairs; ++k) {
                int rc = pair_dense(&gs[pi[k]], &gs[pj[k]], q, h, alpha, &K_out[k], NULL);
                if (rc) {
#pragma omp critical
                    if (!err) err = rc;
                }
            }
        } else {
            for (int64_t k = 0; k < n_pairs; ++k) {
                int rc = pair_matrix_free(&gs[pi[k]], &gs[pj[k]], q, h, alpha, 1e-13, 100000,
                                          &K_out[k], NULL, NULL);
                if (rc && !err) err = rc;
            }
        }
    }
    for (int g = 0; g < n_graphs; ++g) free_graph(&gs[g]);
    free(gs);
    return err;
}

/* One pair with the nodal solution x (n*n' doubles, row i*n'+i') returned. */
int mgk_oracle_pair_nodal(int32_t n1, const int32_t* label1, int32_t m1, const int32_t* src1,
                          const int32_t* dst1, const float* w1, const float* e1,
                          int32_t n2, const int32_t* label2, int32_t m2, const int32_t* src2,
                          const int32_t* dst2, const float* w2, const float* e2,
                          double q, double h, double length_scale, int32_t tier,
                          double* K_out, double* x_out) {
    const double alpha = 1.0 / (2.0 * length_scale * length_scale);
    ograph a, b;
    int rc = build_graph(&a, n1, label1, NULL, m1, src1, dst1, w1, e1, q);
    if (rc) return rc;
    rc = build_graph(&b, n2, label2, NULL, m2, src2, dst2, w2, e2, q);
    if (rc) { free_graph(&a); return rc; }
    if (tier == 0) rc = pair_dense(&a, &b, q, h, alpha, K_out, x_out);
    else rc = pair_matrix_free(&a, &b, q, h, alpha, 1e-13, 100000, K_out, NULL, x_out);
    free_graph(&a); free_graph(&b);
    return rc;
}

/* out = S u for one pair (fp64), for a-posteriori residual checks of a
 * solution produced elsewhere. */
int mgk_oracle_apply(int32_t n1, const int32_t* label1, int32_t m1, const int32_t* src1,
                     const int32_t* dst1, const float* w1, const float* e1,
                     int32_t n2, const int32_t* label2, int32_t m2, const int32_t* src2,
                     const int32_t* dst2, const float* w2, const float* e2,
                     double q, double h, double length_scale,
                     const double* u, double* out) {
    const double alpha = 1.0 / (2.0 * length_scale * length_scale);
    ograph a, b;
    int rc = build_graph(&a, n1, label1, NULL, m1, src1, dst1, w1, e1, q);
    if (rc) return rc;
    rc = build_graph(&b, n2, label2, NULL, m2, src2, dst2, w2, e2, q);
    if (rc) { free_graph(&a); return rc; }
    apply_S(&a, &b, h, alpha, u, out);
    free_graph(&a); free_graph(&b);
    return 0;
}

int mgk_oracle_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
