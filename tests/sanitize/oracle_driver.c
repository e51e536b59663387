/* Sanitizer driver for the C edition of the oracle: built with -fsanitize=address,undefined
 * together with oracle/mgk_oracle.c by tests/test_sanitizers.py.  Runs both tiers on a small
 * batch (start probabilities included), the nodal solution and the operator, and checks
 * that the tiers agree. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int mgk_oracle_set_edge_kernel(int32_t kind, int32_t dim, const double* par, int32_t n_par);
int mgk_oracle_pairs(int32_t n_graphs, const int64_t* vtx_off, const int32_t* vtx_label,
                     const double* start_prob, const int64_t* edge_off, const int32_t* src, const int32_t* dst,
                     const float* weight, const float* edge_label, double q, double h, double length_scale,
                     int64_t n_pairs, const int32_t* pi, const int32_t* pj, int32_t tier, int32_t n_threads,
                     double* K_out);
int mgk_oracle_pair_nodal(int32_t n1, const int32_t* label1, int32_t m1, const int32_t* src1, const int32_t* dst1,
                          const float* w1, const float* e1, int32_t n2, const int32_t* label2, int32_t m2,
                          const int32_t* src2, const int32_t* dst2, const float* w2, const float* e2, double q,
                          double h, double length_scale, int32_t tier, double* K_out, double* x_out);
int mgk_oracle_apply(int32_t n1, const int32_t* label1, int32_t m1, const int32_t* src1, const int32_t* dst1,
                     const float* w1, const float* e1, int32_t n2, const int32_t* label2, int32_t m2,
                     const int32_t* src2, const int32_t* dst2, const float* w2, const float* e2, double q, double h,
                     double length_scale, const double* u, double* out);

#define CHECK(c) do { if (!(c)) { printf("FAILED line %d: %s\n", __LINE__, #c); return 1; } } while (0)

int main(void) {
    /* three graphs: a path of 4, a triangle with a tail (5 vertices), a single vertex */
    const int64_t voff[] = {0, 4, 9, 10}, eoff[] = {0, 3, 8, 8};
    const int32_t lab[] = {0, 1, 0, 2, 1, 1, 0, 2, 0, 1};
    const int32_t src[] = {0, 1, 2, 0, 1, 0, 2, 3}, dst[] = {1, 2, 3, 1, 2, 2, 3, 4};
    const float w[] = {1.f, 0.5f, 0.75f, 1.f, 1.f, 0.6f, 0.9f, 0.8f};
    const float e[] = {1.0f, 1.5f, 1.2f, 1.1f, 1.9f, 1.4f, 1.3f, 1.0f};
    const double sp[] = {0.1, 0.2, 0.3, 0.4, 0.3, 0.2, 0.2, 0.2, 0.1, 1.0};
    const int32_t pi[] = {0, 0, 0, 1, 1, 2}, pj[] = {0, 1, 2, 1, 2, 2};
    double K0[6], K1[6], Ks[6];
    CHECK(mgk_oracle_set_edge_kernel(0, 1, NULL, 0) == 0);
    CHECK(mgk_oracle_pairs(3, voff, lab, NULL, eoff, src, dst, w, e, 0.05, 0.5, 1.0, 6, pi, pj, 0, 2, K0) == 0);
    CHECK(mgk_oracle_pairs(3, voff, lab, NULL, eoff, src, dst, w, e, 0.05, 0.5, 1.0, 6, pi, pj, 1, 2, K1) == 0);
    CHECK(mgk_oracle_pairs(3, voff, lab, sp, eoff, src, dst, w, e, 0.05, 0.5, 1.0, 6, pi, pj, 0, 2, Ks) == 0);
    for (int k = 0; k < 6; ++k) {
        CHECK(K0[k] > 0.0 && fabs(K0[k] - K1[k]) <= 1e-10 * K0[k]);
        CHECK(Ks[k] > 0.0);
    }
    /* single vertex against itself: K = p p' kappa_v q q' = 0.0025 (Eq. 1 without edges) */
    CHECK(fabs(K0[5] - 0.0025) <= 1e-15);
    double K, x[20], y[20];
    CHECK(mgk_oracle_pair_nodal(4, lab, 3, src, dst, w, e, 5, lab + 4, 5, src + 3, dst + 3, w + 3, e + 3, 0.05, 0.5, 1.0,
                                0, &K, x) == 0);
    CHECK(fabs(K - K0[1]) <= 1e-12 * K);
    CHECK(mgk_oracle_apply(4, lab, 3, src, dst, w, e, 5, lab + 4, 5, src + 3, dst + 3, w + 3, e + 3, 0.05, 0.5, 1.0, x,
                           y) == 0);
    /* S x = b = d d' q^2 > 0 */
    for (int k = 0; k < 20; ++k) CHECK(y[k] > 0.0);
    /* a self loop is refused */
    const int32_t s_bad[] = {1}, d_bad[] = {1};
    const int64_t v1[] = {0, 2}, e1[] = {0, 1};
    const int32_t z[] = {0};
    CHECK(mgk_oracle_pairs(1, v1, lab, NULL, e1, s_bad, d_bad, w, e, 0.05, 0.5, 1.0, 1, z, z, 0, 1, K0) != 0);
    printf("oracle sanitizer driver: ok\n");
    return 0;
}
