// Sanitizer driver for the host side of the library (loader, reordering, packer, planner
// entry checks) on a host-only context: built with -fsanitize=address,undefined together
// with mgk_host.cpp and mgk_reorder.cpp by tests/test_sanitizers.py.  No GPU code runs:
// the kernel launchers are replaced by stubs that fail.
#include <hip/hip_runtime_api.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

#include "../../include/mgk.h"
#include "../../paper_1910_06310_amd/csrc/mgk_launch.h"

// ---- launcher stubs (a host-only context never reaches them) -------------------------------
#define STUB_SMALL(W)                                                                               \
    hipError_t mgk_launch_small_w##W(int, bool, bool, const MgkBatchDev&, const MgkBatchDev&,       \
                                     const MgkJob*, int, const MgkParams&, size_t, const MgkOutputs&, \
                                     hipStream_t) { return hipErrorUnknown; }
STUB_SMALL(1) STUB_SMALL(2) STUB_SMALL(4) STUB_SMALL(8) STUB_SMALL(16)
hipError_t mgk_launch_small_w4_fine(int, bool, bool, const MgkBatchDev&, const MgkBatchDev&, const MgkJob*, int,
                                    const MgkParams&, size_t, const MgkOutputs&, hipStream_t) { return hipErrorUnknown; }
#define STUB_REGS(W, C)                                                                             \
    hipError_t mgk_launch_regs_w##W##_c##C(int, bool, const MgkBatchDev&, const MgkBatchDev&, const MgkJob*, int, \
                                           const MgkParams&, size_t, const MgkOutputs&, hipStream_t) { return hipErrorUnknown; }
STUB_REGS(4, 1) STUB_REGS(4, 2) STUB_REGS(8, 1) STUB_REGS(8, 2)
#define STUB_SELL(W)                                                                                \
    hipError_t mgk_launch_sell_w##W(int, int, const MgkBatchDev&, const MgkBatchDev&, const MgkJob*, int, \
                                    const MgkParams&, size_t, const MgkOutputs&, hipStream_t) { return hipErrorUnknown; }
STUB_SELL(4) STUB_SELL(8) STUB_SELL(16)
hipError_t mgk_noalloc_job_storage(int, MgkJob**, int64_t*) { return hipErrorUnknown; }
hipError_t mgk_launch_expand(const MgkBatchDev&, const MgkParams&, MgkEntry*, MgkEntry*, hipStream_t) { return hipErrorUnknown; }
hipError_t mgk_launch_expand_dense(const MgkBatchDev&, const MgkParams&, float*, float*, float*, hipStream_t) { return hipErrorUnknown; }
hipError_t mgk_launch_large_init(const MgkBatchDev&, const MgkBatchDev&, const MgkLargePair*, MgkPairState*, float*,
                                 const MgkParams&, int, int, hipStream_t) { return hipErrorUnknown; }
hipError_t mgk_launch_large_iteration(const MgkBatchDev&, const MgkBatchDev&, const MgkExpanded&, const MgkExpanded&,
                                      const MgkLargePair*, MgkPairState*, float*, const MgkParams&, bool, int, int, int,
                                      int*, int, const MgkDenseTiles*, const MgkDenseTiles*, int, int, int, hipStream_t) { return hipErrorUnknown; }
hipError_t mgk_launch_large_final(const MgkBatchDev&, const MgkBatchDev&, const MgkExpanded&, const MgkExpanded&,
                                  const MgkLargePair*, MgkPairState*, float*, const MgkParams&, bool, int, int, int,
                                  const MgkDenseTiles*, const MgkDenseTiles*, int, int, int, const MgkOutputs&, hipStream_t) { return hipErrorUnknown; }
hipError_t mgk_launch_normalize(float*, float*, int, hipStream_t) { return hipErrorUnknown; }

#define CHECK(cond)                                                              \
    do {                                                                         \
        if (!(cond)) { std::printf("FAILED line %d: %s\n", __LINE__, #cond); return 1; } \
    } while (0)

struct Batch {
    std::vector<int64_t> voff{0}, eoff{0};
    std::vector<int32_t> lab, src, dst;
    std::vector<float> w, e, xyz;
};

// random connected-ish graphs: a random tree plus extra edges, no duplicates
static void add_graph(Batch& b, std::mt19937& rng, int n, int extra) {
    std::vector<std::vector<char>> has(n, std::vector<char>(n, 0));
    auto edge = [&](int a, int c) {
        if (a == c || has[a][c]) return;
        has[a][c] = has[c][a] = 1;
        b.src.push_back(std::min(a, c));
        b.dst.push_back(std::max(a, c));
        b.w.push_back(0.5f + (rng() % 1000) / 1000.0f);
        b.e.push_back((rng() % 1000) / 500.0f);
    };
    for (int v = 1; v < n; ++v) edge(v, (int)(rng() % v));
    for (int k = 0; k < extra; ++k) edge((int)(rng() % n), (int)(rng() % n));
    for (int v = 0; v < n; ++v) {
        b.lab.push_back((int)(rng() % 4));
        for (int a = 0; a < 3; ++a) b.xyz.push_back((rng() % 10000) / 10000.0f);
    }
    b.voff.push_back(b.voff.back() + n);
    b.eoff.push_back((int64_t)b.src.size());
}

int main() {
    mgk_ctx* ctx = nullptr;
    CHECK(mgk_create(&ctx, -1) == MGK_OK);
    CHECK(mgk_set_vertex_kernel_delta(ctx, 0.5f) == MGK_OK);
    CHECK(mgk_set_edge_kernel_se(ctx, 1.0f) == MGK_OK);
    CHECK(mgk_set_stop_prob(ctx, 0.05f) == MGK_OK);
    std::mt19937 rng(1910);
    Batch b;
    const int sizes[] = {1, 2, 7, 8, 9, 33, 64, 65, 130, 300};
    for (int rep = 0; rep < 3; ++rep)
        for (int n : sizes) add_graph(b, rng, n, rep * n);
    const int G = (int)b.voff.size() - 1;
    for (int reorder = 0; reorder <= 2; ++reorder) {
        mgk_batch* B = nullptr;
        CHECK(mgk_load_graphs(ctx, G, b.voff.data(), b.lab.data(), nullptr, b.eoff.data(), b.src.data(), b.dst.data(),
                              b.w.data(), b.e.data(), reorder, &B) == MGK_OK);
        int64_t ng = 0, nv = 0, nnz = 0, nt = 0, no = 0;
        CHECK(mgk_batch_stats(B, &ng, &nv, &nnz, &nt, &no) == MGK_OK);
        CHECK(ng == G && nv == b.voff.back() && nnz == 2 * (int64_t)b.src.size());
        std::vector<int32_t> perm((size_t)nv);
        CHECK(mgk_batch_permutation(B, perm.data()) == MGK_OK);
        int64_t tiles_seen = 0, nnz_seen = 0;
        for (int g = 0; g < G; ++g) {
            int32_t t = 0, z = 0;
            CHECK(mgk_batch_get_tiles(B, g, &t, &z, nullptr, nullptr, nullptr, nullptr, nullptr) == MGK_OK);
            std::vector<int32_t> tr(t), tc(t);
            std::vector<uint64_t> bm(t);
            std::vector<float> w(z), e(z);
            CHECK(mgk_batch_get_tiles(B, g, &t, &z, tr.data(), tc.data(), bm.data(), w.data(), e.data()) == MGK_OK);
            int64_t bits = 0;
            for (int k = 0; k < t; ++k) bits += __builtin_popcountll(bm[k]);
            CHECK(bits == z);
            tiles_seen += t;
            nnz_seen += z;
            // the permutation of this graph is a bijection
            const int n = (int)(b.voff[g + 1] - b.voff[g]);
            std::vector<char> hit(n, 0);
            for (int v = 0; v < n; ++v) {
                const int32_t p = perm[(size_t)b.voff[g] + v];
                CHECK(p >= 0 && p < n && !hit[p]);
                hit[p] = 1;
            }
        }
        CHECK(tiles_seen == nt && nnz_seen == nnz);
        // a host-only context refuses to solve, with a status
        float dummy = 0.f;
        CHECK(mgk_gram(ctx, B, &dummy, nullptr, nullptr, nullptr) == MGK_ESTATE);
        mgk_free_batch(ctx, B);
    }
    {   // graphs with coordinates, numbered along the space-filling curve
        mgk_batch* B = nullptr;
        CHECK(mgk_load_graphs_embedded(ctx, G, b.voff.data(), b.lab.data(), nullptr, b.eoff.data(), b.src.data(),
                                       b.dst.data(), b.w.data(), b.e.data(), 3, b.xyz.data(), &B) == MGK_OK);
        mgk_free_batch(ctx, B);
    }
    {   // rejected inputs: each must come back as a status, with nothing leaked or overrun
        mgk_batch* B = nullptr;
        const int64_t bad_v[] = {0, 100, 50}, zero_e[] = {0, 0, 0};
        std::vector<int32_t> lab(150, 0);
        CHECK(mgk_load_graphs(ctx, 2, bad_v, lab.data(), nullptr, zero_e, nullptr, nullptr, nullptr, nullptr, 0, &B) == MGK_EINVAL);
        const int64_t v2[] = {0, 3}, e2[] = {0, 2};
        const int32_t s_loop[] = {0, 1}, d_loop[] = {1, 1};
        CHECK(mgk_load_graphs(ctx, 1, v2, lab.data(), nullptr, e2, s_loop, d_loop, nullptr, nullptr, 1, &B) == MGK_EINVAL);
        const int32_t s_dup[] = {0, 1}, d_dup[] = {1, 0};
        CHECK(mgk_load_graphs(ctx, 1, v2, lab.data(), nullptr, e2, s_dup, d_dup, nullptr, nullptr, 1, &B) == MGK_EINVAL);
        const int32_t s_rng[] = {0, 1}, d_rng[] = {1, 7};
        CHECK(mgk_load_graphs(ctx, 1, v2, lab.data(), nullptr, e2, s_rng, d_rng, nullptr, nullptr, 2, &B) == MGK_EINVAL);
        const int32_t s_ok[] = {0, 1}, d_ok[] = {1, 2};
        const float w_nan[] = {1.f, NAN};
        CHECK(mgk_load_graphs(ctx, 1, v2, lab.data(), nullptr, e2, s_ok, d_ok, w_nan, nullptr, 1, &B) == MGK_EINVAL);
        CHECK(mgk_set_vertex_kernel_delta(ctx, 0.f) == MGK_EINVAL);
        CHECK(mgk_last_error(ctx)[0] != 0);
    }
    mgk_destroy(ctx);
    std::printf("host sanitizer driver: ok\n");
    return 0;
}
