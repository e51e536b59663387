// Host-callable launchers of the HIP kernels (defined in the .hip files).
#ifndef MGK_LAUNCH_H
#define MGK_LAUNCH_H

#include <hip/hip_runtime_api.h>
#include <stddef.h>
#include <stdint.h>

#include "mgk_internal.h"

// On-chip solver: one workgroup of `waves` wavefronts per job, each thread
// owning up to `ept` vector elements (waves * 64 * ept >= n n' of every job),
// `lds_bytes` of dynamic LDS (the largest MgkSmallPlan::total of the jobs).
// atomic_rows: some inner graph of the jobs has a row of more than 16 nonzeros.
// One definition per workgroup size, each in its own translation unit.
#define MGK_DECL_SMALL(W)                                                                         \
    hipError_t mgk_launch_small_w##W(int ept, bool weighted, bool atomic_rows, const MgkBatchDev& X, \
                                     const MgkBatchDev& Y, const MgkJob* jobs_dev, int n_jobs,    \
                                     const MgkParams& prm, size_t lds_bytes,                      \
                                     const MgkOutputs& out, hipStream_t stream);
MGK_DECL_SMALL(1)
MGK_DECL_SMALL(2)
MGK_DECL_SMALL(4)
MGK_DECL_SMALL(8)
MGK_DECL_SMALL(16)
#undef MGK_DECL_SMALL
// four wavefronts with 6, 10 or 14 elements per thread (a translation unit of its own)
hipError_t mgk_launch_small_w4_fine(int ept, bool weighted, bool atomic_rows, const MgkBatchDev& X,
                                    const MgkBatchDev& Y, const MgkJob* jobs_dev, int n_jobs,
                                    const MgkParams& prm, size_t lds_bytes, const MgkOutputs& out,
                                    hipStream_t stream);

static inline hipError_t mgk_launch_small(int waves, int ept, bool weighted, bool atomic_rows, const MgkBatchDev& X,
                                          const MgkBatchDev& Y, const MgkJob* jobs_dev, int n_jobs,
                                          const MgkParams& prm, size_t lds_bytes,
                                          const MgkOutputs& out, hipStream_t stream) {
    switch (waves) {
        case 1: return mgk_launch_small_w1(ept, weighted, atomic_rows, X, Y, jobs_dev, n_jobs, prm, lds_bytes, out, stream);
        case 2: return mgk_launch_small_w2(ept, weighted, atomic_rows, X, Y, jobs_dev, n_jobs, prm, lds_bytes, out, stream);
        case 4:
            if (ept == 6 || ept == 10 || ept == 14)
                return mgk_launch_small_w4_fine(ept, weighted, atomic_rows, X, Y, jobs_dev, n_jobs, prm, lds_bytes, out, stream);
            return mgk_launch_small_w4(ept, weighted, atomic_rows, X, Y, jobs_dev, n_jobs, prm, lds_bytes, out, stream);
        case 8: return mgk_launch_small_w8(ept, weighted, atomic_rows, X, Y, jobs_dev, n_jobs, prm, lds_bytes, out, stream);
        case 16: return mgk_launch_small_w16(ept, weighted, atomic_rows, X, Y, jobs_dev, n_jobs, prm, lds_bytes, out, stream);
        default: return hipErrorInvalidValue;
    }
}

// Register-resident on-chip solver (mgk_regs.hip): `waves` (4 or 8) wavefronts
// per job, `chunks` 64-lane chunks of the inner graph, ept * waves * 64 >= n n'
// of every job, `lds_bytes` the largest MgkRegsPlan::total of the jobs.  One
// definition per (waves, chunks), each in its own translation unit.
#define MGK_DECL_REGS(W, C)                                                                       \
    hipError_t mgk_launch_regs_w##W##_c##C(int ept, bool weighted, const MgkBatchDev& X,          \
                                           const MgkBatchDev& Y, const MgkJob* jobs_dev,          \
                                           int n_jobs, const MgkParams& prm, size_t lds_bytes,    \
                                           const MgkOutputs& out, hipStream_t stream);
MGK_DECL_REGS(4, 1)
MGK_DECL_REGS(4, 2)
MGK_DECL_REGS(8, 1)
MGK_DECL_REGS(8, 2)
#undef MGK_DECL_REGS

static inline hipError_t mgk_launch_regs(int waves, int chunks, int ept, bool weighted,
                                         const MgkBatchDev& X, const MgkBatchDev& Y,
                                         const MgkJob* jobs_dev, int n_jobs, const MgkParams& prm,
                                         size_t lds_bytes, const MgkOutputs& out, hipStream_t stream) {
    switch (waves * 10 + chunks) {
        case 41: return mgk_launch_regs_w4_c1(ept, weighted, X, Y, jobs_dev, n_jobs, prm, lds_bytes, out, stream);
        case 42: return mgk_launch_regs_w4_c2(ept, weighted, X, Y, jobs_dev, n_jobs, prm, lds_bytes, out, stream);
        case 81: return mgk_launch_regs_w8_c1(ept, weighted, X, Y, jobs_dev, n_jobs, prm, lds_bytes, out, stream);
        case 82: return mgk_launch_regs_w8_c2(ept, weighted, X, Y, jobs_dev, n_jobs, prm, lds_bytes, out, stream);
        default: return hipErrorInvalidValue;
    }
}

// Owner-computes on-chip solver (mgk_sell.hip): `waves` (4, 8 or 16) wavefronts per job,
// `ept` vector slots per lane (2 waves ept >= tiles of every job), `regs` entry registers
// per lane (>= what mgk_sell_need returns for every job), `lds_bytes` the largest
// MgkSellPlan::total of the jobs.  Launch shapes (waves, ept, regs); one translation unit
// per workgroup size.
#define MGK_SELL_SHAPES_W4(F) F(4, 4, 32) F(4, 6, 40) F(4, 8, 48)
#define MGK_SELL_SHAPES_W8(F) F(8, 2, 16) F(8, 3, 24) F(8, 4, 32) F(8, 5, 36)
#define MGK_SELL_SHAPES_W16(F) F(16, 3, 24) F(16, 4, 28)
struct MgkSellShape { int waves, ept, regs; };
static const MgkSellShape kMgkSellShapes[] = {
#define MGK_SELL_ROW(W, E, R) {W, E, R},
    MGK_SELL_SHAPES_W4(MGK_SELL_ROW) MGK_SELL_SHAPES_W8(MGK_SELL_ROW) MGK_SELL_SHAPES_W16(MGK_SELL_ROW)
#undef MGK_SELL_ROW
};
#define MGK_DECL_SELL(W)                                                                             \
    hipError_t mgk_launch_sell_w##W(int ept, int regs, const MgkBatchDev& X, const MgkBatchDev& Y,    \
                                    const MgkJob* jobs_dev, int n_jobs, const MgkParams& prm,         \
                                    size_t lds_bytes, const MgkOutputs& out, hipStream_t stream);
MGK_DECL_SELL(4)
MGK_DECL_SELL(8)
MGK_DECL_SELL(16)
#undef MGK_DECL_SELL
static inline hipError_t mgk_launch_sell(int waves, int ept, int regs, const MgkBatchDev& X, const MgkBatchDev& Y,
                                         const MgkJob* jobs_dev, int n_jobs, const MgkParams& prm,
                                         size_t lds_bytes, const MgkOutputs& out, hipStream_t stream) {
    switch (waves) {
        case 4: return mgk_launch_sell_w4(ept, regs, X, Y, jobs_dev, n_jobs, prm, lds_bytes, out, stream);
        case 8: return mgk_launch_sell_w8(ept, regs, X, Y, jobs_dev, n_jobs, prm, lds_bytes, out, stream);
        case 16: return mgk_launch_sell_w16(ept, regs, X, Y, jobs_dev, n_jobs, prm, lds_bytes, out, stream);
        default: return hipErrorInvalidValue;
    }
}

// Fixed job-list array in device memory for the entry point that allocates nothing
// (mgk_noalloc.hip): its device address on `device` and how many jobs it holds.
#define MGK_NOALLOC_MAX_PAIRS 65536
hipError_t mgk_noalloc_job_storage(int device, MgkJob** jobs, int64_t* capacity);

// ---- solver with vectors in global memory (mgk_large.hip) --------------------
// Expand every octile of batch B into the outer (CSR order) and inner (lane
// layout) entry lists; `outer` holds B.nnz_total entries, `inner` B.lanes_total.
hipError_t mgk_launch_expand(const MgkBatchDev& B, const MgkParams& prm, MgkEntry* outer, MgkEntry* inner,
                             hipStream_t stream);
// Expand every octile of B to dense 8x8 blocks (64 * B.n_tiles_total floats per array).
hipError_t mgk_launch_expand_dense(const MgkBatchDev& B, const MgkParams& prm, float* dw, float* de,
                                   float* dlw, hipStream_t stream);
// Set-up of Alg. 1 for n_pairs pairs (state must be zero-filled before).
hipError_t mgk_launch_large_init(const MgkBatchDev& X, const MgkBatchDev& Y, const MgkLargePair* pairs,
                                 MgkPairState* state, float* vec, const MgkParams& prm, int n_pairs,
                                 int vec_blocks, hipStream_t stream);
// Iteration `it` (0, 1, ...) of Alg. 1 for all pairs that have not stopped: the product, then
// three kernels over the vectors that also do the scalar steps and the stop test.  n_active[0]
// is decremented for every pair that stops, n_active[1] raised to the number of iterations
// it took.  DX/DY non-null: dense tile-pair XMV
// (xmv_blocks = workgroups of 4 output blocks); else the sparse XMV on the
// expanded lists: with rows_threads > 0 the one that stages rows of p in
// rows_lds_bytes of LDS (xmv_blocks = outer rows, one workgroup of rows_threads
// each; every row of p must fit; rows_chunks = 1, 2 or 4 chunks of the inner layout
// per pass of a wavefront), with rows_threads == 0 the one that gathers p from global
// memory.
hipError_t mgk_launch_large_iteration(const MgkBatchDev& X, const MgkBatchDev& Y, const MgkExpanded& EX,
                                      const MgkExpanded& EY, const MgkLargePair* pairs,
                                      MgkPairState* state, float* vec, const MgkParams& prm,
                                      bool weighted, int n_pairs, int xmv_blocks, int vec_blocks,
                                      int* n_active, int it, const MgkDenseTiles* DX,
                                      const MgkDenseTiles* DY, int rows_threads, int rows_lds_bytes,
                                      int rows_chunks, hipStream_t stream);
// K = p_x^T x, the nodal solution, a check of the true residual for pairs whose solution grew
// far beyond the Jacobi guess (one more product, arguments as for an iteration), and the
// per-pair outputs.
hipError_t mgk_launch_large_final(const MgkBatchDev& X, const MgkBatchDev& Y, const MgkExpanded& EX,
                                  const MgkExpanded& EY, const MgkLargePair* pairs, MgkPairState* state,
                                  float* vec, const MgkParams& prm, bool weighted, int n_pairs, int xmv_blocks,
                                  int vec_blocks, const MgkDenseTiles* DX, const MgkDenseTiles* DY,
                                  int rows_threads, int rows_lds_bytes, int rows_chunks, const MgkOutputs& out,
                                  hipStream_t stream);
// In-place normalisation K[i][j] /= sqrt(K[i][i] K[j][j]) of an n x n matrix; diag holds n floats.
hipError_t mgk_launch_normalize(float* K, float* diag, int n, hipStream_t stream);

#endif
