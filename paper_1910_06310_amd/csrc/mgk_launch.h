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
                                     const MgkParams& prm, size_t lds_bytes, float* K,            \
                                     int32_t* iters, int32_t* flags, hipStream_t stream);
MGK_DECL_SMALL(1)
MGK_DECL_SMALL(2)
MGK_DECL_SMALL(4)
MGK_DECL_SMALL(8)
MGK_DECL_SMALL(16)
#undef MGK_DECL_SMALL

static inline hipError_t mgk_launch_small(int waves, int ept, bool weighted, bool atomic_rows, const MgkBatchDev& X,
                                          const MgkBatchDev& Y, const MgkJob* jobs_dev, int n_jobs,
                                          const MgkParams& prm, size_t lds_bytes, float* K,
                                          int32_t* iters, int32_t* flags, hipStream_t stream) {
    switch (waves) {
        case 1: return mgk_launch_small_w1(ept, weighted, atomic_rows, X, Y, jobs_dev, n_jobs, prm, lds_bytes, K, iters, flags, stream);
        case 2: return mgk_launch_small_w2(ept, weighted, atomic_rows, X, Y, jobs_dev, n_jobs, prm, lds_bytes, K, iters, flags, stream);
        case 4: return mgk_launch_small_w4(ept, weighted, atomic_rows, X, Y, jobs_dev, n_jobs, prm, lds_bytes, K, iters, flags, stream);
        case 8: return mgk_launch_small_w8(ept, weighted, atomic_rows, X, Y, jobs_dev, n_jobs, prm, lds_bytes, K, iters, flags, stream);
        case 16: return mgk_launch_small_w16(ept, weighted, atomic_rows, X, Y, jobs_dev, n_jobs, prm, lds_bytes, K, iters, flags, stream);
        default: return hipErrorInvalidValue;
    }
}

#endif
