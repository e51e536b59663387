// Host-callable launchers of the HIP kernels (defined in the .hip files).
#ifndef MGK_LAUNCH_H
#define MGK_LAUNCH_H

#include <hip/hip_runtime_api.h>
#include <stddef.h>
#include <stdint.h>

#include "mgk_internal.h"

// On-chip solver: one workgroup of `waves` wavefronts per job, `lds_bytes` of
// dynamic LDS (the largest mgk_small_lds_words() of the jobs, in bytes).
hipError_t mgk_launch_small(int waves, bool weighted, const MgkBatchDev& X, const MgkBatchDev& Y,
                            const MgkJob* jobs_dev, int n_jobs, const MgkParams& prm,
                            size_t lds_bytes, float* K, int32_t* iters, int32_t* flags,
                            hipStream_t stream);

#endif
