// Job-list storage for mgk_pairs_noalloc: a fixed array in device memory that exists once
// per GPU for the life of the process, so that the entry point needs no device allocation.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mgk_internal.h"
#include "mgk_launch.h"

namespace {

// The job list of one call: MGK_NOALLOC_MAX_PAIRS jobs of 16 bytes (1 MiB).  Every call on
// a GPU uses this one array and overwrites it from the start; it keeps the previous
// call's jobs until then, and nothing in it has to be cleared.
static __device__ __align__(256) unsigned char scratch[(size_t)MGK_NOALLOC_MAX_PAIRS * sizeof(MgkJob)];

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};   // device address of `scratch` on each GPU, 0 = not looked up yet

}  // namespace

// Device address of the array on `device` (each GPU holds its own copy at its own
// address), looked up once per device with that device current.  In host code the array's
// name stands for the symbol, not for an address a kernel could use: only the pointer
// returned here is ever passed on.
hipError_t mgk_noalloc_job_storage(int device, MgkJob** jobs, int64_t* capacity) {
    if (device < 0 || device >= kMaxDevices || !jobs || !capacity) return hipErrorInvalidValue;
    if (g_scratch_ptr[device] == nullptr) {
        int current = -1;
        hipError_t e = hipGetDevice(&current);
        if (e != hipSuccess) return e;
        if (current != device) {
            e = hipSetDevice(device);
            if (e != hipSuccess) return e;
        }
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (current != device && current >= 0) (void)hipSetDevice(current);
        if (e != hipSuccess) return e;
        if (ptr == nullptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[device] = ptr;
    }
    *jobs = static_cast<MgkJob*>(g_scratch_ptr[device]);
    *capacity = MGK_NOALLOC_MAX_PAIRS;
    return hipSuccess;
}
