// gs_noalloc.hip -- the gradient norm for callers that cannot allocate device memory (code under
// HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): gs_grad_sqnorm with the
// workgroup partials kept in a fixed array of the library's own instead of a caller workspace.
//
// The array is a file-scope __device__ object, so every GPU the library runs on holds its own
// copy at its own address from the moment the code object is loaded until the process ends.  In
// host code the array's name is only a handle for the runtime; the device address is asked for
// once per device with hipGetSymbolAddress (with that device current) and kept in a table, and
// only that address is ever handed to a kernel.
#include <hip/hip_runtime.h>

#include <cstring>
#include <mutex>

#include "gs_internal.h"

namespace gs {

constexpr size_t kScratchDoubles = (size_t)GS_SQNORM_MAX_BLOCKS + GS_FINAL_SLICES;   // 2 098 176 bytes

// workgroup partials + folding slices of the norm kernels; contents are scratch between calls
static __device__ __align__(256) __attribute__((used)) double scratch[kScratchDoubles];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static double *g_scratch_ptr[kMaxDevices];   // device address of `scratch` on device d, or null until asked

// Device address of the current device's copy of `scratch` (resolved on the first call per device).
static gs_status scratch_for_current_device(double **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return GS_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) {
            gs_status r = hip_fail(e, "hipGetSymbolAddress(scratch)");
            (void)hipGetLastError();
            return r;
        }
        if (!ptr || (reinterpret_cast<uintptr_t>(ptr) & 7u)) return GS_ERR_HIP;
        g_scratch_ptr[dev] = static_cast<double *>(ptr);
    }
    *out = g_scratch_ptr[dev];
    return GS_OK;
}

}  // namespace gs

using namespace gs;

extern "C" gs_status gs_grad_sqnorm_noalloc(const uint16_t *const *grads, int k, int64_t begin, int64_t end,
                                            double *d_sqnorm, int accumulate, void *stream)
{
    gs_status st = validate_grads(grads, k);
    if (st != GS_OK) return st;
    if (begin < 0 || end < begin) return GS_ERR_INVALID_ARG;
    if (!d_sqnorm || (reinterpret_cast<uintptr_t>(d_sqnorm) & 7u)) return GS_ERR_INVALID_ARG;
    if (end - begin > GS_NOALLOC_MAX_ELEMS) return GS_ERR_TOO_LARGE;
    if (begin == end && accumulate) return GS_OK;

    double *partials = nullptr;
    st = scratch_for_current_device(&partials);
    if (st != GS_OK) return st;

    // Nothing in the array has to start at zero: every workgroup of the norm kernel overwrites its
    // own partial, and the folding kernels read exactly the partials this launch wrote.
    SqnormArgs A;
    memset(&A, 0, sizeof A);
    for (int j = 0; j < k; ++j) A.gt.g[j] = grads[j];
    A.k = k;
    A.begin = begin;
    A.end = end;
    A.partials = partials;
    A.acc = nullptr;
    hipError_t e = launch_grad_sqnorm(A, kScratchDoubles * sizeof(double), d_sqnorm, accumulate,
                                      static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e, "gs_grad_sqnorm_noalloc launch");
    return GS_OK;
}
