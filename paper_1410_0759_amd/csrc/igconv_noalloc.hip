// igcConvolutionBackwardFilterNoAlloc: the backward-filter pass for callers that can neither
// allocate nor lend device memory.  Its partial results go to a scratch array that is part of
// the library's code object instead of a caller's workspace.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <mutex>

#include "igconv_desc.h"

namespace igc {

constexpr size_t kScratchBytes = IGC_NOALLOC_SCRATCH_BYTES;

// One copy per GPU the library runs on, held until the process ends.  In host code this name
// is only a handle for the runtime's symbol lookup, never an address: the kernels get the
// address scratch_address() returns.
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
static std::mutex g_lock;
static void *g_scratch_ptr[kMaxDevices] = {};

// Address of the current device's copy of `scratch`; looked up once per device.
static igcStatus scratch_address(void **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        return IGC_STATUS_EXECUTION_FAILED;
    }
    std::lock_guard<std::mutex> guard(g_lock);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) {
            (void)hipGetLastError();
            fprintf(stderr, "igconv: no address for the library's scratch array on device %d: %s\n", dev, hipGetErrorString(e));
            return IGC_STATUS_EXECUTION_FAILED;
        }
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return IGC_STATUS_SUCCESS;
}

}  // namespace igc

using namespace igc;

extern "C" igcStatus igcConvolutionBackwardFilterNoAlloc(igcHandle_t handle, const void *alpha, igcTensorDescriptor_t xDesc,
                                                         const void *x, igcTensorDescriptor_t dyDesc, const void *dy,
                                                         igcConvolutionDescriptor_t convDesc, const void *beta,
                                                         igcFilterDescriptor_t dwDesc, void *dw) {
    if (!handle) return IGC_STATUS_BAD_PARAM;
    // what the pass would ask a caller for; validates the descriptors, touches no GPU
    size_t need = 0;
    igcStatus st = igcGetConvolutionBackwardFilterWorkspaceSize(handle, xDesc, dyDesc, convDesc, dwDesc, &need);
    if (st != IGC_STATUS_SUCCESS) return st;
    if (need > kScratchBytes) {
        fprintf(stderr, "igconv: igcConvolutionBackwardFilterNoAlloc: this problem wants %zu bytes of scratch memory, the library "
                        "holds %zu; use igcConvolutionBackwardFilter with a workspace\n", need, kScratchBytes);
        return IGC_STATUS_NOT_SUPPORTED;
    }
    void *ptr = nullptr;
    if (need > 0) {
        st = scratch_address(&ptr);
        if (st != IGC_STATUS_SUCCESS) return st;
    }
    // Nothing has to be cleared: every element of the scratch array the summing pass reads is
    // written by this call's reduction kernel first (one workgroup per tile and range).
    return igcConvolutionBackwardFilter(handle, alpha, xDesc, x, dyDesc, dy, convDesc, ptr, need, beta, dwDesc, dw);
}
