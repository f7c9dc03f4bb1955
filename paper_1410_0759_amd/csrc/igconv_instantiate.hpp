// Helper shared by the translation units that instantiate kernels.  A unit defines
// IGC_KERNEL_LIST(X) as a list of X(name, bf16, BM, BN, BK, WM, WN, swap, veca, gmode)
// and expands it twice: once to instantiate the device code, once (host pass only) to
// fill its group of the kernel table.
#ifndef IGCONV_INSTANTIATE_HPP_
#define IGCONV_INSTANTIATE_HPP_

#include <cstdio>
#include <cstdlib>

#include "igconv_kernel.hpp"
#include "igconv_kernel_table.h"

namespace igc {

// Launches `kernel` and returns the runtime's verdict on this launch (0 = accepted): the
// launch call's own return value, not the thread's last-error state, which other users of
// the runtime in the same thread may have left set.  With IGCONV_DEBUG set in the
// environment a rejected launch is also described on stderr.
template <class Kernel>
int launch_checked(Kernel kernel, const char *what, const ConvKernelParams &p, int grid, int threads, void *stream) {
    ConvKernelParams args = p;
    void *argv[] = {&args};
    const hipError_t e = hipLaunchKernel(reinterpret_cast<const void *>(kernel), dim3(grid), dim3(threads), argv, 0,
                                         static_cast<hipStream_t>(stream));
    if (e != hipSuccess && std::getenv("IGCONV_DEBUG"))
        std::fprintf(stderr, "igconv: launch of %s failed: %s\n", what, hipGetErrorString(e));
    return static_cast<int>(e);
}

template <class Cfg>
int launch_kernel(const ConvKernelParams &p, int grid, void *stream) {
    return launch_checked(&igconv_fwd_kernel<Cfg>, "igconv_fwd_kernel", p, grid, Cfg::THREADS, stream);
}

#define IGC_INSTANTIATE(NAME, BF16, BM, BN, BK, WM, WN, SWAP, VECA, GMODE) \
    template __global__ void igconv_fwd_kernel<KernelConfig<BF16, BM, BN, BK, WM, WN, SWAP, VECA, GMODE>>(const ConvKernelParams);

#define IGC_TABLE_ROW(NAME, BF16, BM, BN, BK, WM, WN, SWAP, VECA, GMODE)                        \
    {NAME, BF16, BM, BN, BK, SWAP, VECA, GMODE, 256,                                            \
     KernelConfig<BF16, BM, BN, BK, WM, WN, SWAP, VECA, GMODE>::LDS_BYTES,                      \
     &launch_kernel<KernelConfig<BF16, BM, BN, BK, WM, WN, SWAP, VECA, GMODE>>},

// Instantiates the kernels of IGC_KERNEL_LIST and defines the group GROUP.
#if !defined(__HIP_DEVICE_COMPILE__)
#define IGC_DEFINE_GROUP(GROUP)                                                     \
    namespace igc {                                                                 \
    IGC_KERNEL_LIST(IGC_INSTANTIATE)                                                \
    static const KernelInfo GROUP##_rows[] = {IGC_KERNEL_LIST(IGC_TABLE_ROW)};      \
    const KernelGroup GROUP = {GROUP##_rows, sizeof(GROUP##_rows) / sizeof(GROUP##_rows[0])}; \
    }
#else
#define IGC_DEFINE_GROUP(GROUP) \
    namespace igc {             \
    IGC_KERNEL_LIST(IGC_INSTANTIATE) \
    }
#endif

}  // namespace igc
#endif
