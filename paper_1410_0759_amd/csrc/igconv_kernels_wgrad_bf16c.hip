// Backward-filter kernels for bf16 tensors with contiguous channels (tiles transposed in
// registers on their way into LDS).
#include <cstdio>
#include <cstdlib>

#include "igconv_kernel_table.h"
#include "igconv_kernel_wgrad_bf16c.hpp"

namespace igc {

template <class Cfg>
static int launch_wgc(const ConvKernelParams &p, int grid, void *stream) {
    ConvKernelParams args = p;
    void *argv[] = {&args};
    const hipError_t e = hipLaunchKernel(reinterpret_cast<const void *>(&igconv_wgrad_bf16c_kernel<Cfg>), dim3(grid), dim3(256),
                                         argv, 0, static_cast<hipStream_t>(stream));
    if (e != hipSuccess && std::getenv("IGCONV_DEBUG"))
        std::fprintf(stderr, "igconv: launch of igconv_wgrad_bf16c_kernel failed: %s\n", hipGetErrorString(e));
    return static_cast<int>(e);
}

#define IGC_WGC_LIST(X)                                   \
    X("bf16 128x128x64 wgrad channels", 128, 128)         \
    X("bf16 64x128x64 wgrad channels", 64, 128)           \
    X("bf16 128x64x64 wgrad channels", 128, 64)           \
    X("bf16 64x64x64 wgrad channels", 64, 64)

#define IGC_WGC_INSTANTIATE(NAME, BM, BN) \
    template __global__ void igconv_wgrad_bf16c_kernel<WgradBf16cConfig<BM, BN>>(const ConvKernelParams);
IGC_WGC_LIST(IGC_WGC_INSTANTIATE)

#if !defined(__HIP_DEVICE_COMPILE__)
#define IGC_WGC_ROW(NAME, BM, BN) \
    {NAME, true, BM, BN, kWgcBK, false, true, 10, 256, WgradBf16cConfig<BM, BN>::LDS_BYTES, &launch_wgc<WgradBf16cConfig<BM, BN>>},
static const KernelInfo kRows[] = {IGC_WGC_LIST(IGC_WGC_ROW)};
const KernelGroup kGroupWgradBF16Channels = {kRows, sizeof(kRows) / sizeof(kRows[0])};
#endif

}  // namespace igc
