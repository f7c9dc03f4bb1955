// bf16 kernels for nine-tap filters over channel-contiguous inputs (16-byte channel
// vectors straight into v_mfma_f32_32x32x16_bf16).
#include "igconv_kernel_bf16c.hpp"
#include "igconv_kernel_table.h"

namespace igc {

template <class Cfg>
static int launch_bf16c(const ConvKernelParams &p, int grid, void *stream) {
    hipLaunchKernelGGL(igconv_fwd_bf16c_kernel<Cfg>, dim3(grid), dim3(Cfg::THREADS), 0,
                       static_cast<hipStream_t>(stream), p);
    return static_cast<int>(hipGetLastError());
}

//    name, BM, BN, WM, WN, swap
#define IGC_BF16C_LIST(X) \
    X("bf16 128x128x144 channels", 128, 128, 2, 2, false) \
    X("bf16 64x128x144 channels", 64, 128, 2, 2, false) \
    X("bf16 128x128x144 channels swap", 128, 128, 2, 2, true) \
    X("bf16 64x128x144 channels swap", 64, 128, 2, 2, true)

#define IGC_BF16C_INSTANTIATE(NAME, BM, BN, WM, WN, SWAP) \
    template __global__ void igconv_fwd_bf16c_kernel<Bf16cConfig<BM, BN, WM, WN, SWAP>>(const ConvKernelParams);
IGC_BF16C_LIST(IGC_BF16C_INSTANTIATE)

#if !defined(__HIP_DEVICE_COMPILE__)
#define IGC_BF16C_ROW(NAME, BM, BN, WM, WN, SWAP)                                               \
    {NAME, true, BM, BN, Bf16cConfig<BM, BN, WM, WN, SWAP>::BK, SWAP, true, 4, 256,              \
     Bf16cConfig<BM, BN, WM, WN, SWAP>::LDS_BYTES, &launch_bf16c<Bf16cConfig<BM, BN, WM, WN, SWAP>>},
static const KernelInfo kRows[] = {IGC_BF16C_LIST(IGC_BF16C_ROW)};
const KernelGroup kGroupBF16Channels = {kRows, sizeof(kRows) / sizeof(kRows[0])};
#endif

}  // namespace igc
