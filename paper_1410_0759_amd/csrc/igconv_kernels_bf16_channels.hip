// bf16 kernels for nine-tap filters over channel-contiguous inputs (16-byte channel
// vectors straight into v_mfma_f32_32x32x16_bf16).
#include "igconv_instantiate.hpp"
#include "igconv_kernel_bf16c.hpp"

namespace igc {

template <class Cfg>
static int launch_bf16c(const ConvKernelParams &p, int grid, void *stream) {
    return launch_checked(&igconv_fwd_bf16c_kernel<Cfg>, "igconv_fwd_bf16c_kernel", p, grid, Cfg::THREADS, stream);
}

//    name, BM, BN, WM, WN, swap, patch
#define IGC_BF16C_LIST(X) \
    X("bf16 128x128x144 channels", 128, 128, 2, 2, false, false) \
    X("bf16 64x128x144 channels", 64, 128, 2, 2, false, false) \
    X("bf16 128x128x144 channels swap", 128, 128, 2, 2, true, false) \
    X("bf16 64x128x144 channels swap", 64, 128, 2, 2, true, false) \
    X("bf16 128x128x144 patch", 128, 128, 2, 2, false, true) \
    X("bf16 64x128x144 patch", 64, 128, 2, 2, false, true) \
    X("bf16 128x128x144 patch swap", 128, 128, 2, 2, true, true) \
    X("bf16 64x128x144 patch swap", 64, 128, 2, 2, true, true) \
    X("bf16 64x256x144 patch", 64, 256, 1, 4, false, true) \
    X("bf16 64x256x144 patch swap", 64, 256, 1, 4, true, true)

// two teams of four wavefronts per workgroup, each on half of the reduction steps
#define IGC_BF16C_TEAMS_LIST(X) \
    X("bf16 64x256x144 patch teams", 64, 256, 1, 4, false, true) \
    X("bf16 64x256x144 patch teams swap", 64, 256, 1, 4, true, true)

#define IGC_BF16C_INSTANTIATE(NAME, BM, BN, WM, WN, SWAP, PATCH) \
    template __global__ void igconv_fwd_bf16c_kernel<Bf16cConfig<BM, BN, WM, WN, SWAP, PATCH>>(const ConvKernelParams);
IGC_BF16C_LIST(IGC_BF16C_INSTANTIATE)
#define IGC_BF16C_TEAMS_INSTANTIATE(NAME, BM, BN, WM, WN, SWAP, PATCH) \
    template __global__ void igconv_fwd_bf16c_kernel<Bf16cConfig<BM, BN, WM, WN, SWAP, PATCH, 2>>(const ConvKernelParams);
IGC_BF16C_TEAMS_LIST(IGC_BF16C_TEAMS_INSTANTIATE)

#if !defined(__HIP_DEVICE_COMPILE__)
#define IGC_BF16C_ROW(NAME, BM, BN, WM, WN, SWAP, PATCH)                                 \
    {NAME, true, BM, BN, Bf16cConfig<BM, BN, WM, WN, SWAP, PATCH>::BK, SWAP, true, PATCH ? 5 : 4, 256, \
     Bf16cConfig<BM, BN, WM, WN, SWAP, PATCH>::LDS_BYTES,                                 \
     &launch_bf16c<Bf16cConfig<BM, BN, WM, WN, SWAP, PATCH>>, 0},
static_assert(Bf16cConfig<128, 128, 2, 2, false, true>::PATCH_PIX == 512, "the host's patch capacity must match");
// (variant 2: the two-team kernels)
#define IGC_BF16C_TEAMS_ROW(NAME, BM, BN, WM, WN, SWAP, PATCH)                                 \
    {NAME, true, BM, BN, Bf16cConfig<BM, BN, WM, WN, SWAP, PATCH, 2>::BK, SWAP, true, PATCH ? 5 : 4, 512, \
     Bf16cConfig<BM, BN, WM, WN, SWAP, PATCH, 2>::LDS_BYTES,                                 \
     &launch_bf16c<Bf16cConfig<BM, BN, WM, WN, SWAP, PATCH, 2>>, 2},
static const KernelInfo kRows[] = {IGC_BF16C_LIST(IGC_BF16C_ROW) IGC_BF16C_TEAMS_LIST(IGC_BF16C_TEAMS_ROW)};
const KernelGroup kGroupBF16Channels = {kRows, sizeof(kRows) / sizeof(kRows[0])};
#endif

}  // namespace igc
