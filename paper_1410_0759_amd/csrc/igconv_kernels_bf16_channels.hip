// bf16 kernels for nine-tap filters over channel-contiguous inputs (16-byte channel
// vectors straight into v_mfma_f32_32x32x16_bf16).
#include "igconv_instantiate.hpp"
#include "igconv_kernel_bf16c.hpp"
#include "igconv_kernel_bf16s.hpp"

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

// four multiplying and four moving wavefronts per workgroup (igconv_kernel_bf16s.hpp)
template <class Cfg>
static int launch_bf16s(const ConvKernelParams &p, int grid, void *stream) {
    return launch_checked(&igconv_fwd_bf16s_kernel<Cfg>, "igconv_fwd_bf16s_kernel", p, grid, Cfg::THREADS, stream);
}
//    name, BM, BN, swap, multiplier groups, patch pixels, register sets for filter rows, intervals of slack
#define IGC_BF16S_LIST(X) \
    X("bf16 64x256x288 patch movers two groups", 64, 256, false, 2, 448, 2, 0) \
    X("bf16 64x256x288 patch movers two groups swap", 64, 256, true, 2, 448, 2, 0) \
    X("bf16 128x256x144 patch movers", 128, 256, false, 1, 512, 2, 1) \
    X("bf16 128x256x144 patch movers swap", 128, 256, true, 1, 512, 2, 1)
#define IGC_BF16S_INSTANTIATE(NAME, BM, BN, SWAP, GROUPS, PIX, DA, SLACK) \
    template __global__ void igconv_fwd_bf16s_kernel<Bf16sConfig<BM, BN, SWAP, GROUPS, PIX, DA, SLACK>>(const ConvKernelParams);
IGC_BF16S_LIST(IGC_BF16S_INSTANTIATE)

#if !defined(__HIP_DEVICE_COMPILE__)
// (variant 3: the kernels with moving wavefronts)
#define IGC_BF16S_ROW(NAME, BM, BN, SWAP, GROUPS, PIX, DA, SLACK)                                 \
    {NAME, true, BM, BN, Bf16sConfig<BM, BN, SWAP, GROUPS, PIX, DA, SLACK>::BK, SWAP, true, 5,     \
     Bf16sConfig<BM, BN, SWAP, GROUPS, PIX, DA, SLACK>::THREADS,                                   \
     Bf16sConfig<BM, BN, SWAP, GROUPS, PIX, DA, SLACK>::LDS_BYTES,                                 \
     &launch_bf16s<Bf16sConfig<BM, BN, SWAP, GROUPS, PIX, DA, SLACK>>, 3, false, PIX},
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
static const KernelInfo kRows[] = {IGC_BF16C_LIST(IGC_BF16C_ROW) IGC_BF16C_TEAMS_LIST(IGC_BF16C_TEAMS_ROW) IGC_BF16S_LIST(IGC_BF16S_ROW)};
const KernelGroup kGroupBF16Channels = {kRows, sizeof(kRows) / sizeof(kRows[0])};
#endif

}  // namespace igc
