// fp32 kernels with several teams of four wavefronts per workgroup (see KernelConfig::TEAMS): one
// tile per workgroup, the reduction steps divided among the teams, their sums added through LDS.
#include "igconv_instantiate.hpp"

namespace igc {

//    name, BM, BN, BK, WM, WN, veca, gather mode, teams
#define IGC_TEAMS_LIST(X) \
    X("f32 64x64x32 nopad teams4", 64, 64, 32, 2, 2, false, GATHER_NOPAD, 4) \
    X("f32 64x64x32 nopad vecw teams4", 64, 64, 32, 2, 2, true, GATHER_NOPAD, 4) \
    X("f32 64x128x32 nopad vecw teams2", 64, 128, 32, 2, 2, true, GATHER_NOPAD, 2) \
    X("f32 64x64x72 taps9 teams2", 64, 64, 72, 2, 2, true, GATHER_TAPS9, 2)

#define IGC_TEAMS_INSTANTIATE(NAME, BM, BN, BK, WM, WN, VECA, GMODE, TEAMS) \
    template __global__ void igconv_fwd_kernel<KernelConfig<false, BM, BN, BK, WM, WN, false, VECA, GMODE, TEAMS>>(const ConvKernelParams);
IGC_TEAMS_LIST(IGC_TEAMS_INSTANTIATE)

#if !defined(__HIP_DEVICE_COMPILE__)
// (variant 2: teams; `threads` tells how many)
#define IGC_TEAMS_ROW(NAME, BM, BN, BK, WM, WN, VECA, GMODE, TEAMS)                                        \
    {NAME, false, BM, BN, BK, false, VECA, GMODE, 256 * TEAMS,                                            \
     KernelConfig<false, BM, BN, BK, WM, WN, false, VECA, GMODE, TEAMS>::LDS_BYTES,                       \
     &launch_kernel<KernelConfig<false, BM, BN, BK, WM, WN, false, VECA, GMODE, TEAMS>>, 2},
static const KernelInfo kRows[] = {IGC_TEAMS_LIST(IGC_TEAMS_ROW)};
const KernelGroup kGroupF32Teams = {kRows, sizeof(kRows) / sizeof(kRows[0])};
#endif

}  // namespace igc
