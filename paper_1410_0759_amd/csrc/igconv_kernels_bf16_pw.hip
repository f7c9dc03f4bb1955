// bf16 kernels for 1x1 filters over channel-contiguous inputs.
#include "igconv_instantiate.hpp"
#include "igconv_kernel_bf16_pw.hpp"

namespace igc {

template <class Cfg>
static int launch_pw(const ConvKernelParams &p, int grid, void *stream) {
    return launch_checked(&igconv_fwd_bf16_pw_kernel<Cfg>, "igconv_fwd_bf16_pw_kernel", p, grid, Cfg::THREADS, stream);
}

#define IGC_PW_LIST(X)                                      \
    X("bf16 128x128x64 pointwise", 128, 128, false)         \
    X("bf16 64x128x64 pointwise", 64, 128, false)           \
    X("bf16 128x128x64 pointwise swap", 128, 128, true)     \
    X("bf16 64x128x64 pointwise swap", 64, 128, true)

#define IGC_PW_INSTANTIATE(NAME, BM, BN, SWAP) \
    template __global__ void igconv_fwd_bf16_pw_kernel<Bf16PwConfig<BM, BN, SWAP>>(const ConvKernelParams);
IGC_PW_LIST(IGC_PW_INSTANTIATE)

#if !defined(__HIP_DEVICE_COMPILE__)
#define IGC_PW_ROW(NAME, BM, BN, SWAP) \
    {NAME, true, BM, BN, kPwBK, SWAP, true, 12, Bf16PwConfig<BM, BN, SWAP>::THREADS, Bf16PwConfig<BM, BN, SWAP>::LDS_BYTES, &launch_pw<Bf16PwConfig<BM, BN, SWAP>>},
static const KernelInfo kRows[] = {IGC_PW_LIST(IGC_PW_ROW)};
const KernelGroup kGroupBF16Pointwise = {kRows, sizeof(kRows) / sizeof(kRows[0])};
#endif

}  // namespace igc
