// bf16-input kernel variants (v_mfma_f32_32x32x16_bf16, fp32 accumulate and output).
#include "igconv_instantiate.hpp"

//    name                         bf16  BM   BN  BK WM WN swap   veca
#define IGC_KERNEL_LIST(X)                                              \
    X("bf16 64x128x32",            true, 64, 128, 32, 2, 2, false, false) \
    X("bf16 64x128x32 vecw",       true, 64, 128, 32, 2, 2, false, true)  \
    X("bf16 128x128x32",           true, 128, 128, 32, 2, 2, false, false) \
    X("bf16 128x128x32 vecw",      true, 128, 128, 32, 2, 2, false, true)  \
    X("bf16 64x128x32 swap",       true, 64, 128, 32, 2, 2, true, false)  \
    X("bf16 64x128x32 swap vecw",  true, 64, 128, 32, 2, 2, true, true)   \
    X("bf16 128x128x32 swap",      true, 128, 128, 32, 2, 2, true, false) \
    X("bf16 128x128x32 swap vecw", true, 128, 128, 32, 2, 2, true, true)

namespace igc {

IGC_KERNEL_LIST(IGC_INSTANTIATE)

#if !defined(__HIP_DEVICE_COMPILE__)
const KernelInfo kKernelsBF16[] = {IGC_KERNEL_LIST(IGC_TABLE_ROW)};
const int kNumKernelsBF16 = sizeof(kKernelsBF16) / sizeof(kKernelsBF16[0]);
#endif

}  // namespace igc
