// fp32 kernel variants (v_mfma_f32_32x32x2_f32).
#include "igconv_instantiate.hpp"

//    name                        bf16   BM   BN  BK WM WN swap   veca
#define IGC_KERNEL_LIST(X)                                              \
    X("f32 32x128x32",            false, 32, 128, 32, 1, 4, false, false) \
    X("f32 32x128x32 vecw",       false, 32, 128, 32, 1, 4, false, true)  \
    X("f32 64x128x32",            false, 64, 128, 32, 2, 2, false, false) \
    X("f32 64x128x32 vecw",       false, 64, 128, 32, 2, 2, false, true)  \
    X("f32 64x256x32",            false, 64, 256, 32, 1, 4, false, false) \
    X("f32 64x256x32 vecw",       false, 64, 256, 32, 1, 4, false, true)  \
    X("f32 96x128x32",            false, 96, 128, 32, 1, 4, false, false) \
    X("f32 96x128x32 vecw",       false, 96, 128, 32, 1, 4, false, true)  \
    X("f32 128x128x32",           false, 128, 128, 32, 2, 2, false, false) \
    X("f32 128x128x32 vecw",      false, 128, 128, 32, 2, 2, false, true)  \
    X("f32 64x128x32 swap",       false, 64, 128, 32, 2, 2, true, false)  \
    X("f32 64x128x32 swap vecw",  false, 64, 128, 32, 2, 2, true, true)   \
    X("f32 128x128x32 swap",      false, 128, 128, 32, 2, 2, true, false) \
    X("f32 128x128x32 swap vecw", false, 128, 128, 32, 2, 2, true, true)

namespace igc {

IGC_KERNEL_LIST(IGC_INSTANTIATE)

#if !defined(__HIP_DEVICE_COMPILE__)
const KernelInfo kKernelsF32[] = {IGC_KERNEL_LIST(IGC_TABLE_ROW)};
const int kNumKernelsF32 = sizeof(kKernelsF32) / sizeof(kKernelsF32[0]);
#endif

}  // namespace igc
