// fp32 kernels (v_mfma_f32_32x32x2_f32), fast gathers with the channel-fastest (NHWC-style) epilogue.
#include "igconv_instantiate.hpp"

//    name, bf16, BM, BN, BK, WM, WN, swap, veca, gather mode
#define IGC_KERNEL_LIST(X) \
    X("f32 64x128x32 tapmajor swap", false, 64, 128, 32, 2, 2, true, false, GATHER_TAPMAJOR) \
    X("f32 128x128x32 tapmajor swap", false, 128, 128, 32, 2, 2, true, false, GATHER_TAPMAJOR) \
    X("f32 64x128x32 nopad swap", false, 64, 128, 32, 2, 2, true, false, GATHER_NOPAD) \
    X("f32 64x128x32 nopad swap vecw", false, 64, 128, 32, 2, 2, true, true, GATHER_NOPAD) \
    X("f32 128x128x32 nopad swap", false, 128, 128, 32, 2, 2, true, false, GATHER_NOPAD) \
    X("f32 128x128x32 nopad swap vecw", false, 128, 128, 32, 2, 2, true, true, GATHER_NOPAD)

IGC_DEFINE_GROUP(kGroupF32Swap)
