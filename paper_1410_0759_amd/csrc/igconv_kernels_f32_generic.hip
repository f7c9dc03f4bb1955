// fp32 kernels (v_mfma_f32_32x32x2_f32), generic gather (any R, S, pad), both epilogues.
#include "igconv_instantiate.hpp"

//    name, bf16, BM, BN, BK, WM, WN, swap, veca, gather mode
#define IGC_KERNEL_LIST(X) \
    X("f32 64x128x32 generic", false, 64, 128, 32, 2, 2, false, false, GATHER_GENERIC) \
    X("f32 64x128x32 generic vecw", false, 64, 128, 32, 2, 2, false, true, GATHER_GENERIC) \
    X("f32 128x128x32 generic", false, 128, 128, 32, 2, 2, false, false, GATHER_GENERIC) \
    X("f32 128x128x32 generic vecw", false, 128, 128, 32, 2, 2, false, true, GATHER_GENERIC) \
    X("f32 64x128x32 generic swap", false, 64, 128, 32, 2, 2, true, false, GATHER_GENERIC) \
    X("f32 64x128x32 generic swap vecw", false, 64, 128, 32, 2, 2, true, true, GATHER_GENERIC) \
    X("f32 128x128x32 generic swap", false, 128, 128, 32, 2, 2, true, false, GATHER_GENERIC) \
    X("f32 128x128x32 generic swap vecw", false, 128, 128, 32, 2, 2, true, true, GATHER_GENERIC)

IGC_DEFINE_GROUP(kGroupF32Generic)
