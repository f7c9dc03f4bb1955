// fp32 kernels (v_mfma_f32_32x32x2_f32), filter-order reduction with the tap tracked by the scalar unit and the
// window test read from a 64-bit mask per column (up to 63 taps, any pad), both epilogues.
#include "igconv_instantiate.hpp"

//    name, bf16, BM, BN, BK, WM, WN, swap, veca, gather mode
#define IGC_KERNEL_LIST(X) \
    X("f32 64x128x32 masked", false, 64, 128, 32, 2, 2, false, false, GATHER_MASKED) \
    X("f32 64x128x32 masked vecw", false, 64, 128, 32, 2, 2, false, true, GATHER_MASKED) \
    X("f32 96x128x32 masked", false, 96, 128, 32, 1, 4, false, false, GATHER_MASKED) \
    X("f32 96x128x32 masked vecw", false, 96, 128, 32, 1, 4, false, true, GATHER_MASKED) \
    X("f32 128x128x32 masked", false, 128, 128, 32, 2, 2, false, false, GATHER_MASKED) \
    X("f32 128x128x32 masked vecw", false, 128, 128, 32, 2, 2, false, true, GATHER_MASKED) \
    X("f32 64x128x32 masked swap", false, 64, 128, 32, 2, 2, true, false, GATHER_MASKED) \
    X("f32 64x128x32 masked swap vecw", false, 64, 128, 32, 2, 2, true, true, GATHER_MASKED) \
    X("f32 128x128x32 masked swap", false, 128, 128, 32, 2, 2, true, false, GATHER_MASKED) \
    X("f32 128x128x32 masked swap vecw", false, 128, 128, 32, 2, 2, true, true, GATHER_MASKED)

IGC_DEFINE_GROUP(kGroupF32Masked)
