// fp32 kernels (v_mfma_f32_32x32x2_f32), nine-tap filters gathered from a per-column tap table, steps of four channels; both epilogues.
// "strided": the filter is read element by element through row / channel / tap strides (backward data, unaligned filters).
#include "igconv_instantiate.hpp"

//    name, bf16, BM, BN, BK, WM, WN, swap, veca, gather mode
#define IGC_KERNEL_LIST(X) \
    X("f32 32x128x36 taps9", false, 32, 128, 36, 1, 4, false, true, GATHER_TAPS9) \
    X("f32 64x128x36 taps9", false, 64, 128, 36, 2, 2, false, true, GATHER_TAPS9) \
    X("f32 96x128x36 taps9", false, 96, 128, 36, 1, 4, false, true, GATHER_TAPS9) \
    X("f32 128x128x36 taps9", false, 128, 128, 36, 2, 2, false, true, GATHER_TAPS9) \
    X("f32 64x128x36 taps9 swap", false, 64, 128, 36, 2, 2, true, true, GATHER_TAPS9) \
    X("f32 96x128x36 taps9 swap", false, 96, 128, 36, 1, 4, true, true, GATHER_TAPS9) \
    X("f32 64x64x72 taps9", false, 64, 64, 72, 2, 2, false, true, GATHER_TAPS9) \
    X("f32 64x128x36 taps9 strided", false, 64, 128, 36, 2, 2, false, false, GATHER_TAPS9) \
    X("f32 96x128x36 taps9 strided", false, 96, 128, 36, 1, 4, false, false, GATHER_TAPS9) \
    X("f32 128x128x36 taps9 strided", false, 128, 128, 36, 2, 2, false, false, GATHER_TAPS9) \
    X("f32 64x128x36 taps9 strided swap", false, 64, 128, 36, 2, 2, true, false, GATHER_TAPS9)

IGC_DEFINE_GROUP(kGroupF32Taps9)
