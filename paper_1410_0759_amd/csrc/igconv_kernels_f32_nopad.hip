// fp32 kernels (v_mfma_f32_32x32x2_f32), unpadded gather in filter order, NCHW-style epilogue.
#include "igconv_instantiate.hpp"

//    name, bf16, BM, BN, BK, WM, WN, swap, veca, gather mode
#define IGC_KERNEL_LIST(X) \
    X("f32 32x128x32 nopad", false, 32, 128, 32, 1, 4, false, false, GATHER_NOPAD) \
    X("f32 32x128x32 nopad vecw", false, 32, 128, 32, 1, 4, false, true, GATHER_NOPAD) \
    X("f32 64x128x32 nopad", false, 64, 128, 32, 2, 2, false, false, GATHER_NOPAD) \
    X("f32 64x128x32 nopad vecw", false, 64, 128, 32, 2, 2, false, true, GATHER_NOPAD) \
    X("f32 96x128x32 nopad", false, 96, 128, 32, 1, 4, false, false, GATHER_NOPAD) \
    X("f32 96x128x32 nopad vecw", false, 96, 128, 32, 1, 4, false, true, GATHER_NOPAD) \
    X("f32 128x128x32 nopad", false, 128, 128, 32, 2, 2, false, false, GATHER_NOPAD) \
    X("f32 128x128x32 nopad vecw", false, 128, 128, 32, 2, 2, false, true, GATHER_NOPAD) \
    X("f32 64x64x32 nopad", false, 64, 64, 32, 2, 2, false, false, GATHER_NOPAD) \
    X("f32 64x64x32 nopad vecw", false, 64, 64, 32, 2, 2, false, true, GATHER_NOPAD) \
    X("f32 32x128x32 nopad table", false, 32, 128, 32, 1, 4, false, false, GATHER_NOPAD_TABLE) \
    X("f32 64x128x32 nopad table", false, 64, 128, 32, 2, 2, false, false, GATHER_NOPAD_TABLE) \
    X("f32 96x128x32 nopad table", false, 96, 128, 32, 1, 4, false, false, GATHER_NOPAD_TABLE) \
    X("f32 128x128x32 nopad table", false, 128, 128, 32, 2, 2, false, false, GATHER_NOPAD_TABLE) \
    X("f32 96x128x32 nopad table vecw", false, 96, 128, 32, 1, 4, false, true, GATHER_NOPAD_TABLE) \
    X("f32 128x128x32 nopad table vecw", false, 128, 128, 32, 2, 2, false, true, GATHER_NOPAD_TABLE) \
    X("f32 96x128x16 nopad table", false, 96, 128, 16, 1, 4, false, false, GATHER_NOPAD_TABLE) \
    X("f32 96x128x16 nopad table odd", false, 96, 128, 16, 1, 4, false, false, GATHER_NOPAD_TABLE_ODD) \
    X("f32 64x128x16 nopad table", false, 64, 128, 16, 2, 2, false, false, GATHER_NOPAD_TABLE) \
    X("f32 64x128x16 nopad table odd", false, 64, 128, 16, 2, 2, false, false, GATHER_NOPAD_TABLE_ODD) \
    X("f32 32x128x32 nopad table short", false, 32, 128, 32, 1, 4, false, false, GATHER_NOPAD_TABLE_SHORT) \
    X("f32 64x128x32 nopad table short", false, 64, 128, 32, 2, 2, false, false, GATHER_NOPAD_TABLE_SHORT) \
    X("f32 96x128x32 nopad table short", false, 96, 128, 32, 1, 4, false, false, GATHER_NOPAD_TABLE_SHORT) \
    X("f32 128x128x32 nopad table short", false, 128, 128, 32, 2, 2, false, false, GATHER_NOPAD_TABLE_SHORT)

IGC_DEFINE_GROUP(kGroupF32Nopad)
