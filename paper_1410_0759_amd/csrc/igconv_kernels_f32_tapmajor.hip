// fp32 kernels (v_mfma_f32_32x32x2_f32), tap-major reduction order, NCHW-style epilogue.
#include "igconv_instantiate.hpp"

//    name, bf16, BM, BN, BK, WM, WN, swap, veca, gather mode
#define IGC_KERNEL_LIST(X) \
    X("f32 32x128x32 tapmajor", false, 32, 128, 32, 1, 4, false, false, GATHER_TAPMAJOR) \
    X("f32 64x128x32 tapmajor", false, 64, 128, 32, 2, 2, false, false, GATHER_TAPMAJOR) \
    X("f32 96x128x32 tapmajor", false, 96, 128, 32, 1, 4, false, false, GATHER_TAPMAJOR) \
    X("f32 128x128x32 tapmajor", false, 128, 128, 32, 2, 2, false, false, GATHER_TAPMAJOR)

IGC_DEFINE_GROUP(kGroupF32TapMajor)
