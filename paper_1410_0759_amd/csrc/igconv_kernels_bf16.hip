// bf16-input kernels (v_mfma_f32_32x32x16_bf16, fp32 accumulate and output).
#include "igconv_instantiate.hpp"

//    name, bf16, BM, BN, BK, WM, WN, swap, veca, gather mode
#define IGC_KERNEL_LIST(X) \
    X("bf16 64x128x32 generic", true, 64, 128, 32, 2, 2, false, false, GATHER_GENERIC) \
    X("bf16 64x128x32 generic vecw", true, 64, 128, 32, 2, 2, false, true, GATHER_GENERIC) \
    X("bf16 128x128x32 generic", true, 128, 128, 32, 2, 2, false, false, GATHER_GENERIC) \
    X("bf16 128x128x32 generic vecw", true, 128, 128, 32, 2, 2, false, true, GATHER_GENERIC) \
    X("bf16 64x128x32 generic swap", true, 64, 128, 32, 2, 2, true, false, GATHER_GENERIC) \
    X("bf16 64x128x32 generic swap vecw", true, 64, 128, 32, 2, 2, true, true, GATHER_GENERIC) \
    X("bf16 128x128x32 generic swap", true, 128, 128, 32, 2, 2, true, false, GATHER_GENERIC) \
    X("bf16 128x128x32 generic swap vecw", true, 128, 128, 32, 2, 2, true, true, GATHER_GENERIC) \
    X("bf16 64x128x32 tapmajor", true, 64, 128, 32, 2, 2, false, false, GATHER_TAPMAJOR) \
    X("bf16 128x128x32 tapmajor", true, 128, 128, 32, 2, 2, false, false, GATHER_TAPMAJOR) \
    X("bf16 64x128x32 tapmajor swap", true, 64, 128, 32, 2, 2, true, false, GATHER_TAPMAJOR) \
    X("bf16 128x128x32 tapmajor swap", true, 128, 128, 32, 2, 2, true, false, GATHER_TAPMAJOR)

IGC_DEFINE_GROUP(kGroupBF16)
