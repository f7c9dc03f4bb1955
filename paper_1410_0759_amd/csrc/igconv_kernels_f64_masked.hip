// Double-precision kernels with the pipelined masked gather (igconv_kernel_f64m.hpp): forward pass and backward-data
// phases of filters with up to 63 taps.
#include "igconv_instantiate.hpp"
#include "igconv_kernel_f64m.hpp"

namespace igc {

template <class Cfg>
static int launch_f64m(const ConvKernelParams &p, int grid, void *stream) {
    return launch_checked(&igconv_f64m_kernel<Cfg>, "igconv_f64m_kernel", p, grid, 256, stream);
}

//    name, BM, BN, 16-byte filter loads
#define IGC_F64M_LIST(X) \
    X("f64 64x64x16 masked", 64, 64, false) \
    X("f64 64x64x16 masked vecw", 64, 64, true) \
    X("f64 128x64x16 masked", 128, 64, false) \
    X("f64 128x64x16 masked vecw", 128, 64, true)

#define IGC_F64M_INSTANTIATE(NAME, BM, BN, VECA) \
    template __global__ void igconv_f64m_kernel<F64mConfig<BM, BN, VECA>>(const ConvKernelParams);
IGC_F64M_LIST(IGC_F64M_INSTANTIATE)

#if !defined(__HIP_DEVICE_COMPILE__)
static KernelInfo f64m_row(const char *name, int bm, int bn, bool veca, int lds, int (*launch)(const ConvKernelParams &, int, void *)) {
    KernelInfo k{name, false, bm, bn, 16, false, veca, 14, 256, lds, launch};
    k.f64 = true;
    return k;
}
#define IGC_F64M_ROW(NAME, BM, BN, VECA) f64m_row(NAME, BM, BN, VECA, F64mConfig<BM, BN, VECA>::LDS_BYTES, &launch_f64m<F64mConfig<BM, BN, VECA>>),
static const KernelInfo kRows[] = {IGC_F64M_LIST(IGC_F64M_ROW)};
const KernelGroup kGroupF64Masked = {kRows, sizeof(kRows) / sizeof(kRows[0])};
#endif

}  // namespace igc
