// fp32 kernels for few output elements and long reductions: 32 x 32 tiles, the reduction cut among the wavefronts of
// a workgroup, MFMA operands loaded straight from global memory (igconv_kernel_f32d.hpp).
#include "igconv_instantiate.hpp"
#include "igconv_kernel_f32d.hpp"

namespace igc {

template <class Cfg>
static int launch_f32d(const ConvKernelParams &p, int grid, void *stream) {
    return launch_checked(&igconv_f32d_kernel<Cfg>, "igconv_f32d_kernel", p, grid, Cfg::THREADS, stream);
}

//    name, wavefronts, 16-byte filter loads, runs of four reduction indices per lane and step, filter rows staged in LDS,
//    zero border (gather mode 16)
#define IGC_F32D_LIST(X) \
    X("f32 32x32x8 direct waves8", 8, false, 1, false, false) \
    X("f32 32x32x8 direct waves8 vecw", 8, true, 1, false, false) \
    X("f32 32x32x8 direct waves16 vecw", 16, true, 1, false, false) \
    X("f32 32x32x8 direct waves8 vecw rows staged", 8, true, 1, true, false) \
    X("f32 32x32x8 direct waves8 vecw border", 8, true, 1, false, true) \
    X("f32 32x32x8 direct waves8 vecw rows staged border", 8, true, 1, true, true)

#define IGC_F32D_INSTANTIATE(NAME, WAVES, VECA, NV, ALDS, MSK) \
    template __global__ void igconv_f32d_kernel<DirectConfig<WAVES, VECA, NV, ALDS, MSK>>(const ConvKernelParams);
IGC_F32D_LIST(IGC_F32D_INSTANTIATE)

#if !defined(__HIP_DEVICE_COMPILE__)
// (variant 1: the filter rows staged in LDS - steps per wavefront in eights, four register sets of gathers)
#define IGC_F32D_ROW(NAME, WAVES, VECA, NV, ALDS, MSK) \
    {NAME, false, 32, 32, 8 * NV, false, VECA, MSK ? 16 : 15, 64 * WAVES, DirectConfig<WAVES, VECA, NV, ALDS, MSK>::LDS_BYTES, \
     &launch_f32d<DirectConfig<WAVES, VECA, NV, ALDS, MSK>>, ALDS ? 1 : 0},
static const KernelInfo kRows[] = {IGC_F32D_LIST(IGC_F32D_ROW)};
const KernelGroup kGroupF32Direct = {kRows, sizeof(kRows) / sizeof(kRows[0])};
#endif

}  // namespace igc
