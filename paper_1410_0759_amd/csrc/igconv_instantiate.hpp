// Helper shared by the translation units that instantiate kernels.  A unit defines
// IGC_KERNEL_LIST(X) as a list of X(name, bf16, BM, BN, BK, WM, WN, swap, veca) and
// expands it twice: once to instantiate the device code, once (host pass only) to
// fill its slice of the kernel table.
#ifndef IGCONV_INSTANTIATE_HPP_
#define IGCONV_INSTANTIATE_HPP_

#include "igconv_kernel.hpp"
#include "igconv_kernel_table.h"

namespace igc {

template <class Cfg>
int launch_kernel(const ConvKernelParams &p, int grid, void *stream) {
    hipLaunchKernelGGL(igconv_fwd_kernel<Cfg>, dim3(grid), dim3(Cfg::THREADS), 0,
                       static_cast<hipStream_t>(stream), p);
    return static_cast<int>(hipGetLastError());
}

#define IGC_INSTANTIATE(NAME, BF16, BM, BN, BK, WM, WN, SWAP, VECA) \
    template __global__ void igconv_fwd_kernel<KernelConfig<BF16, BM, BN, BK, WM, WN, SWAP, VECA>>(const ConvKernelParams);

#define IGC_TABLE_ROW(NAME, BF16, BM, BN, BK, WM, WN, SWAP, VECA)                               \
    {NAME, BF16, BM, BN, BK, SWAP, VECA, 256,                                                   \
     KernelConfig<BF16, BM, BN, BK, WM, WN, SWAP, VECA>::LDS_BYTES,                             \
     &launch_kernel<KernelConfig<BF16, BM, BN, BK, WM, WN, SWAP, VECA>>},

}  // namespace igc
#endif
