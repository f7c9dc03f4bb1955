// Double-precision kernels (v_mfma_f64_16x16x4_f64) and the ordered sum of double partial results.
#include <cstdio>
#include <cstdlib>

#include "igconv_kernel_f64.hpp"
#include "igconv_kernel_table.h"

namespace igc {

template <bool WGRAD, int NB>
static int launch_f64(const ConvKernelParams &p, int grid, void *stream) {
    ConvKernelParams args = p;
    void *argv[] = {&args};
    const hipError_t e = hipLaunchKernel(reinterpret_cast<const void *>(&igconv_f64_kernel<WGRAD, NB>), dim3(grid), dim3(kF64Threads), argv, 0,
                                         static_cast<hipStream_t>(stream));
    if (e != hipSuccess && std::getenv("IGCONV_DEBUG"))
        std::fprintf(stderr, "igconv: launch of igconv_f64_kernel failed: %s\n", hipGetErrorString(e));
    return static_cast<int>(e);
}

template __global__ void igconv_f64_kernel<false, 2>(const ConvKernelParams);
template __global__ void igconv_f64_kernel<true, 2>(const ConvKernelParams);

// out[e] = alpha * (part_0[e] + part_1[e] + ...) + beta * out[e] in double.  The order of the additions is
// fixed by `count` alone: eight consecutive runs of parts, each added in order by 32 threads of the workgroup
// (four loads in flight), the eight sums added in order through LDS.
__global__ __launch_bounds__(256) void igconv_sum_parts_f64_kernel(const double *parts, double *out, uint32_t n, int count,
                                                                   uint32_t stride, double alpha, double beta) {
    __shared__ double runs[8][32];
    const uint32_t el = threadIdx.x & 31u, g = threadIdx.x >> 5;
    const uint32_t e = blockIdx.x * 32u + el;
    const int per = (count + 7) / 8, s0 = (int)g * per, s1 = min(count, s0 + per);
    double acc = 0.0;
    if (e < n) {
        const double *src = parts + e;
        int s = s0;
        for (; s + 4 <= s1; s += 4) {
            const double a = src[(size_t)s * stride], b = src[(size_t)(s + 1) * stride], c = src[(size_t)(s + 2) * stride],
                         d = src[(size_t)(s + 3) * stride];
            acc += a;
            acc += b;
            acc += c;
            acc += d;
        }
        for (; s < s1; ++s) acc += src[(size_t)s * stride];
    }
    runs[g][el] = acc;
    __syncthreads();
    if (g != 0 || e >= n) return;
    double sum = runs[0][el];
#pragma unroll
    for (int k = 1; k < 8; ++k) sum += runs[k][el];
    double r = alpha * sum;
    if (beta != 0.0) r += beta * out[e];
    out[e] = r;
}

int launch_sum_parts_f64(const double *parts, double *out, uint32_t n, int count, uint32_t stride, double alpha, double beta,
                         void *stream) {
    void *argv[] = {&parts, &out, &n, &count, &stride, &alpha, &beta};
    return static_cast<int>(hipLaunchKernel(reinterpret_cast<const void *>(&igconv_sum_parts_f64_kernel), dim3((n + 31u) / 32u),
                                            dim3(256), argv, 0, static_cast<hipStream_t>(stream)));
}

#if !defined(__HIP_DEVICE_COMPILE__)
static KernelInfo f64_row(const char *name, int nb, int gmode, int (*launch)(const ConvKernelParams &, int, void *)) {
    KernelInfo k{name, false, 32 * nb, 32 * nb, kF64BK, false, false, gmode, kF64Threads, f64_lds_bytes(nb), launch};
    k.f64 = true;
    return k;
}
static const KernelInfo kRows[] = {f64_row("f64 64x64x16 generic", 2, 0, &launch_f64<false, 2>),
                                   f64_row("f64 64x64x16 wgrad", 2, 6, &launch_f64<true, 2>)};
const KernelGroup kGroupF64 = {kRows, sizeof(kRows) / sizeof(kRows[0])};
#endif

}  // namespace igc
