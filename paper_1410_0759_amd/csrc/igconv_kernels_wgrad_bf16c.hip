// Backward-filter kernels for bf16 tensors with contiguous channels (tiles transposed in
// registers on their way into LDS).
#include <cstdio>
#include <cstdlib>

#include "igconv_kernel_table.h"
#include "igconv_kernel_wgrad_bf16c.hpp"

namespace igc {

template <class Cfg>
static int launch_wgc(const ConvKernelParams &p, int grid, void *stream) {
    ConvKernelParams args = p;
    void *argv[] = {&args};
    const hipError_t e = hipLaunchKernel(reinterpret_cast<const void *>(&igconv_wgrad_bf16c_kernel<Cfg>), dim3(grid), dim3(Cfg::THREADS),
                                         argv, 0, static_cast<hipStream_t>(stream));
    if (e != hipSuccess && std::getenv("IGCONV_DEBUG"))
        std::fprintf(stderr, "igconv: launch of igconv_wgrad_bf16c_kernel failed: %s\n", hipGetErrorString(e));
    return static_cast<int>(e);
}

// out[k][c][t] = alpha * sum over the parts of part[t][row position of k][column position of c] + beta * out[k][c][t]:
// adds the ranges in order and undoes the order the channel-vector kernels keep their results in
// (channel 8 cv + ch of a tile of B channels sits at position ch*(B/8) + cv; parts are KP x CP positions per tap).
// One thread per (row position, column position), lanes along the column positions: every tap's read is a
// contiguous run per wavefront, and a thread writes the R*S taps of its (k, c), contiguous in dw.
__global__ __launch_bounds__(256) void igconv_sum_positions_kernel(const float *__restrict__ parts, float *__restrict__ out, uint32_t n, int count,
                                                                   uint32_t stride, float alpha, float beta, int C, int RS,
                                                                   int BM, int BN, int KP, int CP) {
    const uint32_t e = blockIdx.x * 256u + threadIdx.x;
    if (e >= (uint32_t)KP * (uint32_t)CP) return;
    const uint32_t row = e / (uint32_t)CP, col = e - row * (uint32_t)CP;
    const uint32_t rl = row % (uint32_t)BM, cl = col % (uint32_t)BN;
    const uint32_t nva = (uint32_t)BM / 8u, nvb = (uint32_t)BN / 8u;
    const uint32_t k = row - rl + (rl % nva) * 8u + rl / nva;     // position ch*nv + cv holds channel 8 cv + ch
    const uint32_t c = col - cl + (cl % nvb) * 8u + cl / nvb;
    if (c >= (uint32_t)C || (size_t)(k * (uint32_t)C + c) * RS >= n) return;
    float *dst = out + (size_t)(k * (uint32_t)C + c) * RS;
    // (three taps at a time: their loads are requested together; the parts of a tap are added in order)
    int t = 0;
    for (; t + 3 <= RS; t += 3) {
        const float *s0 = parts + ((size_t)t * KP + row) * CP + col, *s1 = s0 + (size_t)KP * CP, *s2 = s1 + (size_t)KP * CP;
        float a0 = 0.f, a1 = 0.f, a2 = 0.f;
        for (int s = 0; s < count; ++s) {
            const float v0 = s0[(size_t)s * stride], v1 = s1[(size_t)s * stride], v2 = s2[(size_t)s * stride];
            a0 += v0;
            a1 += v1;
            a2 += v2;
        }
        float r0 = alpha * a0, r1 = alpha * a1, r2 = alpha * a2;
        if (beta != 0.f) {
            r0 += beta * dst[t];
            r1 += beta * dst[t + 1];
            r2 += beta * dst[t + 2];
        }
        dst[t] = r0;
        dst[t + 1] = r1;
        dst[t + 2] = r2;
    }
    for (; t < RS; ++t) {
        const size_t src = ((size_t)t * KP + row) * CP + col;
        float acc = 0.f;
        for (int s = 0; s < count; ++s) acc += parts[(size_t)s * stride + src];
        float r = alpha * acc;
        if (beta != 0.f) r += beta * dst[t];
        dst[t] = r;
    }
}

int launch_sum_positions(const float *parts, float *out, uint32_t n, int count, uint32_t stride, float alpha, float beta, int C,
                         int RS, int BM, int BN, int KP, int CP, void *stream) {
    void *argv[] = {&parts, &out, &n, &count, &stride, &alpha, &beta, &C, &RS, &BM, &BN, &KP, &CP};
    const uint32_t threads = (uint32_t)KP * (uint32_t)CP;
    return static_cast<int>(hipLaunchKernel(reinterpret_cast<const void *>(&igconv_sum_positions_kernel), dim3((threads + 255u) / 256u),
                                            dim3(256), argv, 0, static_cast<hipStream_t>(stream)));
}

#define IGC_WGC_LIST(X)                                   \
    X("bf16 128x128x64 wgrad channels", 128, 128)         \
    X("bf16 64x128x64 wgrad channels", 64, 128)           \
    X("bf16 128x64x64 wgrad channels", 128, 64)           \
    X("bf16 64x64x64 wgrad channels", 64, 64)

#define IGC_WGC_INSTANTIATE(NAME, BM, BN) \
    template __global__ void igconv_wgrad_bf16c_kernel<WgradBf16cConfig<BM, BN>>(const ConvKernelParams);
IGC_WGC_LIST(IGC_WGC_INSTANTIATE)
#if !defined(__HIP_DEVICE_COMPILE__)
#define IGC_WGC_ROW(NAME, BM, BN) \
    {NAME, true, BM, BN, kWgcBK, false, true, 10, WgradBf16cConfig<BM, BN>::THREADS, WgradBf16cConfig<BM, BN>::LDS_BYTES, &launch_wgc<WgradBf16cConfig<BM, BN>>},
static const KernelInfo kRows[] = {IGC_WGC_LIST(IGC_WGC_ROW)};
const KernelGroup kGroupWgradBF16Channels = {kRows, sizeof(kRows) / sizeof(kRows[0])};
#endif

}  // namespace igc
