// Backward-filter kernels: the generic gather with columns (c,r,s) and the reduction over
// (n,p,q), plus the kernel that adds up the ranges of a cut reduction.
#include "igconv_instantiate.hpp"

//    name, bf16, BM, BN, BK, WM, WN, swap, veca, gather mode
#define IGC_KERNEL_LIST(X) \
    X("f32 64x128x32 wgrad", false, 64, 128, 32, 2, 2, false, false, GATHER_WGRAD) \
    X("f32 128x128x32 wgrad", false, 128, 128, 32, 2, 2, false, false, GATHER_WGRAD) \
    X("bf16 64x128x32 wgrad", true, 64, 128, 32, 2, 2, false, false, GATHER_WGRAD) \
    X("bf16 128x128x32 wgrad", true, 128, 128, 32, 2, 2, false, false, GATHER_WGRAD) \
    X("f32 64x64x32 wgrad tap", false, 64, 64, 32, 2, 2, false, false, GATHER_WGRAD_TAP) \
    X("f32 128x64x32 wgrad tap", false, 128, 64, 32, 2, 2, false, false, GATHER_WGRAD_TAP) \
    X("f32 64x128x32 wgrad tap", false, 64, 128, 32, 2, 2, false, false, GATHER_WGRAD_TAP) \
    X("f32 128x128x32 wgrad tap", false, 128, 128, 32, 2, 2, false, false, GATHER_WGRAD_TAP) \
    X("bf16 64x64x32 wgrad tap", true, 64, 64, 32, 2, 2, false, false, GATHER_WGRAD_TAP) \
    X("bf16 128x64x32 wgrad tap", true, 128, 64, 32, 2, 2, false, false, GATHER_WGRAD_TAP) \
    X("bf16 64x128x32 wgrad tap", true, 64, 128, 32, 2, 2, false, false, GATHER_WGRAD_TAP) \
    X("bf16 128x128x32 wgrad tap", true, 128, 128, 32, 2, 2, false, false, GATHER_WGRAD_TAP) \
    X("f32 64x128x32 wgrad nopad", false, 64, 128, 32, 2, 2, false, false, GATHER_WGRAD_NOPAD) \
    X("f32 96x128x32 wgrad nopad", false, 96, 128, 32, 1, 4, false, false, GATHER_WGRAD_NOPAD) \
    X("f32 128x128x32 wgrad nopad", false, 128, 128, 32, 2, 2, false, false, GATHER_WGRAD_NOPAD) \
    X("f32 96x128x32 wgrad tap", false, 96, 128, 32, 1, 4, false, false, GATHER_WGRAD_TAP) \
    X("f32 96x128x32 wgrad", false, 96, 128, 32, 1, 4, false, false, GATHER_WGRAD) \
    X("bf16 64x128x32 wgrad nopad", true, 64, 128, 32, 2, 2, false, false, GATHER_WGRAD_NOPAD) \
    X("bf16 128x128x32 wgrad nopad", true, 128, 128, 32, 2, 2, false, false, GATHER_WGRAD_NOPAD)

IGC_DEFINE_GROUP(kGroupWgrad)

namespace igc {

// out[e] = alpha * (part_0[e] + part_1[e] + ...) + beta * out[e], parts `stride` floats apart.
// The order of the additions is fixed by `count` alone, so the result does not depend on how the
// work was spread: the parts are cut into eight consecutive runs, a workgroup of 256 threads takes
// 32 elements and gives each run to 32 of its threads (which add the run's parts in order, four
// loads in flight), and the eight sums are added in order through LDS.  (One thread per element
// adding all parts kept one load in flight per thread, on a fraction of the chip: 112 parts of
// 147 KB took 28 us.)
__global__ __launch_bounds__(256) void igconv_sum_parts_kernel(const float *parts, float *out, uint32_t n, int count,
                                                               uint32_t stride, float alpha, float beta) {
    __shared__ float runs[8][32];
    const uint32_t el = threadIdx.x & 31u, g = threadIdx.x >> 5;
    const uint32_t e = blockIdx.x * 32u + el;
    const int per = (count + 7) / 8, s0 = (int)g * per, s1 = min(count, s0 + per);
    float acc = 0.f;
    if (e < n) {
        const float *src = parts + e;
        int s = s0;
        for (; s + 4 <= s1; s += 4) {
            const float a = src[(size_t)s * stride], b = src[(size_t)(s + 1) * stride], c = src[(size_t)(s + 2) * stride],
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
    float sum = runs[0][el];
#pragma unroll
    for (int k = 1; k < 8; ++k) sum += runs[k][el];
    float r = alpha * sum;
    if (beta != 0.f) r += beta * out[e];
    out[e] = r;
}

int launch_sum_parts(const float *parts, float *out, uint32_t n, int count, uint32_t stride, float alpha, float beta,
                     void *stream) {
    void *argv[] = {&parts, &out, &n, &count, &stride, &alpha, &beta};
    return static_cast<int>(hipLaunchKernel(reinterpret_cast<const void *>(&igconv_sum_parts_kernel), dim3((n + 31u) / 32u),
                                            dim3(256), argv, 0, static_cast<hipStream_t>(stream)));
}

// wt[c][k][t] = w[k][c][t] for 2-byte elements (t: the taps of one (k,c) pair, kept in order):
// a workgroup moves a block of 16 k x 16 c through LDS so that both sides are read and
// written in runs of 16*taps elements.  Host guarantees sizes below 2^31.
template <int taps>
__global__ __launch_bounds__(256) void igconv_filter_exchange_kernel(const uint16_t *w, uint16_t *wt, int K, int C) {
    __shared__ uint16_t blk[16 * 16 * taps];
    const int k0 = blockIdx.x * 16, c0 = blockIdx.y * 16;
    const int run = 16 * taps, total = 16 * run;
    // (total = 256 * taps: every thread moves `taps` elements, all requested before the first is written to LDS)
    uint16_t v[taps];
#pragma unroll
    for (int i = 0; i < taps; ++i) {
        const int e = (int)threadIdx.x + 256 * i;
        const int k = e / run, rem = e - k * run;     // rem = c_local * taps + t
        const int c = rem / taps;
        v[i] = 0;
        if (k0 + k < K && c0 + c < C) v[i] = w[((size_t)(k0 + k) * C + c0) * taps + rem];
    }
#pragma unroll
    for (int i = 0; i < taps; ++i) blk[threadIdx.x + 256 * i] = v[i];
    __syncthreads();
    for (int e = threadIdx.x; e < total; e += 256) {
        const int c = e / run, rem = e - c * run;     // rem = k_local * taps + t
        const int k = rem / taps, t = rem - k * taps;
        if (k0 + k < K && c0 + c < C) wt[((size_t)(c0 + c) * K + k0) * taps + rem] = blk[(k * 16 + c) * taps + t];
    }
}

int launch_filter_exchange(const void *w, void *wt, int K, int C, int taps, void *stream) {
    void *argv[] = {&w, &wt, &K, &C};
    const void *kernel = taps == 9 ? reinterpret_cast<const void *>(&igconv_filter_exchange_kernel<9>)
                                   : reinterpret_cast<const void *>(&igconv_filter_exchange_kernel<1>);
    return static_cast<int>(hipLaunchKernel(kernel,
                                            dim3((K + 15) / 16, (C + 15) / 16), dim3(256), argv, 0,
                                            static_cast<hipStream_t>(stream)));
}

}  // namespace igc
