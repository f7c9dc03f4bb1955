// Measurement aids that belong to the library's test and bench tier (nothing on the hot path
// calls them): the rate of a register-only MFMA loop - the arithmetic ceiling a kernel on this
// chip can reach with the clocks it actually gets, beside the datasheet peak - and the device's
// compute-unit count and clock as the runtime reports them.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "igconv_desc.h"

namespace igc {

using f32x16 = float __attribute__((ext_vector_type(16)));
using f64x4 = double __attribute__((ext_vector_type(4)));
using bf16x8 = __bf16 __attribute__((ext_vector_type(8)));

constexpr int kProbeAcc = 4;      // independent accumulators: back-to-back MFMAs never wait for each other
constexpr int kProbeUnroll = 8;

// The result must leave the kernel or the loop is removed; it leaves through a buffer
// descriptor of size zero, whose stores the hardware drops.
__device__ __forceinline__ void sink(float v) {
    const __amdgpu_buffer_rsrc_t none = __builtin_amdgcn_make_buffer_rsrc(nullptr, 0, 0, 0x00020000u);
    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, v), none, threadIdx.x * 4u, 0, 0);
}

constexpr int kProbeSets = 4;     // operand sets the instructions rotate through

// Operand values of the probe.  Uniform: one value per lane, the same in every set and every instruction (the matrix
// pipes switch few bits: the rate at the highest clocks the chip gives).  Random: finite values of mixed sign and
// magnitude below 1, another set with every instruction, as the operands of a real product change - the pipes then
// draw more power and the chip sustains lower clocks: the ceiling a kernel fed with real data can reach.
__device__ __forceinline__ uint32_t probe_hash(uint32_t x) {
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return x;
}
__device__ __forceinline__ float probe_value(uint32_t index) {   // in [-1, 1)
    return __builtin_bit_cast(float, 0x3F800000u | (probe_hash(index) >> 9)) * 2.f - 3.f;
}

__global__ __launch_bounds__(256) void mfma_rate_f32(int iters, float a0, int random) {
    f32x16 acc[kProbeAcc];
    for (int i = 0; i < kProbeAcc; ++i)
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    float a[kProbeSets], b[kProbeSets];
    for (int s = 0; s < kProbeSets; ++s) {
        const uint32_t id = (blockIdx.x * 256u + threadIdx.x) * 2u * kProbeSets + 2u * s;
        a[s] = random ? probe_value(id) : a0 + threadIdx.x * 1e-9f;
        b[s] = random ? probe_value(id + 1u) : a0 * 2.f;
    }
    for (int it = 0; it < iters; ++it)
#pragma unroll
        for (int u = 0; u < kProbeUnroll; ++u)
#pragma unroll
            for (int i = 0; i < kProbeAcc; ++i)
                acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[(i + u) % kProbeSets], b[(i + 3 * u + 1) % kProbeSets], acc[i], 0, 0, 0);
    float s = 0;
    for (int i = 0; i < kProbeAcc; ++i)
        for (int v = 0; v < 16; ++v) s += acc[i][v];
    sink(s);
}

__global__ __launch_bounds__(256) void mfma_rate_bf16(int iters, float a0, int random) {
    f32x16 acc[kProbeAcc];
    for (int i = 0; i < kProbeAcc; ++i)
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    bf16x8 a[kProbeSets], b[kProbeSets];
    for (int s = 0; s < kProbeSets; ++s)
        for (int i = 0; i < 8; ++i) {
            const uint32_t id = ((blockIdx.x * 256u + threadIdx.x) * kProbeSets + s) * 16u + 2u * i;
            a[s][i] = (__bf16)(random ? probe_value(id) : a0 + i);
            b[s][i] = (__bf16)(random ? probe_value(id + 1u) : a0 - i);
        }
    for (int it = 0; it < iters; ++it)
#pragma unroll
        for (int u = 0; u < kProbeUnroll; ++u)
#pragma unroll
            for (int i = 0; i < kProbeAcc; ++i)
                acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(i + u) % kProbeSets], b[(i + 3 * u + 1) % kProbeSets], acc[i], 0, 0, 0);
    float s = 0;
    for (int i = 0; i < kProbeAcc; ++i)
        for (int v = 0; v < 16; ++v) s += acc[i][v];
    sink(s);
}

__global__ __launch_bounds__(256) void mfma_rate_f64(int iters, double a0, int random) {
    f64x4 acc[kProbeAcc];
    for (int i = 0; i < kProbeAcc; ++i)
        for (int v = 0; v < 4; ++v) acc[i][v] = 0.0;
    double a[kProbeSets], b[kProbeSets];
    for (int s = 0; s < kProbeSets; ++s) {
        const uint32_t id = (blockIdx.x * 256u + threadIdx.x) * 4u * kProbeSets + 4u * s;
        // (two hashed words per value: all 52 bits of the significand vary)
        a[s] = random ? (double)probe_value(id) + (double)probe_value(id + 1u) * 0x1p-24 : a0 + threadIdx.x * 1e-12;
        b[s] = random ? (double)probe_value(id + 2u) + (double)probe_value(id + 3u) * 0x1p-24 : a0 * 2.0;
    }
    for (int it = 0; it < iters; ++it)
#pragma unroll
        for (int u = 0; u < kProbeUnroll; ++u)
#pragma unroll
            for (int i = 0; i < kProbeAcc; ++i)
                acc[i] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[(i + u) % kProbeSets], b[(i + 3 * u + 1) % kProbeSets], acc[i], 0, 0, 0);
    double s = 0;
    for (int i = 0; i < kProbeAcc; ++i)
        for (int v = 0; v < 4; ++v) s += acc[i][v];
    sink((float)s);
}

}  // namespace igc

using namespace igc;

namespace igc {
int query_compute_units() {
    int dev = 0, n = 0;
    if (hipGetDeviceCount(&n) != hipSuccess || n < 1 || hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) {
        (void)hipGetLastError();
        return 0;
    }
    return n;
}
}  // namespace igc

extern "C" {

igcStatus igcGetDeviceProperties(igcHandle_t handle, int *computeUnits, int *clockKHz) {
    if (!handle || !computeUnits || !clockKHz) return IGC_STATUS_BAD_PARAM;
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) {
        (void)hipGetLastError();
        return IGC_STATUS_EXECUTION_FAILED;
    }
    *computeUnits = prop.multiProcessorCount;
    *clockKHz = prop.clockRate;
    return IGC_STATUS_SUCCESS;
}

igcStatus igcMeasureMatrixRate(igcHandle_t handle, igcDataType dataType, int milliseconds, double *tflops) {
    return igcMeasureMatrixRateOperands(handle, dataType, milliseconds, 0, tflops);
}

igcStatus igcMeasureMatrixRateOperands(igcHandle_t handle, igcDataType dataType, int milliseconds, int randomOperands, double *tflops) {
    if (!handle || !tflops || milliseconds < 1 || milliseconds > 2000 || (randomOperands != 0 && randomOperands != 1)) return IGC_STATUS_BAD_PARAM;
    if (dataType != IGC_DATA_FLOAT && dataType != IGC_DATA_BFLOAT16 && dataType != IGC_DATA_DOUBLE) return IGC_STATUS_BAD_PARAM;
    int cus = 0, khz = 0;
    igcStatus st = igcGetDeviceProperties(handle, &cus, &khz);
    if (st != IGC_STATUS_SUCCESS) return st;
    hipStream_t stream = static_cast<hipStream_t>(handle->stream);
    // flops of one MFMA and the cycles it occupies a SIMD's matrix pipe at the datasheet rate
    const double flops_per_mfma = dataType == IGC_DATA_FLOAT ? 4096.0 : (dataType == IGC_DATA_BFLOAT16 ? 32768.0 : 2048.0);
    const double cycles_per_mfma = dataType == IGC_DATA_FLOAT ? 64.0 : (dataType == IGC_DATA_BFLOAT16 ? 32.0 : 64.0);
    const int grid = cus * 2;   // two workgroups of four wavefronts per compute unit: two waves per SIMD
    // iterations that fill about the requested time at the reported clock (two waves share a SIMD)
    const double per_iter_cycles = 2.0 * kProbeAcc * kProbeUnroll * cycles_per_mfma;
    long long iters = (long long)((double)milliseconds * (double)khz / per_iter_cycles);
    if (iters < 16) iters = 16;
    if (iters > (1 << 24)) iters = 1 << 24;
    auto launch = [&](int n) {
        if (dataType == IGC_DATA_FLOAT) hipLaunchKernelGGL(mfma_rate_f32, dim3(grid), dim3(256), 0, stream, n, 1.f, randomOperands);
        else if (dataType == IGC_DATA_BFLOAT16) hipLaunchKernelGGL(mfma_rate_bf16, dim3(grid), dim3(256), 0, stream, n, 1.f, randomOperands);
        else hipLaunchKernelGGL(mfma_rate_f64, dim3(grid), dim3(256), 0, stream, n, 1.0, randomOperands);
    };
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) {
        if (e0) (void)hipEventDestroy(e0);
        return IGC_STATUS_EXECUTION_FAILED;
    }
    bool ok = true;
    launch((int)(iters / 4 + 1));   // warm-up: clocks and code
    ok = ok && hipEventRecord(e0, stream) == hipSuccess;
    launch((int)iters);
    ok = ok && hipGetLastError() == hipSuccess;
    ok = ok && hipEventRecord(e1, stream) == hipSuccess;
    ok = ok && hipEventSynchronize(e1) == hipSuccess;
    float ms = 0.f;
    ok = ok && hipEventElapsedTime(&ms, e0, e1) == hipSuccess && ms > 0.f;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (!ok) return IGC_STATUS_EXECUTION_FAILED;
    const double total = (double)grid * 4.0 * (double)iters * kProbeUnroll * kProbeAcc * flops_per_mfma;
    *tflops = total / ((double)ms * 1e-3) / 1e12;
    return IGC_STATUS_SUCCESS;
}

}  // extern "C"
