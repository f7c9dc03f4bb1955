// Gradient with respect to the bias of a convolution layer (paper, Section 4: the backward pass computes the gradients
// with respect to the bias, the filter weights and the bottom data):
//
//   db[c] = alpha * sum over n, h, w of dy[n,c,h,w] + beta * db[c]
//
// the transpose of the broadcast addition of a (1,C,1,1) tensor (igcAddTensor).  A reduction bound by reading dy once:
//  * dy with unit channel stride (NHWC-style): a workgroup takes 64 feature maps - the lanes, so a wavefront reads 64
//    consecutive elements of a pixel - and a range of the N*H*W pixels, its four wavefronts on every fourth pixel;
//    (a tensor packed N,H,W,C whose C divides a workgroup's round of 16-byte loads is read as one run of elements, 16
//    bytes per thread and load);
//  * any other layout: a workgroup takes one feature map and a range of the N*(H*W) positions, threads along the
//    flattened (h,w) index (consecutive addresses when w has unit stride).
// Every thread adds in double, whatever dy's type (float, bfloat16 or double): a map of 400 000 pixels would otherwise
// lose the digits the parity bound asks for.  The threads' sums are added through LDS in a fixed order.  With a lent
// workspace the positions are cut into ranges across workgroups, one double per (range, feature map), and a second
// kernel adds the ranges in order; without, one workgroup per (group of) feature map(s) does it all.  Deterministic
// either way; nothing is allocated.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "igconv_desc.h"
#include "igconv_params.h"

namespace igc {
namespace {

constexpr long long kMaxBytesBias = 1ll << 31;
constexpr int kMaxRanges = 1024;

__device__ __forceinline__ uint32_t mdiv(uint32_t n, Magic m) { return (__umulhi(n, m.mul) + n) >> m.shift; }

struct BiasGradArgs {
    const void *dy;
    uint32_t dy_bytes;
    int C, W;
    uint32_t HW, positions;       // H*W, N*H*W
    Magic mHW, mW;
    uint32_t runs;                // 1 when a feature map is one run of H*W elements (w-stride 1, h-stride W)
    uint32_t HWv;                 // H*W in 16-byte vectors (feature maps stored as runs: the vector form below)
    Magic mHWv;
    uint32_t sN, sC, sH, sW;      // element strides of dy
    uint32_t per;                 // positions per range
    int ranges;
    double *parts;                // [range][C] when ranges > 1
    void *db;                     // else the result itself
    uint32_t dbStride;
    double alpha, beta;
};

template <class T> __device__ __forceinline__ double load_as_double(__amdgpu_buffer_rsrc_t buf, uint32_t elem);
template <> __device__ __forceinline__ double load_as_double<float>(__amdgpu_buffer_rsrc_t buf, uint32_t elem) {
    return (double)__builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(buf, elem * 4u, 0, 0));
}
template <> __device__ __forceinline__ double load_as_double<uint16_t>(__amdgpu_buffer_rsrc_t buf, uint32_t elem) {   // bfloat16
    const uint32_t bits = (uint32_t)(uint16_t)__builtin_amdgcn_raw_buffer_load_b16(buf, elem * 2u, 0, 0);
    return (double)__builtin_bit_cast(float, bits << 16);
}
template <> __device__ __forceinline__ double load_as_double<double>(__amdgpu_buffer_rsrc_t buf, uint32_t elem) {
    typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
    return __builtin_bit_cast(double, (u32x2_t)__builtin_amdgcn_raw_buffer_load_b64(buf, elem * 8u, 0, 0));
}

template <class OUT>
__device__ __forceinline__ void finish(const BiasGradArgs &a, int c, int range, double sum) {
    if (a.ranges > 1) {
        a.parts[(size_t)range * a.C + c] = sum;
    } else {
        OUT *dst = static_cast<OUT *>(a.db) + (size_t)c * a.dbStride;
        double r = a.alpha * sum;
        if (a.beta != 0.0) r += a.beta * (double)*dst;
        *dst = (OUT)r;
    }
}

// dy with unit channel stride: lanes along 64 feature maps, the wavefronts on every fourth position of the range
template <class T, class OUT>
__global__ __launch_bounds__(256) void bias_grad_channels_kernel(const BiasGradArgs a) {
    __shared__ double sums[4][64];
    const __amdgpu_buffer_rsrc_t buf = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(a.dy), 0, a.dy_bytes, 0x00020000u);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = (int)blockIdx.x * 64 + lane, range = (int)blockIdx.y;
    const uint32_t begin = (uint32_t)range * a.per, end = begin + a.per < a.positions ? begin + a.per : a.positions;
    double sum = 0.0;
    if (c < a.C)
#pragma unroll 8
        for (uint32_t i = begin + (uint32_t)wave; i < end; i += 4u) {
            const uint32_t n = mdiv(i, a.mHW), rem = i - n * a.HW;
            const uint32_t h = mdiv(rem, a.mW), w = rem - h * (uint32_t)a.W;
            sum += load_as_double<T>(buf, n * a.sN + h * a.sH + w * a.sW + (uint32_t)c);
        }
    sums[wave][lane] = sum;
    __syncthreads();
    if (wave == 0 && c < a.C) finish<OUT>(a, c, range, ((sums[0][lane] + sums[1][lane]) + sums[2][lane]) + sums[3][lane]);
}

// dy packed with the channels innermost (N,H,W,C without gaps), C a whole number of 16-byte vectors, at most 256 of
// them: the tensor is one run of positions * C elements, a thread loads 16 bytes at a time; the first S threads work,
// S the largest multiple of C / V up to 256, and advance by S vectors per round, so a thread meets the same V = 4
// (bfloat16: 8) feature maps every round; the threads that share feature maps are added in thread order at the end.
template <class T> struct Pack;
template <> struct Pack<float> { static constexpr int V = 4; };
template <> struct Pack<uint16_t> { static constexpr int V = 8; };
template <> struct Pack<double> { static constexpr int V = 2; };

template <class T, class OUT>
__global__ __launch_bounds__(256) void bias_grad_packed_kernel(const BiasGradArgs a) {
    constexpr int V = Pack<T>::V;
    typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
    __shared__ double sums[256][V];
    const __amdgpu_buffer_rsrc_t buf = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(a.dy), 0, a.dy_bytes, 0x00020000u);
    const int range = (int)blockIdx.x;
    const uint32_t begin = (uint32_t)range * a.per, end = begin + a.per < a.positions ? begin + a.per : a.positions;
    const uint32_t e_end = end * (uint32_t)a.C;   // (elements; below 2^31 by the size limit)
    double acc[V];
#pragma unroll
    for (int v = 0; v < V; ++v) acc[v] = 0.0;
    // Eight loads requested, then added in their order (left to itself the compiler asked for one load at a time and
    // waited for it); a load past the end of the range has its offset out of range and brings zeros.
    const uint32_t vectors = (uint32_t)a.C / (uint32_t)V, active = (256u / vectors) * vectors;
    const uint32_t STRIDE = active * V;
    for (uint32_t e = threadIdx.x < active ? begin * (uint32_t)a.C + threadIdx.x * (uint32_t)V : e_end; e < e_end; e += 8u * STRIDE) {
        u32x4_t q[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint32_t ei = e + (uint32_t)i * STRIDE;
            q[i] = __builtin_amdgcn_raw_buffer_load_b128(buf, ei < e_end ? ei * (uint32_t)sizeof(T) : 0x80000000u, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            // (the four dwords by name: indexed with the variable of an unrolled loop they were compiled as four copies of the first)
            const uint32_t q0 = q[i].x, q1 = q[i].y, q2 = q[i].z, q3 = q[i].w;
            if constexpr (V == 4) {
                acc[0] += (double)__builtin_bit_cast(float, q0);
                acc[1] += (double)__builtin_bit_cast(float, q1);
                acc[2] += (double)__builtin_bit_cast(float, q2);
                acc[3] += (double)__builtin_bit_cast(float, q3);
            } else if constexpr (V == 8) {
                acc[0] += (double)__builtin_bit_cast(float, q0 << 16);
                acc[1] += (double)__builtin_bit_cast(float, q0 & 0xFFFF0000u);
                acc[2] += (double)__builtin_bit_cast(float, q1 << 16);
                acc[3] += (double)__builtin_bit_cast(float, q1 & 0xFFFF0000u);
                acc[4] += (double)__builtin_bit_cast(float, q2 << 16);
                acc[5] += (double)__builtin_bit_cast(float, q2 & 0xFFFF0000u);
                acc[6] += (double)__builtin_bit_cast(float, q3 << 16);
                acc[7] += (double)__builtin_bit_cast(float, q3 & 0xFFFF0000u);
            } else {
                typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
                acc[0] += __builtin_bit_cast(double, u32x2_t{q0, q1});
                acc[1] += __builtin_bit_cast(double, u32x2_t{q2, q3});
            }
        }
    }
#pragma unroll
    for (int v = 0; v < V; ++v) sums[threadIdx.x][v] = acc[v];
    __syncthreads();
    for (int c = (int)threadIdx.x; c < a.C; c += 256) {
        const int first = c / V, step = a.C / V;   // threads first, first + step, ... hold feature map c at slot c % V
        double sum = 0.0;
        for (int t = first; t < (int)active; t += step) sum += sums[t][c % V];
        finish<OUT>(a, c, range, sum);
    }
}

// any layout: one feature map per workgroup, threads along the flattened (n, h*w) positions of the range
template <class T, class OUT>
__global__ __launch_bounds__(256) void bias_grad_map_kernel(const BiasGradArgs a) {
    __shared__ double sums[256];
    const __amdgpu_buffer_rsrc_t buf = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(a.dy), 0, a.dy_bytes, 0x00020000u);
    const int c = (int)blockIdx.x, range = (int)blockIdx.y;
    const uint32_t begin = (uint32_t)range * a.per, end = begin + a.per < a.positions ? begin + a.per : a.positions;
    double sum = 0.0;
#pragma unroll 8
    for (uint32_t i = begin + threadIdx.x; i < end; i += 256u) {
        const uint32_t n = mdiv(i, a.mHW), rem = i - n * a.HW;
        if (a.runs) {   // (one division per element)
            sum += load_as_double<T>(buf, n * a.sN + (uint32_t)c * a.sC + rem);
        } else {
            const uint32_t h = mdiv(rem, a.mW), w = rem - h * (uint32_t)a.W;
            sum += load_as_double<T>(buf, n * a.sN + (uint32_t)c * a.sC + h * a.sH + w * a.sW);
        }
    }
    sums[threadIdx.x] = sum;
    __syncthreads();
    for (int width = 128; width > 0; width >>= 1) {   // (a fixed tree: the same order every time)
        if ((int)threadIdx.x < width) sums[threadIdx.x] += sums[threadIdx.x + width];
        __syncthreads();
    }
    if (threadIdx.x == 0) finish<OUT>(a, c, range, sums[0]);
}

// feature maps stored as runs (w-stride 1, h-stride W), H*W and the strides of n and c whole 16-byte vectors, dy on a
// 16-byte boundary: as above with a thread on 16 bytes of its feature map at a time - one division per 16 bytes
// instead of two per element, eight loads requested before they are added
template <class T, class OUT>
__global__ __launch_bounds__(256) void bias_grad_map_vectors_kernel(const BiasGradArgs a) {
    constexpr int V = Pack<T>::V;
    typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
    __shared__ double sums[256];
    const __amdgpu_buffer_rsrc_t buf = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(a.dy), 0, a.dy_bytes, 0x00020000u);
    const int c = (int)blockIdx.x, range = (int)blockIdx.y;
    const uint32_t perv = a.per / (uint32_t)V, total = a.positions / (uint32_t)V;   // (the host made `per` a multiple of V)
    const uint32_t begin = (uint32_t)range * perv, end = begin + perv < total ? begin + perv : total;
    const uint32_t cbase = (uint32_t)c * a.sC;
    double sum = 0.0;
    for (uint32_t i0 = begin + threadIdx.x; i0 < end; i0 += 8u * 256u) {
        u32x4_t q[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t i = i0 + (uint32_t)j * 256u;
            const uint32_t n = mdiv(i, a.mHWv), rem = i - n * a.HWv;
            const uint32_t off = (n * a.sN + cbase + rem * (uint32_t)V) * (uint32_t)sizeof(T);
            q[j] = __builtin_amdgcn_raw_buffer_load_b128(buf, i < end ? off : 0x80000000u, 0, 0);   // (past the end: zeros)
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t q0 = q[j].x, q1 = q[j].y, q2 = q[j].z, q3 = q[j].w;   // (by name: see the packed kernel)
            if constexpr (V == 4) {
                sum += (double)__builtin_bit_cast(float, q0);
                sum += (double)__builtin_bit_cast(float, q1);
                sum += (double)__builtin_bit_cast(float, q2);
                sum += (double)__builtin_bit_cast(float, q3);
            } else if constexpr (V == 8) {
                sum += (double)__builtin_bit_cast(float, q0 << 16);
                sum += (double)__builtin_bit_cast(float, q0 & 0xFFFF0000u);
                sum += (double)__builtin_bit_cast(float, q1 << 16);
                sum += (double)__builtin_bit_cast(float, q1 & 0xFFFF0000u);
                sum += (double)__builtin_bit_cast(float, q2 << 16);
                sum += (double)__builtin_bit_cast(float, q2 & 0xFFFF0000u);
                sum += (double)__builtin_bit_cast(float, q3 << 16);
                sum += (double)__builtin_bit_cast(float, q3 & 0xFFFF0000u);
            } else {
                typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
                sum += __builtin_bit_cast(double, u32x2_t{q0, q1});
                sum += __builtin_bit_cast(double, u32x2_t{q2, q3});
            }
        }
    }
    sums[threadIdx.x] = sum;
    __syncthreads();
    for (int width = 128; width > 0; width >>= 1) {   // (a fixed tree: the same order every time)
        if ((int)threadIdx.x < width) sums[threadIdx.x] += sums[threadIdx.x + width];
        __syncthreads();
    }
    if (threadIdx.x == 0) finish<OUT>(a, c, range, sums[0]);
}

// db[c] = alpha * (sum of parts[r][c] over the ranges r) + beta * db[c]: one workgroup of 64 threads per feature map, thread
// t adds the ranges t, t + 64, ... and the 64 sums are added in a fixed tree (one thread walking a thousand ranges would
// wait for a thousand loads one after the other)
template <class OUT>
__global__ __launch_bounds__(64) void bias_grad_sum_kernel(const double *parts, int ranges, int C, OUT *db, uint32_t dbStride, double alpha,
                                                           double beta) {
    __shared__ double sums[64];
    const int c = (int)blockIdx.x;
    double sum = 0.0;
#pragma unroll 4
    for (int r = (int)threadIdx.x; r < ranges; r += 64) sum += parts[(size_t)r * C + c];
    sums[threadIdx.x] = sum;
    __syncthreads();
    for (int width = 32; width > 0; width >>= 1) {
        if ((int)threadIdx.x < width) sums[threadIdx.x] += sums[threadIdx.x + width];
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        OUT *dst = db + (size_t)c * dbStride;
        double v = alpha * sums[0];
        if (beta != 0.0) v += beta * (double)*dst;
        *dst = (OUT)v;
    }
}

struct BiasGradPlan {
    BiasGradArgs a;
    bool packed;     // dy is one run of positions * C elements and the workgroup's round holds whole multiples of C
    bool channels;   // dy has unit channel stride
    bool vectors;    // feature maps are runs of whole 16-byte vectors
    bool f64;
    igcDataType in;
};

igcStatus plan_bias_grad(const igcContext *h, igcTensorDescriptor_t dyDesc, igcTensorDescriptor_t dbDesc, BiasGradPlan *pl) {
    if (!dyDesc || !dbDesc) return IGC_STATUS_BAD_PARAM;
    if (!dyDesc->set || !dbDesc->set) return IGC_STATUS_NOT_INITIALIZED;
    for (int d = 0; d < 4; ++d)
        if (dyDesc->dim[d] < 1 || dyDesc->stride[d] < 0 || dbDesc->stride[d] < 0) return IGC_STATUS_BAD_PARAM;
    if (dbDesc->dim[0] != 1 || dbDesc->dim[1] != dyDesc->dim[1] || dbDesc->dim[2] != 1 || dbDesc->dim[3] != 1) return IGC_STATUS_BAD_PARAM;
    const bool f64 = dyDesc->dtype == IGC_DATA_DOUBLE;
    if (dbDesc->dtype != (f64 ? IGC_DATA_DOUBLE : IGC_DATA_FLOAT)) return IGC_STATUS_NOT_SUPPORTED;
    if (dbDesc->dim[1] > 1 && dbDesc->stride[1] < 1) return IGC_STATUS_BAD_PARAM;   // (feature maps must not share an element)
    const long long dy_bytes = extent(dyDesc->dim, dyDesc->stride) * elem_size(dyDesc->dtype);
    const long long db_bytes = extent(dbDesc->dim, dbDesc->stride) * elem_size(dbDesc->dtype);
    const long long positions = (long long)dyDesc->dim[0] * dyDesc->dim[2] * dyDesc->dim[3];
    if (dy_bytes >= kMaxBytesBias || db_bytes >= kMaxBytesBias || positions >= (1ll << 31)) return IGC_STATUS_NOT_SUPPORTED;
    BiasGradArgs &a = pl->a;
    a = BiasGradArgs{};
    a.dy_bytes = (uint32_t)dy_bytes;
    a.C = dyDesc->dim[1];
    a.W = dyDesc->dim[3];
    a.HW = (uint32_t)(dyDesc->dim[2] * dyDesc->dim[3]);
    a.positions = (uint32_t)positions;
    if (!magic_for(a.HW, &a.mHW) || !magic_for((uint32_t)a.W, &a.mW)) return IGC_STATUS_NOT_SUPPORTED;
    a.sN = (uint32_t)dyDesc->stride[0]; a.sC = (uint32_t)dyDesc->stride[1]; a.sH = (uint32_t)dyDesc->stride[2]; a.sW = (uint32_t)dyDesc->stride[3];
    a.dbStride = (uint32_t)dbDesc->stride[1];
    pl->channels = a.C > 1 && dyDesc->stride[1] == 1;
    const int per16 = 16 / elem_size(dyDesc->dtype);
    pl->packed = pl->channels && a.C % per16 == 0 && a.C / per16 <= 256 && dyDesc->stride[3] == a.C &&
                 dyDesc->stride[2] == (long long)a.W * a.C && dyDesc->stride[0] == (long long)a.HW * a.C;
    a.runs = dyDesc->stride[3] == 1 && dyDesc->stride[2] == a.W ? 1u : 0u;
    pl->vectors = !pl->channels && dyDesc->stride[3] == 1 && dyDesc->stride[2] == a.W && a.HW % per16 == 0 &&
                  dyDesc->stride[0] % per16 == 0 && dyDesc->stride[1] % per16 == 0;
    if (pl->vectors) {
        a.HWv = a.HW / (uint32_t)per16;
        if (!magic_for(a.HWv, &a.mHWv)) return IGC_STATUS_NOT_SUPPORTED;
    }
    pl->f64 = f64;
    pl->in = dyDesc->dtype;
    // ranges: enough workgroups for about eight per compute unit (the loads' latency is covered by workgroups in flight),
    // each with at least 64 KB of dy to read
    const long long groups = pl->packed ? 1 : (pl->channels ? (a.C + 63) / 64 : a.C);
    // (the packed form keeps eight 16-byte loads per thread in flight: one workgroup per compute unit reaches the rate, and
    // the final sum has an eighth of the ranges to add - measured 21.0 -> 18.8 us on 128 x 64 x 56 x 56)
    const long long per_cu = pl->packed ? 1 : 8;
    long long ranges = (per_cu * h->computeUnits + groups - 1) / groups;
    const long long group_bytes = (pl->packed ? a.C : (pl->channels ? 64 : 1)) * (long long)elem_size(dyDesc->dtype);
    ranges = std::min<long long>(ranges, (positions * group_bytes + 65535) / 65536);
    ranges = std::max<long long>(1, std::min<long long>(ranges, kMaxRanges));
    a.ranges = (int)ranges;
    a.per = (uint32_t)((positions + ranges - 1) / ranges);
    if (pl->vectors) a.per = (a.per + (uint32_t)per16 - 1u) / (uint32_t)per16 * (uint32_t)per16;   // (whole vectors per range)
    a.ranges = (int)((positions + a.per - 1) / a.per);
    return IGC_STATUS_SUCCESS;
}

// (the launch calls' own return values, not the thread's last-error state, which other users of the runtime may have set)
template <class T, class OUT>
int launch_bias_grad(const BiasGradPlan &pl, hipStream_t stream) {
    BiasGradArgs a = pl.a;
    void *argv[] = {&a};
    // (the packed form wants dy itself on a 16-byte boundary)
    const bool packed = pl.packed && (uintptr_t)a.dy % 16 == 0;
    const bool vectors = pl.vectors && (uintptr_t)a.dy % 16 == 0;
    const void *kernel = packed ? reinterpret_cast<const void *>(&bias_grad_packed_kernel<T, OUT>)
                                : (pl.channels ? reinterpret_cast<const void *>(&bias_grad_channels_kernel<T, OUT>)
                                               : (vectors ? reinterpret_cast<const void *>(&bias_grad_map_vectors_kernel<T, OUT>)
                                                          : reinterpret_cast<const void *>(&bias_grad_map_kernel<T, OUT>)));
    const dim3 grid = packed ? dim3(a.ranges) : dim3(pl.channels ? (a.C + 63) / 64 : a.C, a.ranges);
    if (hipLaunchKernel(kernel, grid, dim3(256), argv, 0, stream) != hipSuccess) return 1;
    if (a.ranges > 1) {
        const double *parts = a.parts;
        int ranges = a.ranges, C = a.C;
        OUT *db = static_cast<OUT *>(a.db);
        uint32_t stride = a.dbStride;
        double alpha = a.alpha, beta = a.beta;
        void *argv2[] = {&parts, &ranges, &C, &db, &stride, &alpha, &beta};
        if (hipLaunchKernel(reinterpret_cast<const void *>(&bias_grad_sum_kernel<OUT>), dim3(a.C), dim3(64), argv2, 0, stream) !=
            hipSuccess)
            return 1;
    }
    return 0;
}

}  // namespace
}  // namespace igc

using namespace igc;

extern "C" {

igcStatus igcGetConvolutionBackwardBiasWorkspaceSize(igcHandle_t handle, igcTensorDescriptor_t dyDesc, igcTensorDescriptor_t dbDesc,
                                                     size_t *sizeInBytes) {
    if (!handle || !sizeInBytes) return IGC_STATUS_BAD_PARAM;
    BiasGradPlan pl;
    const igcStatus st = plan_bias_grad(handle, dyDesc, dbDesc, &pl);
    if (st != IGC_STATUS_SUCCESS) return st;
    *sizeInBytes = pl.a.ranges > 1 ? (size_t)pl.a.ranges * pl.a.C * sizeof(double) : 0;
    return IGC_STATUS_SUCCESS;
}

igcStatus igcConvolutionBackwardBias(igcHandle_t handle, const void *alpha, igcTensorDescriptor_t dyDesc, const void *dy, void *workSpace,
                                     size_t workSpaceSizeInBytes, const void *beta, igcTensorDescriptor_t dbDesc, void *db) {
    if (!handle || !alpha || !beta || !dy || !db) return IGC_STATUS_BAD_PARAM;
    BiasGradPlan pl;
    const igcStatus st = plan_bias_grad(handle, dyDesc, dbDesc, &pl);
    if (st != IGC_STATUS_SUCCESS) return st;
    if ((uintptr_t)dy % elem_size(dyDesc->dtype) || (uintptr_t)db % elem_size(dbDesc->dtype)) return IGC_STATUS_BAD_PARAM;
    BiasGradArgs &a = pl.a;
    a.dy = dy;
    a.db = db;
    a.alpha = pl.f64 ? *static_cast<const double *>(alpha) : (double)*static_cast<const float *>(alpha);
    a.beta = pl.f64 ? *static_cast<const double *>(beta) : (double)*static_cast<const float *>(beta);
    // without room for the ranges' sums (or with a misaligned one): one range
    const size_t need = (size_t)a.ranges * a.C * sizeof(double);
    if (a.ranges > 1 && (!workSpace || (uintptr_t)workSpace % 8 != 0 || workSpaceSizeInBytes < need)) {
        a.ranges = 1;
        a.per = a.positions;
    }
    a.parts = static_cast<double *>(workSpace);
    hipStream_t stream = static_cast<hipStream_t>(handle->stream);
    int rc;
    if (pl.f64) rc = launch_bias_grad<double, double>(pl, stream);
    else if (pl.in == IGC_DATA_BFLOAT16) rc = launch_bias_grad<uint16_t, float>(pl, stream);
    else rc = launch_bias_grad<float, float>(pl, stream);
    return rc == 0 ? IGC_STATUS_SUCCESS : IGC_STATUS_EXECUTION_FAILED;
}

}  // extern "C"
