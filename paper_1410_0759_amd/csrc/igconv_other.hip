// The library's other functions (paper, Section 2.2): activations, softmax, pooling and
// tensor addition with broadcasting.  All are bound by HBM bandwidth, so the kernels only
// care about two things: every wavefront reads and writes consecutive addresses, and no
// tensor is read twice from memory when once suffices.
//
// Element-wise functions (activations, addition): the host orders the four dimensions by the
// output's strides, drops those of size 1 and merges neighbours that are contiguous in every
// tensor involved, so that a packed tensor becomes one run of elements and "bias (1,C,1,1)
// onto NCHW" becomes (N*C rows) x (H*W contiguous elements); threads then run along the
// innermost dimension, four elements each (16-byte accesses) when every tensor allows it.
// Softmax per location: one thread per (n,h,w), lanes along the contiguous spatial dimension,
// running maximum and rescaled sum in one pass over the channels, a second pass to write.
// Softmax per image: one workgroup per image, the same two passes with a block reduction.
// Pooling: one thread per output element, ordered by the output's strides.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <cstdio>
#include <cstdlib>
#include <new>

#include "igconv_desc.h"
#include "igconv_params.h"

namespace igc {
namespace {

constexpr long long kMaxBytesOther = 1ll << 31;

__device__ __forceinline__ uint32_t mdiv(uint32_t n, Magic m) { return (__umulhi(n, m.mul) + n) >> m.shift; }

// Up to four dimensions, outermost first, with the element strides of up to four tensors
// (tensor 0 is the output).
constexpr int kMaxTensors = 4;
struct View {
    int rank;
    uint32_t dim[4];
    Magic mdim[4];
    uint32_t stride[kMaxTensors][4];
    int which[4];   // logical dimension (0 n, 1 c, 2 h, 3 w) behind each entry (meaningful when nothing was merged)
};

// Builds the view: dimensions ordered by the output's stride (largest first); with `merge`,
// size-1 dimensions dropped and neighbours merged where every tensor is contiguous across them.
View make_view(const int dim[4], const long long (*stride)[4], int tensors, bool merge) {
    int order[4] = {0, 1, 2, 3};
    std::stable_sort(order, order + 4, [&](int a, int b) { return stride[0][a] > stride[0][b]; });
    View v{};
    for (int i = 0; i < 4; ++i) {
        const int d = order[i];
        if (merge && dim[d] == 1) continue;
        bool fused = false;
        if (merge && v.rank > 0) {
            fused = true;
            for (int t = 0; t < tensors; ++t)
                if ((long long)v.stride[t][v.rank - 1] != stride[t][d] * dim[d]) fused = false;
        }
        if (fused) {
            v.dim[v.rank - 1] *= (uint32_t)dim[d];
            for (int t = 0; t < tensors; ++t) v.stride[t][v.rank - 1] = (uint32_t)stride[t][d];
        } else {
            v.dim[v.rank] = (uint32_t)dim[d];
            v.which[v.rank] = d;
            for (int t = 0; t < tensors; ++t) v.stride[t][v.rank] = (uint32_t)stride[t][d];
            ++v.rank;
        }
    }
    if (v.rank == 0) {   // a single element
        v.rank = 1;
        v.dim[0] = 1;
    }
    for (int i = 0; i < v.rank; ++i) magic_for(v.dim[i], &v.mdim[i]);
    return v;
}

// idx (row-major over the view's dimensions) -> element offset in each of `T` tensors
template <int T>
__device__ __forceinline__ void offsets_of(const View &v, uint32_t idx, uint32_t scale_inner, uint32_t (&off)[T]) {
#pragma unroll
    for (int t = 0; t < T; ++t) off[t] = 0;
    uint32_t rem = idx;
    for (int d = v.rank - 1; d >= 0; --d) {
        uint32_t i;
        if (d == 0) {
            i = rem;
        } else {
            const uint32_t q = mdiv(rem, v.mdim[d]);
            i = rem - q * v.dim[d];
            rem = q;
        }
        if (d == v.rank - 1) i *= scale_inner;
#pragma unroll
        for (int t = 0; t < T; ++t) off[t] += i * v.stride[t][d];
    }
}

// ---- host side ---------------------------------------------------------------------------
template <class Kernel, class Args>
igcStatus launch(Kernel kernel, const char *what, const Args &args, uint32_t blocks, void *stream, size_t lds_bytes = 0) {
    Args copy = args;
    void *argv[] = {&copy};
    const hipError_t e = hipLaunchKernel(reinterpret_cast<const void *>(kernel), dim3(blocks), dim3(256), argv, lds_bytes,
                                         static_cast<hipStream_t>(stream));
    if (e != hipSuccess && std::getenv("IGCONV_DEBUG"))
        std::fprintf(stderr, "igconv: launch of %s failed: %s\n", what, hipGetErrorString(e));
    return e == hipSuccess ? IGC_STATUS_SUCCESS : IGC_STATUS_EXECUTION_FAILED;
}


bool same_dims(igcTensorDescriptor_t a, igcTensorDescriptor_t b) {
    for (int i = 0; i < 4; ++i)
        if (a->dim[i] != b->dim[i]) return false;
    return true;
}


// The scalar-type specific parts: 4-byte-scaled offsets as the kernels form them (element offset * 4, or
// 0x80000000 for "outside"), turned into the type's own byte offsets.
namespace f32 {
typedef float real_t;
typedef float vec4_t __attribute__((ext_vector_type(4)));
constexpr igcDataType kType = IGC_DATA_FLOAT;
__device__ __forceinline__ real_t rload(__amdgpu_buffer_rsrc_t buf, uint32_t off4) {
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(buf, off4, 0, 0));
}
__device__ __forceinline__ void rstore(__amdgpu_buffer_rsrc_t buf, uint32_t off4, real_t v) {
    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, v), buf, off4, 0, 0);
}
// 16 bytes at once (the address need only be a multiple of 4)
constexpr int kWide = 4;
typedef float wide_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ wide_t rload_wide(__amdgpu_buffer_rsrc_t buf, uint32_t off4) {
    typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
    return __builtin_bit_cast(wide_t, (u32x4_t)__builtin_amdgcn_raw_buffer_load_b128(buf, off4, 0, 0));
}
__device__ __forceinline__ real_t rexp(real_t x) { return __expf(x); }
__device__ __forceinline__ real_t rmax(real_t a, real_t b) { return fmaxf(a, b); }
#include "igconv_other_impl.inc"
}  // namespace f32

namespace f64 {
typedef double real_t;
typedef double vec4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
constexpr igcDataType kType = IGC_DATA_DOUBLE;
__device__ __forceinline__ real_t rload(__amdgpu_buffer_rsrc_t buf, uint32_t off4) {
    const u32x2_t v = __builtin_amdgcn_raw_buffer_load_b64(buf, off4 >= 0x80000000u ? 0x80000000u : off4 * 2u, 0, 0);
    return __builtin_bit_cast(double, v);
}
__device__ __forceinline__ void rstore(__amdgpu_buffer_rsrc_t buf, uint32_t off4, real_t v) {
    __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2_t, v), buf, off4 >= 0x80000000u ? 0x80000000u : off4 * 2u, 0, 0);
}
constexpr int kWide = 2;
typedef double wide_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ wide_t rload_wide(__amdgpu_buffer_rsrc_t buf, uint32_t off4) {
    typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
    return __builtin_bit_cast(wide_t, (u32x4_t)__builtin_amdgcn_raw_buffer_load_b128(buf, off4 >= 0x80000000u ? 0x80000000u : off4 * 2u, 0, 0));
}
__device__ __forceinline__ real_t rexp(real_t x) { return exp(x); }
__device__ __forceinline__ real_t rmax(real_t a, real_t b) { return fmax(a, b); }
#include "igconv_other_impl.inc"
}  // namespace f64

bool is_double(igcTensorDescriptor_t d) { return d && d->set && d->dtype == IGC_DATA_DOUBLE; }

}  // namespace
}  // namespace igc

using namespace igc;

extern "C" {

igcStatus igcCreatePoolingDescriptor(igcPoolingDescriptor_t *desc) {
    if (!desc) return IGC_STATUS_BAD_PARAM;
    igcPoolingStruct *p = new (std::nothrow) igcPoolingStruct;
    if (!p) return IGC_STATUS_ALLOC_FAILED;
    *desc = p;
    return IGC_STATUS_SUCCESS;
}

igcStatus igcDestroyPoolingDescriptor(igcPoolingDescriptor_t desc) {
    if (!desc) return IGC_STATUS_BAD_PARAM;
    delete desc;
    return IGC_STATUS_SUCCESS;
}

igcStatus igcSetPooling2dDescriptor(igcPoolingDescriptor_t desc, igcPoolingMode mode, int windowHeight, int windowWidth,
                                    int pad_h, int pad_w, int u, int v) {
    if (!desc) return IGC_STATUS_BAD_PARAM;
    if (mode != IGC_POOLING_MAX && mode != IGC_POOLING_AVERAGE) return IGC_STATUS_BAD_PARAM;
    if (windowHeight < 1 || windowWidth < 1 || u < 1 || v < 1 || pad_h < 0 || pad_w < 0) return IGC_STATUS_BAD_PARAM;
    if (pad_h >= windowHeight || pad_w >= windowWidth) return IGC_STATUS_BAD_PARAM;   // every window must meet the image
    desc->mode = mode;
    desc->win_h = windowHeight; desc->win_w = windowWidth;
    desc->pad_h = pad_h; desc->pad_w = pad_w; desc->u = u; desc->v = v;
    desc->set = true;
    return IGC_STATUS_SUCCESS;
}

igcStatus igcGetPooling2dDescriptor(igcPoolingDescriptor_t desc, igcPoolingMode *mode, int *windowHeight, int *windowWidth,
                                    int *pad_h, int *pad_w, int *u, int *v) {
    if (!desc || !mode || !windowHeight || !windowWidth || !pad_h || !pad_w || !u || !v) return IGC_STATUS_BAD_PARAM;
    if (!desc->set) return IGC_STATUS_NOT_INITIALIZED;
    *mode = desc->mode;
    *windowHeight = desc->win_h; *windowWidth = desc->win_w;
    *pad_h = desc->pad_h; *pad_w = desc->pad_w; *u = desc->u; *v = desc->v;
    return IGC_STATUS_SUCCESS;
}

igcStatus igcGetPooling2dForwardOutputDim(igcPoolingDescriptor_t poolDesc, igcTensorDescriptor_t xDesc, int *n, int *c,
                                          int *p, int *q) {
    if (!poolDesc || !xDesc || !n || !c || !p || !q) return IGC_STATUS_BAD_PARAM;
    if (!poolDesc->set || !xDesc->set) return IGC_STATUS_NOT_INITIALIZED;
    const long long nh = (long long)xDesc->dim[2] + 2 * poolDesc->pad_h - poolDesc->win_h;
    const long long nw = (long long)xDesc->dim[3] + 2 * poolDesc->pad_w - poolDesc->win_w;
    if (nh < 0 || nw < 0) return IGC_STATUS_BAD_PARAM;
    *n = xDesc->dim[0];
    *c = xDesc->dim[1];
    *p = (int)(nh / poolDesc->u + 1);
    *q = (int)(nw / poolDesc->v + 1);
    return IGC_STATUS_SUCCESS;
}

igcStatus igcActivationForward(igcHandle_t handle, igcActivationMode mode, const void *alpha, igcTensorDescriptor_t xDesc,
                               const void *x, const void *beta, igcTensorDescriptor_t yDesc, void *y) {
    return is_double(yDesc) ? f64::ActivationForward(handle, mode, alpha, xDesc, x, beta, yDesc, y) : f32::ActivationForward(handle, mode, alpha, xDesc, x, beta, yDesc, y);
}

igcStatus igcActivationBackward(igcHandle_t handle, igcActivationMode mode, const void *alpha, igcTensorDescriptor_t yDesc,
                                const void *y, igcTensorDescriptor_t dyDesc, const void *dy, igcTensorDescriptor_t xDesc,
                                const void *x, const void *beta, igcTensorDescriptor_t dxDesc, void *dx) {
    return is_double(dxDesc) ? f64::ActivationBackward(handle, mode, alpha, yDesc, y, dyDesc, dy, xDesc, x, beta, dxDesc, dx) : f32::ActivationBackward(handle, mode, alpha, yDesc, y, dyDesc, dy, xDesc, x, beta, dxDesc, dx);
}

igcStatus igcAddTensor(igcHandle_t handle, const void *alpha, igcTensorDescriptor_t bDesc, const void *b, const void *beta,
                       igcTensorDescriptor_t yDesc, void *y) {
    return is_double(yDesc) ? f64::AddTensor(handle, alpha, bDesc, b, beta, yDesc, y) : f32::AddTensor(handle, alpha, bDesc, b, beta, yDesc, y);
}

igcStatus igcSoftmaxForward(igcHandle_t handle, igcSoftmaxMode mode, const void *alpha, igcTensorDescriptor_t xDesc,
                            const void *x, const void *beta, igcTensorDescriptor_t yDesc, void *y) {
    return is_double(yDesc) ? f64::SoftmaxForward(handle, mode, alpha, xDesc, x, beta, yDesc, y) : f32::SoftmaxForward(handle, mode, alpha, xDesc, x, beta, yDesc, y);
}

igcStatus igcPoolingForward(igcHandle_t handle, igcPoolingDescriptor_t poolDesc, const void *alpha, igcTensorDescriptor_t xDesc,
                            const void *x, const void *beta, igcTensorDescriptor_t yDesc, void *y) {
    return is_double(yDesc) ? f64::PoolingForward(handle, poolDesc, alpha, xDesc, x, beta, yDesc, y) : f32::PoolingForward(handle, poolDesc, alpha, xDesc, x, beta, yDesc, y);
}

igcStatus igcSoftmaxBackward(igcHandle_t handle, igcSoftmaxMode mode, const void *alpha, igcTensorDescriptor_t yDesc,
                             const void *y, igcTensorDescriptor_t dyDesc, const void *dy, const void *beta,
                             igcTensorDescriptor_t dxDesc, void *dx) {
    return is_double(dxDesc) ? f64::SoftmaxBackward(handle, mode, alpha, yDesc, y, dyDesc, dy, beta, dxDesc, dx) : f32::SoftmaxBackward(handle, mode, alpha, yDesc, y, dyDesc, dy, beta, dxDesc, dx);
}

igcStatus igcPoolingBackward(igcHandle_t handle, igcPoolingDescriptor_t poolDesc, const void *alpha, igcTensorDescriptor_t dyDesc,
                             const void *dy, igcTensorDescriptor_t xDesc, const void *x, const void *beta,
                             igcTensorDescriptor_t dxDesc, void *dx) {
    return is_double(dxDesc) ? f64::PoolingBackward(handle, poolDesc, alpha, dyDesc, dy, xDesc, x, beta, dxDesc, dx) : f32::PoolingBackward(handle, poolDesc, alpha, dyDesc, dy, xDesc, x, beta, dxDesc, dx);
}

igcStatus igcTransformTensor(igcHandle_t handle, const void *alpha, igcTensorDescriptor_t xDesc, const void *x, const void *beta,
                             igcTensorDescriptor_t yDesc, void *y) {
    return is_double(yDesc) ? f64::TransformTensor(handle, alpha, xDesc, x, beta, yDesc, y) : f32::TransformTensor(handle, alpha, xDesc, x, beta, yDesc, y);
}

}  // extern "C"
