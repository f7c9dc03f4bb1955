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

bool magic_of(uint32_t d, Magic *m) {
    if (d < 1u || d >= (1u << 31)) return false;
    uint32_t shift = 0;
    while ((1ull << shift) < d) ++shift;
    const unsigned __int128 one = 1;
    const unsigned __int128 q = ((one << (32 + shift)) + d - 1) / d;
    m->mul = (uint32_t)(q - (one << 32));
    m->shift = shift;
    return true;
}

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
    for (int i = 0; i < v.rank; ++i) magic_of(v.dim[i], &v.mdim[i]);
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

enum EwOp { EW_ACT_FWD = 0, EW_ACT_BWD = 1, EW_ADD = 2 };

struct EwArgs {
    View v;          // tensor 0: output; 1..: inputs
    uint32_t count;  // work items: elements, or groups of four in vector mode
    int op, mode;
    float alpha, beta;
    float *out;
    const float *in[3];
};

__device__ __forceinline__ float act_fwd(int mode, float x) {
    if (mode == IGC_ACTIVATION_SIGMOID) return 1.f / (1.f + __expf(-x));
    if (mode == IGC_ACTIVATION_RELU) return fmaxf(x, 0.f);
    // tanh(x) = 1 - 2 / (exp(2x) + 1): exact limits for large |x|, no cancellation near 0 beyond rounding
    const float e = __expf(2.f * x);
    return 1.f - 2.f / (e + 1.f);
}

__device__ __forceinline__ float ew_value(const EwArgs &a, float i0, float i1, float i2) {
    if (a.op == EW_ACT_FWD) return act_fwd(a.mode, i0);
    if (a.op == EW_ADD) return i0;
    // backward: i0 = y, i1 = dy, i2 = x
    float d;
    if (a.mode == IGC_ACTIVATION_SIGMOID) d = i0 * (1.f - i0);
    else if (a.mode == IGC_ACTIVATION_RELU) d = i2 > 0.f ? 1.f : 0.f;
    else d = 1.f - i0 * i0;
    return i1 * d;
}

// VEC = 4: each thread handles four consecutive elements of the innermost dimension, which every
// tensor either walks with stride 1 (16-byte access) or does not walk at all (stride 0: broadcast).
template <int VEC>
__global__ __launch_bounds__(256) void igconv_elementwise_kernel(const EwArgs a) {
    const uint32_t idx = blockIdx.x * 256u + threadIdx.x;
    if (idx >= a.count) return;
    const int nin = a.op == EW_ACT_BWD ? 3 : 1;
    uint32_t off[4];
    offsets_of<4>(a.v, idx, VEC, off);
    float in[3][VEC];
    for (int t = 0; t < nin; ++t) {
        // (the rectifier's backward pass does not need y, the others do not need x)
        if (a.op == EW_ACT_BWD && ((a.mode == IGC_ACTIVATION_RELU && t == 0) || (a.mode != IGC_ACTIVATION_RELU && t == 2))) {
#pragma unroll
            for (int e = 0; e < VEC; ++e) in[t][e] = 0.f;
            continue;
        }
        const float *src = a.in[t] + off[t + 1];
        if (VEC == 4 && a.v.stride[t + 1][a.v.rank - 1] == 1u) {
            const float4 q = *reinterpret_cast<const float4 *>(src);
            in[t][0] = q.x; in[t][1] = q.y; in[t][2] = q.z; in[t][VEC - 1] = q.w;
        } else {
#pragma unroll
            for (int e = 0; e < VEC; ++e) in[t][e] = src[0];   // VEC == 1, or a broadcast element
        }
    }
    float res[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) res[e] = a.alpha * ew_value(a, in[0][e], in[1][e], in[2][e]);
    float *dst = a.out + off[0];
    if (a.beta != 0.f) {
        if (VEC == 4) {
            const float4 o = *reinterpret_cast<const float4 *>(dst);
            res[0] += a.beta * o.x; res[1] += a.beta * o.y; res[2] += a.beta * o.z; res[VEC - 1] += a.beta * o.w;
        } else {
            res[0] += a.beta * dst[0];
        }
    }
    if (VEC == 4) {
        *reinterpret_cast<float4 *>(dst) = make_float4(res[0], res[1], res[2], res[VEC - 1]);
    } else {
        dst[0] = res[0];
    }
}

// ---- softmax -------------------------------------------------------------------------
struct SoftmaxArgs {
    View v;            // CHANNEL: the (n,h,w) locations (tensor 0: y, tensor 1: x); INSTANCE: (c,h,w) of one image
    uint32_t count;    // locations (CHANNEL) / elements per image (INSTANCE)
    uint32_t C;
    uint32_t ysC, xsC; // CHANNEL: channel strides; INSTANCE: image strides
    float alpha, beta;
    float *y;
    const float *x;
};

// running (max, sum of exp(x - max)) pair, merged with another
__device__ __forceinline__ void sm_merge(float &m, float &s, float m2, float s2) {
    const float mm = fmaxf(m, m2);
    s = (m == mm ? s : s * __expf(m - mm)) + (m2 == mm ? s2 : s2 * __expf(m2 - mm));
    m = mm;
}

__global__ __launch_bounds__(256) void igconv_softmax_channel_kernel(const SoftmaxArgs a) {
    const uint32_t idx = blockIdx.x * 256u + threadIdx.x;
    if (idx >= a.count) return;
    uint32_t off[2];
    offsets_of<2>(a.v, idx, 1u, off);
    const float *x = a.x + off[1];
    float m = -INFINITY, s = 0.f;
    for (uint32_t c = 0; c < a.C; ++c) {
        const float v = x[c * a.xsC];
        if (v > m) {
            s = s * __expf(m - v) + 1.f;   // (exp(-inf) = 0 on the first element)
            m = v;
        } else {
            s += __expf(v - m);
        }
    }
    const float inv = a.alpha / s;
    float *y = a.y + off[0];
    for (uint32_t c = 0; c < a.C; ++c) {
        float r = __expf(x[c * a.xsC] - m) * inv;
        if (a.beta != 0.f) r += a.beta * y[c * a.ysC];
        y[c * a.ysC] = r;
    }
}

__global__ __launch_bounds__(256) void igconv_softmax_instance_kernel(const SoftmaxArgs a) {
    __shared__ float sh_m[4], sh_s[4];
    const float *x = a.x + (size_t)blockIdx.x * a.xsC;
    float *y = a.y + (size_t)blockIdx.x * a.ysC;
    float m = -INFINITY, s = 0.f;
    for (uint32_t i = threadIdx.x; i < a.count; i += 256u) {
        uint32_t off[2];
        offsets_of<2>(a.v, i, 1u, off);
        const float v = x[off[1]];
        if (v > m) {
            s = s * __expf(m - v) + 1.f;
            m = v;
        } else {
            s += __expf(v - m);
        }
    }
    // (a thread that saw no element holds (-inf, 0); merging with it must not produce NaN)
    for (int d = 32; d >= 1; d >>= 1) {
        const float m2 = __shfl_xor(m, d), s2 = __shfl_xor(s, d);
        if (m2 != -INFINITY) {
            if (m == -INFINITY) { m = m2; s = s2; } else sm_merge(m, s, m2, s2);
        }
    }
    if ((threadIdx.x & 63u) == 0u) {
        sh_m[threadIdx.x >> 6] = m;
        sh_s[threadIdx.x >> 6] = s;
    }
    __syncthreads();
    m = sh_m[0];
    s = sh_s[0];
    for (int w = 1; w < 4; ++w)
        if (sh_m[w] != -INFINITY) {
            if (m == -INFINITY) { m = sh_m[w]; s = sh_s[w]; } else sm_merge(m, s, sh_m[w], sh_s[w]);
        }
    const float inv = a.alpha / s;
    for (uint32_t i = threadIdx.x; i < a.count; i += 256u) {
        uint32_t off[2];
        offsets_of<2>(a.v, i, 1u, off);
        float r = __expf(x[off[1]] - m) * inv;
        if (a.beta != 0.f) r += a.beta * y[off[0]];
        y[off[0]] = r;
    }
}

// ---- pooling ---------------------------------------------------------------------------
struct PoolArgs {
    View v;          // output (n,c,p,q) ordered by y's strides, nothing merged; tensor 0: y
    uint32_t count;
    int mode, H, W, win_h, win_w, pad_h, pad_w, u, v_;
    uint32_t xs[4];
    uint32_t x_bytes, y_bytes;   // extents, the limits of the buffer descriptors
    float alpha, beta;
    float *y;
    const float *x;
};

// WH, WW: the window size when it is known at compile time (loops unrolled, loads issued back
// to back), 0 to take it from the arguments.
template <int WH, int WW>
__global__ __launch_bounds__(256) void igconv_pooling_kernel(const PoolArgs a) {
    const uint32_t idx = blockIdx.x * 256u + threadIdx.x;
    if (idx >= a.count) return;
    // idx -> logical (n,c,p,q) and the output offset
    uint32_t coord[4] = {0, 0, 0, 0}, yoff = 0, rem = idx;
    for (int d = a.v.rank - 1; d >= 0; --d) {
        uint32_t i;
        if (d == 0) {
            i = rem;
        } else {
            const uint32_t q = mdiv(rem, a.v.mdim[d]);
            i = rem - q * a.v.dim[d];
            rem = q;
        }
        coord[a.v.which[d]] = i;
        yoff += i * a.v.stride[0][d];
    }
    const int h0 = (int)coord[2] * a.u - a.pad_h, w0 = (int)coord[3] * a.v_ - a.pad_w;
    // Both tensors are accessed through buffer descriptors of their extents: an offset outside
    // a tensor reads as zero / is not written, it cannot touch foreign memory.
    const __amdgpu_buffer_rsrc_t xbuf = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(a.x), 0, a.x_bytes, 0x00020000u);
    const __amdgpu_buffer_rsrc_t ybuf = __builtin_amdgcn_make_buffer_rsrc(a.y, 0, a.y_bytes, 0x00020000u);
    const uint32_t plane = coord[0] * a.xs[0] + coord[1] * a.xs[1];
    // the part of the window that lies inside the image (never empty: pad < window); inside
    // it h0 + r and w0 + c are non-negative
    const int win_h = WH ? WH : a.win_h, win_w = WW ? WW : a.win_w;
    const int r0 = h0 < 0 ? -h0 : 0, r1 = min(win_h, a.H - h0);
    const int c0 = w0 < 0 ? -w0 : 0, c1 = min(win_w, a.W - w0);
    float m = -INFINITY, s = 0.f;
    if constexpr (WH != 0) {
        // every element of the window is requested; those outside [r0,r1) x [c0,c1) with the
        // out-of-range marker as offset, which reads as zero and is then left out
#pragma unroll
        for (int r = 0; r < WH; ++r)
#pragma unroll
            for (int c = 0; c < WW; ++c) {
                const bool in = r >= r0 && r < r1 && c >= c0 && c < c1;
                const uint32_t e = plane + (uint32_t)(h0 + r) * a.xs[2] + (uint32_t)(w0 + c) * a.xs[3];
                const float val = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(xbuf, in ? e * 4u : 0x80000000u, 0, 0));
                m = in ? fmaxf(m, val) : m;
                s += val;
            }
    } else {
        for (int r = r0; r < r1; ++r) {
            const uint32_t row = plane + (uint32_t)(h0 + r) * a.xs[2];
            for (int c = c0; c < c1; ++c) {
                const uint32_t e = row + (uint32_t)(w0 + c) * a.xs[3];
                const float val = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(xbuf, e * 4u, 0, 0));
                m = fmaxf(m, val);
                s += val;
            }
        }
    }
    const int cnt = (r1 - r0) * (c1 - c0);
    float r = a.alpha * (a.mode == IGC_POOLING_MAX ? m : s / (float)cnt);
    if (a.beta != 0.f) r += a.beta * __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(ybuf, yoff * 4u, 0, 0));
    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, r), ybuf, yoff * 4u, 0, 0);
}

// The same function for tensors whose w stride is 1: a workgroup takes TP output rows of one
// (n,c) plane, loads the rows of x their windows touch into LDS with whole-row reads and
// computes its outputs from there: x leaves HBM once, in contiguous runs.
struct PoolRowsArgs {
    int mode, H, W, P, Q, win_h, win_w, pad_h, pad_w, u, v_;
    int TP, strips, C;           // output rows per workgroup, workgroups per plane, planes are (n,c)
    Magic mStrips, mC, mW, mQ;
    uint32_t xs[3], ys[3];       // n, c, h strides
    uint32_t x_bytes, y_bytes;
    float alpha, beta;
    float *y;
    const float *x;
};

template <int WH, int WW>
__global__ __launch_bounds__(256) void igconv_pooling_rows_kernel(const PoolRowsArgs a) {
    extern __shared__ float pool_rows_lds[];
    const uint32_t plane = mdiv(blockIdx.x, a.mStrips), strip = blockIdx.x - plane * (uint32_t)a.strips;
    const uint32_t n = mdiv(plane, a.mC), c = plane - n * (uint32_t)a.C;
    const int p0 = (int)strip * a.TP, p1 = min(p0 + a.TP, a.P);
    const int win_h = WH ? WH : a.win_h, win_w = WW ? WW : a.win_w;
    const int xr0 = max(p0 * a.u - a.pad_h, 0), xr1 = min((p1 - 1) * a.u - a.pad_h + win_h, a.H);
    const __amdgpu_buffer_rsrc_t xbuf = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(a.x), 0, a.x_bytes, 0x00020000u);
    const __amdgpu_buffer_rsrc_t ybuf = __builtin_amdgcn_make_buffer_rsrc(a.y, 0, a.y_bytes, 0x00020000u);
    {
        const uint32_t base = n * a.xs[0] + c * a.xs[1];
        const int cnt = (xr1 - xr0) * a.W;
        for (int i = threadIdx.x; i < cnt; i += 256) {
            const uint32_t r = mdiv((uint32_t)i, a.mW), w = (uint32_t)i - r * (uint32_t)a.W;
            pool_rows_lds[i] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(
                xbuf, (base + ((uint32_t)xr0 + r) * a.xs[2] + w) * 4u, 0, 0));
        }
    }
    __syncthreads();
    const uint32_t base = n * a.ys[0] + c * a.ys[1];
    const int cnt = (p1 - p0) * a.Q;
    for (int i = threadIdx.x; i < cnt; i += 256) {
        const uint32_t pr = mdiv((uint32_t)i, a.mQ), q = (uint32_t)i - pr * (uint32_t)a.Q;
        const int p = p0 + (int)pr;
        const int h0 = p * a.u - a.pad_h, w0 = (int)q * a.v_ - a.pad_w;
        // the part of the window inside the image (never empty: pad < window)
        const int r0 = max(h0, 0), r1 = min(h0 + win_h, a.H), c0 = max(w0, 0), c1 = min(w0 + win_w, a.W);
        float m = -INFINITY, s = 0.f;
        if (WH != 0 && r1 - r0 == WH && c1 - c0 == WW) {     // whole window inside: fixed trip counts
            const float *src = pool_rows_lds + (r0 - xr0) * a.W + c0;
#pragma unroll
            for (int r = 0; r < (WH ? WH : 1); ++r)
#pragma unroll
                for (int cc = 0; cc < (WW ? WW : 1); ++cc) {
                    const float val = src[r * a.W + cc];
                    m = fmaxf(m, val);
                    s += val;
                }
        } else {
            for (int r = r0; r < r1; ++r)
                for (int cc = c0; cc < c1; ++cc) {
                    const float val = pool_rows_lds[(r - xr0) * a.W + cc];
                    m = fmaxf(m, val);
                    s += val;
                }
        }
        float res = a.alpha * (a.mode == IGC_POOLING_MAX ? m : s / (float)((r1 - r0) * (c1 - c0)));
        const uint32_t off = (base + (uint32_t)p * a.ys[2] + q) * 4u;
        if (a.beta != 0.f) res += a.beta * __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(ybuf, off, 0, 0));
        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, res), ybuf, off, 0, 0);
    }
}

// ---- softmax backward --------------------------------------------------------------------
// dx_i = y_i * (dy_i - sum_j dy_j y_j), j over the group (Jacobian of the softmax applied
// to dy).  Same decomposition as forward: two passes, the first for the dot product.
struct SoftmaxBwdArgs {
    View v;            // tensor 0: y (ordering key), 1: dx, 2: dy
    uint32_t count, C;
    uint32_t sC[3];    // CHANNEL: channel strides of y, dx, dy; INSTANCE: image strides
    float alpha, beta;
    const float *y, *dy;
    float *dx;
};

__global__ __launch_bounds__(256) void igconv_softmax_bwd_channel_kernel(const SoftmaxBwdArgs a) {
    const uint32_t idx = blockIdx.x * 256u + threadIdx.x;
    if (idx >= a.count) return;
    uint32_t off[3];
    offsets_of<3>(a.v, idx, 1u, off);
    const float *y = a.y + off[0], *dy = a.dy + off[2];
    float *dx = a.dx + off[1];
    float dot = 0.f;
    for (uint32_t c = 0; c < a.C; ++c) dot += dy[c * a.sC[2]] * y[c * a.sC[0]];
    for (uint32_t c = 0; c < a.C; ++c) {
        float r = a.alpha * (y[c * a.sC[0]] * (dy[c * a.sC[2]] - dot));
        if (a.beta != 0.f) r += a.beta * dx[c * a.sC[1]];
        dx[c * a.sC[1]] = r;
    }
}

__global__ __launch_bounds__(256) void igconv_softmax_bwd_instance_kernel(const SoftmaxBwdArgs a) {
    __shared__ float sh[4];
    const float *y = a.y + (size_t)blockIdx.x * a.sC[0], *dy = a.dy + (size_t)blockIdx.x * a.sC[2];
    float *dx = a.dx + (size_t)blockIdx.x * a.sC[1];
    float dot = 0.f;
    for (uint32_t i = threadIdx.x; i < a.count; i += 256u) {
        uint32_t off[3];
        offsets_of<3>(a.v, i, 1u, off);
        dot += dy[off[2]] * y[off[0]];
    }
    for (int d = 32; d >= 1; d >>= 1) dot += __shfl_xor(dot, d);
    if ((threadIdx.x & 63u) == 0u) sh[threadIdx.x >> 6] = dot;
    __syncthreads();
    dot = (sh[0] + sh[1]) + (sh[2] + sh[3]);
    for (uint32_t i = threadIdx.x; i < a.count; i += 256u) {
        uint32_t off[3];
        offsets_of<3>(a.v, i, 1u, off);
        float r = a.alpha * (y[off[0]] * (dy[off[2]] - dot));
        if (a.beta != 0.f) r += a.beta * dx[off[1]];
        dx[off[1]] = r;
    }
}

// ---- pooling backward ---------------------------------------------------------------------
// One thread per input element (n,c,h,w), ordered by dx's strides; it visits the windows that
// cover it (at most ceil(win/stride) per axis) in order and sums their contributions, so the
// result does not depend on scheduling.  AVERAGE: dy / (in-image elements of the window).
// MAX: dy when this element is the window's maximum and no element before it in scan order
// (rows, then columns) equals it.
struct PoolBwdArgs {
    View v;          // input (n,c,h,w) ordered by dx's strides, nothing merged; tensor 0: dx
    uint32_t count;
    int mode, H, W, P, Q, win_h, win_w, pad_h, pad_w, u, v_;
    uint32_t xs[4], dys[4];
    uint32_t x_bytes, dy_bytes, dx_bytes;
    float alpha, beta;
    float *dx;
    const float *x, *dy;
};

__global__ __launch_bounds__(256) void igconv_pooling_bwd_kernel(const PoolBwdArgs a) {
    const uint32_t idx = blockIdx.x * 256u + threadIdx.x;
    if (idx >= a.count) return;
    uint32_t coord[4] = {0, 0, 0, 0}, dxoff = 0, rem = idx;
    for (int d = a.v.rank - 1; d >= 0; --d) {
        uint32_t i;
        if (d == 0) {
            i = rem;
        } else {
            const uint32_t q = mdiv(rem, a.v.mdim[d]);
            i = rem - q * a.v.dim[d];
            rem = q;
        }
        coord[a.v.which[d]] = i;
        dxoff += i * a.v.stride[0][d];
    }
    const __amdgpu_buffer_rsrc_t xbuf = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(a.x), 0, a.x_bytes, 0x00020000u);
    const __amdgpu_buffer_rsrc_t dybuf = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(a.dy), 0, a.dy_bytes, 0x00020000u);
    const __amdgpu_buffer_rsrc_t dxbuf = __builtin_amdgcn_make_buffer_rsrc(a.dx, 0, a.dx_bytes, 0x00020000u);
    const int h = (int)coord[2], w = (int)coord[3];
    // windows p with p*u - pad <= h <= p*u - pad + win - 1, inside [0, P)
    const int th = h + a.pad_h - (a.win_h - 1), tw = w + a.pad_w - (a.win_w - 1);
    const int p_lo = th <= 0 ? 0 : (th + a.u - 1) / a.u, p_hi = min(a.P - 1, (h + a.pad_h) / a.u);
    const int q_lo = tw <= 0 ? 0 : (tw + a.v_ - 1) / a.v_, q_hi = min(a.Q - 1, (w + a.pad_w) / a.v_);
    const uint32_t xplane = coord[0] * a.xs[0] + coord[1] * a.xs[1];
    const uint32_t dyplane = coord[0] * a.dys[0] + coord[1] * a.dys[1];
    float own = 0.f;
    if (a.mode == IGC_POOLING_MAX)
        own = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(
                  xbuf, (xplane + (uint32_t)h * a.xs[2] + (uint32_t)w * a.xs[3]) * 4u, 0, 0));
    float acc = 0.f;
    for (int p = p_lo; p <= p_hi; ++p) {
        // the in-image rows [r0, r1) and columns [c0, c1) of the window, as image coordinates
        const int r0 = max(p * a.u - a.pad_h, 0), r1 = min(p * a.u - a.pad_h + a.win_h, a.H);
        for (int q = q_lo; q <= q_hi; ++q) {
            const int c0 = max(q * a.v_ - a.pad_w, 0), c1 = min(q * a.v_ - a.pad_w + a.win_w, a.W);
            const float g = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(
                dybuf, (dyplane + (uint32_t)p * a.dys[2] + (uint32_t)q * a.dys[3]) * 4u, 0, 0));
            if (a.mode == IGC_POOLING_MAX) {
                bool mine = true;
                for (int r = r0; r < r1; ++r) {
                    const uint32_t row = xplane + (uint32_t)r * a.xs[2];
                    for (int c = c0; c < c1; ++c) {
                        const float val = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(
                            xbuf, (row + (uint32_t)c * a.xs[3]) * 4u, 0, 0));
                        const bool before = r < h || (r == h && c < w);
                        if (before ? val >= own : val > own) mine = false;
                    }
                }
                if (mine) acc += g;
            } else {
                acc += g / (float)((r1 - r0) * (c1 - c0));
            }
        }
    }
    float r = a.alpha * acc;
    if (a.beta != 0.f) r += a.beta * __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(dxbuf, dxoff * 4u, 0, 0));
    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, r), dxbuf, dxoff * 4u, 0, 0);
}

// The same function for tensors whose w stride is 1 (x, dy and dx): a workgroup takes TH input
// rows of one (n,c) plane.  It loads the rows of x its windows touch into LDS with coalesced
// reads (MAX only), finds each covering window's share once - the position of its maximum and
// dy, or dy / count - into LDS, and then every input element of the strip sums the shares of
// the windows covering it, in window order.  HBM sees x, dy and dx once, in whole rows.
struct PoolBwdRowsArgs {
    int mode, H, W, P, Q, win_h, win_w, pad_h, pad_w, u, v_;
    int TH, strips, C;          // input rows per workgroup, workgroups per plane, planes are (n,c)
    Magic mStrips, mC, mu, mv, mW, mQ;
    uint32_t xs[3], dys[3], dxs[3];   // n, c, h strides
    uint32_t x_bytes, dy_bytes, dx_bytes;
    int xrows_max, wrows_max;   // LDS room: rows of x, rows of windows
    int wpi, rpi;               // rows of windows / of the image the 256 threads cover at a time with one column each (0: rows too wide)
    float alpha, beta;
    float *dx;
    const float *x, *dy;
};

__global__ __launch_bounds__(256) void igconv_pooling_bwd_rows_kernel(const PoolBwdRowsArgs a) {
    extern __shared__ float pool_lds[];
    float *xl = pool_lds;                                  // [xrows_max][W]
    float *gl = pool_lds + a.xrows_max * a.W;              // [wrows_max][Q] share of dy
    int *al = reinterpret_cast<int *>(gl + a.wrows_max * a.Q);   // [wrows_max][Q] position h*W + w of the maximum
    const uint32_t plane = mdiv(blockIdx.x, a.mStrips), strip = blockIdx.x - plane * (uint32_t)a.strips;
    const uint32_t n = mdiv(plane, a.mC), c = plane - n * (uint32_t)a.C;
    const int h0 = (int)strip * a.TH, h1 = min(h0 + a.TH, a.H);
    const int t0 = h0 + a.pad_h - (a.win_h - 1);
    const int p_lo = t0 <= 0 ? 0 : (int)mdiv((uint32_t)(t0 + a.u - 1), a.mu);
    const int p_hi = min(a.P - 1, (int)mdiv((uint32_t)(h1 - 1 + a.pad_h), a.mu));
    const int nprow = max(p_hi - p_lo + 1, 0);
    const int xr0 = max(p_lo * a.u - a.pad_h, 0), xr1 = min(p_hi * a.u - a.pad_h + a.win_h, a.H);
    const __amdgpu_buffer_rsrc_t xbuf = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(a.x), 0, a.x_bytes, 0x00020000u);
    const __amdgpu_buffer_rsrc_t dybuf = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(a.dy), 0, a.dy_bytes, 0x00020000u);
    const __amdgpu_buffer_rsrc_t dxbuf = __builtin_amdgcn_make_buffer_rsrc(a.dx, 0, a.dx_bytes, 0x00020000u);
    const bool is_max = a.mode == IGC_POOLING_MAX;
    if (is_max && nprow > 0) {
        const uint32_t base = n * a.xs[0] + c * a.xs[1];
        const int cnt = (xr1 - xr0) * a.W;
        for (int i = threadIdx.x; i < cnt; i += 256) {
            const uint32_t r = mdiv((uint32_t)i, a.mW), w = (uint32_t)i - r * (uint32_t)a.W;
            xl[i] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(
                xbuf, (base + ((uint32_t)xr0 + r) * a.xs[2] + w) * 4u, 0, 0));
        }
    }
    __syncthreads();
    {
        const uint32_t base = n * a.dys[0] + c * a.dys[1];
        // the share of window (p_lo + pr, q), whose in-image columns are [c0, c1)
        auto window = [&](int pr, int q, int c0, int c1) {
            const int p = p_lo + pr, wi = pr * a.Q + q;
            const int r0 = max(p * a.u - a.pad_h, 0), r1 = min(p * a.u - a.pad_h + a.win_h, a.H);
            const float g = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(
                dybuf, (base + (uint32_t)p * a.dys[2] + (uint32_t)q) * 4u, 0, 0));
            if (is_max) {
                float m = -INFINITY;
                int arg = r0 * a.W + c0;
                for (int r = r0; r < r1; ++r)
                    for (int cc = c0; cc < c1; ++cc) {
                        const float val = xl[(r - xr0) * a.W + cc];
                        if (val > m) {     // strictly greater: the first of equal maxima stays
                            m = val;
                            arg = r * a.W + cc;
                        }
                    }
                al[wi] = arg;
                gl[wi] = g;
            } else {
                gl[wi] = g / (float)((r1 - r0) * (c1 - c0));
            }
        };
        if (a.wpi) {
            // a thread keeps its column and walks down the window rows: the column's arithmetic is done once
            const int slot = (int)mdiv(threadIdx.x, a.mQ), q = (int)threadIdx.x - slot * a.Q;
            const int c0 = max(q * a.v_ - a.pad_w, 0), c1 = min(q * a.v_ - a.pad_w + a.win_w, a.W);
            if (slot < a.wpi)
                for (int pr = slot; pr < nprow; pr += a.wpi) window(pr, q, c0, c1);
        } else {   // rows wider than the workgroup: element by element
            const int cnt = nprow * a.Q;
            for (int wi = threadIdx.x; wi < cnt; wi += 256) {
                const int pr = (int)mdiv((uint32_t)wi, a.mQ), q = wi - pr * a.Q;
                window(pr, q, max(q * a.v_ - a.pad_w, 0), min(q * a.v_ - a.pad_w + a.win_w, a.W));
            }
        }
    }
    __syncthreads();
    const uint32_t base = n * a.dxs[0] + c * a.dxs[1];
    // input element (h0 + r, w), covered by the window columns [ql, qh]
    auto element = [&](int r, int w, int ql, int qh) {
        const int h = h0 + r;
        const int th = h + a.pad_h - (a.win_h - 1);
        const int pl = th <= 0 ? 0 : (int)mdiv((uint32_t)(th + a.u - 1), a.mu), ph = min(a.P - 1, (int)mdiv((uint32_t)(h + a.pad_h), a.mu));
        const int self = h * a.W + w;
        float acc = 0.f;
        for (int p = pl; p <= ph; ++p)
            for (int q = ql; q <= qh; ++q) {
                const int wi = (p - p_lo) * a.Q + q;
                if (!is_max || al[wi] == self) acc += gl[wi];
            }
        const uint32_t off = (base + (uint32_t)h * a.dxs[2] + (uint32_t)w) * 4u;
        float res = a.alpha * acc;
        if (a.beta != 0.f) res += a.beta * __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(dxbuf, off, 0, 0));
        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, res), dxbuf, off, 0, 0);
    };
    auto q_range = [&](int w, int &ql, int &qh) {
        const int tw = w + a.pad_w - (a.win_w - 1);
        ql = tw <= 0 ? 0 : (int)mdiv((uint32_t)(tw + a.v_ - 1), a.mv);
        qh = min(a.Q - 1, (int)mdiv((uint32_t)(w + a.pad_w), a.mv));
    };
    if (a.rpi) {
        const int slot = (int)mdiv(threadIdx.x, a.mW), w = (int)threadIdx.x - slot * a.W;
        int ql, qh;
        q_range(w, ql, qh);
        if (slot < a.rpi)
            for (int r = slot; r < h1 - h0; r += a.rpi) element(r, w, ql, qh);
    } else {
        const int cnt = (h1 - h0) * a.W;
        for (int i = threadIdx.x; i < cnt; i += 256) {
            const int r = (int)mdiv((uint32_t)i, a.mW), w = i - r * a.W;
            int ql, qh;
            q_range(w, ql, qh);
            element(r, w, ql, qh);
        }
    }
}

// ---- tensor transformation (change of layout) ----------------------------------------------
// y = alpha * x + beta * y where x is contiguous along one dimension (A) and y along another (B):
// a workgroup moves a 64 x 64 tile of the (A, B) plane through LDS, reading runs along A and
// writing runs along B, so that both tensors see contiguous accesses.  The (at most two)
// remaining dimensions are enumerated by the block index.
struct TransposeArgs {
    uint32_t dimA, dimB, tilesA, tilesB, outer1;   // outer index = o0 * outer1 + o1
    Magic mTilesA, mTilesB, mOuter1;
    uint32_t xsB, ysA;                              // (x's stride along A and y's along B are 1)
    uint32_t xsO[2], ysO[2];
    uint32_t x_bytes, y_bytes;
    float alpha, beta;
    float *y;
    const float *x;
};

__global__ __launch_bounds__(256) void igconv_transpose_kernel(const TransposeArgs a) {
    __shared__ float tile[64][65];
    uint32_t rem = blockIdx.x;
    const uint32_t q1 = mdiv(rem, a.mTilesA), ta = rem - q1 * a.tilesA;
    const uint32_t q2 = mdiv(q1, a.mTilesB), tb = q1 - q2 * a.tilesB;
    const uint32_t o0 = mdiv(q2, a.mOuter1), o1 = q2 - o0 * a.outer1;
    const uint32_t a0 = ta * 64u, b0 = tb * 64u;
    const __amdgpu_buffer_rsrc_t xbuf = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(a.x), 0, a.x_bytes, 0x00020000u);
    const __amdgpu_buffer_rsrc_t ybuf = __builtin_amdgcn_make_buffer_rsrc(a.y, 0, a.y_bytes, 0x00020000u);
    const uint32_t xbase = o0 * a.xsO[0] + o1 * a.xsO[1], ybase = o0 * a.ysO[0] + o1 * a.ysO[1];
    const uint32_t lane = threadIdx.x & 63u, grp = threadIdx.x >> 6;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const uint32_t bl = (uint32_t)r * 4u + grp, ia = a0 + lane, ib = b0 + bl;
        const bool ok = ia < a.dimA && ib < a.dimB;
        tile[bl][lane] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(
            xbuf, ok ? (xbase + ia + ib * a.xsB) * 4u : 0x80000000u, 0, 0));
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const uint32_t al = (uint32_t)r * 4u + grp, ia = a0 + al, ib = b0 + lane;
        if (ia < a.dimA && ib < a.dimB) {
            const uint32_t off = (ybase + ia * a.ysA + ib) * 4u;
            float res = a.alpha * tile[lane][al];
            if (a.beta != 0.f) res += a.beta * __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(ybuf, off, 0, 0));
            __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, res), ybuf, off, 0, 0);
        }
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

igcStatus check_float_tensor(igcTensorDescriptor_t d, bool output) {
    if (!d) return IGC_STATUS_BAD_PARAM;
    if (!d->set) return IGC_STATUS_NOT_INITIALIZED;
    if (d->dtype != IGC_DATA_FLOAT) return IGC_STATUS_NOT_SUPPORTED;
    if (extent(d->dim, d->stride) * 4 >= kMaxBytesOther) return IGC_STATUS_NOT_SUPPORTED;
    if (output && !non_aliasing(d->dim, d->stride)) return IGC_STATUS_BAD_PARAM;
    return IGC_STATUS_SUCCESS;
}

bool same_dims(igcTensorDescriptor_t a, igcTensorDescriptor_t b) {
    for (int i = 0; i < 4; ++i)
        if (a->dim[i] != b->dim[i]) return false;
    return true;
}

// Element-wise launch: output `y` and `nin` inputs with (possibly broadcast) strides.
igcStatus run_elementwise(igcHandle_t h, int op, int mode, float alpha, float beta, igcTensorDescriptor_t yd, void *y,
                          int nin, const long long (*in_stride)[4], const void *const *in) {
    long long stride[kMaxTensors][4] = {};
    for (int d = 0; d < 4; ++d) stride[0][d] = yd->stride[d];
    for (int t = 0; t < nin; ++t)
        for (int d = 0; d < 4; ++d) stride[t + 1][d] = in_stride[t][d];
    EwArgs a{};
    a.v = make_view(yd->dim, stride, nin + 1, /*merge=*/true);
    const uint32_t inner = a.v.dim[a.v.rank - 1];
    uint32_t total = 1;
    for (int i = 0; i < a.v.rank; ++i) total *= a.v.dim[i];
    // four elements per thread when the innermost run allows 16-byte accesses in every tensor
    bool vec = inner % 4 == 0 && (uintptr_t)y % 16 == 0 && a.v.stride[0][a.v.rank - 1] == 1;
    for (int t = 0; t <= nin && vec; ++t) {
        const uint32_t si = a.v.stride[t][a.v.rank - 1];
        if (si > 1) vec = false;
        if (t > 0 && si == 1 && (uintptr_t)in[t - 1] % 16 != 0) vec = false;
        for (int d = 0; d + 1 < a.v.rank; ++d)
            if (si == 1 && a.v.stride[t][d] % 4 != 0) vec = false;
    }
    a.op = op; a.mode = mode; a.alpha = alpha; a.beta = beta;
    a.out = static_cast<float *>(y);
    for (int t = 0; t < nin; ++t) a.in[t] = static_cast<const float *>(in[t]);
    if (vec) {
        a.v.dim[a.v.rank - 1] = inner / 4;
        magic_of(a.v.dim[a.v.rank - 1], &a.v.mdim[a.v.rank - 1]);
        a.count = total / 4;
        return launch(&igconv_elementwise_kernel<4>, "igconv_elementwise_kernel", a, (a.count + 255u) / 256u, h->stream);
    }
    a.count = total;
    return launch(&igconv_elementwise_kernel<1>, "igconv_elementwise_kernel", a, (a.count + 255u) / 256u, h->stream);
}

}  // namespace
}  // namespace igc

using namespace igc;

extern "C" {

igcStatus igcActivationForward(igcHandle_t handle, igcActivationMode mode, const void *alpha, igcTensorDescriptor_t xDesc,
                               const void *x, const void *beta, igcTensorDescriptor_t yDesc, void *y) {
    if (!handle || !alpha || !beta || !x || !y) return IGC_STATUS_BAD_PARAM;
    if (mode != IGC_ACTIVATION_SIGMOID && mode != IGC_ACTIVATION_RELU && mode != IGC_ACTIVATION_TANH) return IGC_STATUS_BAD_PARAM;
    igcStatus st = check_float_tensor(xDesc, false);
    if (st == IGC_STATUS_SUCCESS) st = check_float_tensor(yDesc, true);
    if (st != IGC_STATUS_SUCCESS) return st;
    if (!same_dims(xDesc, yDesc) || (uintptr_t)x % 4 || (uintptr_t)y % 4) return IGC_STATUS_BAD_PARAM;
    const void *in[1] = {x};
    return run_elementwise(handle, EW_ACT_FWD, mode, *static_cast<const float *>(alpha), *static_cast<const float *>(beta),
                           yDesc, y, 1, &xDesc->stride, in);
}

igcStatus igcActivationBackward(igcHandle_t handle, igcActivationMode mode, const void *alpha, igcTensorDescriptor_t yDesc,
                                const void *y, igcTensorDescriptor_t dyDesc, const void *dy, igcTensorDescriptor_t xDesc,
                                const void *x, const void *beta, igcTensorDescriptor_t dxDesc, void *dx) {
    if (!handle || !alpha || !beta || !y || !dy || !x || !dx) return IGC_STATUS_BAD_PARAM;
    if (mode != IGC_ACTIVATION_SIGMOID && mode != IGC_ACTIVATION_RELU && mode != IGC_ACTIVATION_TANH) return IGC_STATUS_BAD_PARAM;
    igcTensorDescriptor_t ins[3] = {yDesc, dyDesc, xDesc};
    for (igcTensorDescriptor_t d : ins) {
        const igcStatus st = check_float_tensor(d, false);
        if (st != IGC_STATUS_SUCCESS) return st;
    }
    const igcStatus st = check_float_tensor(dxDesc, true);
    if (st != IGC_STATUS_SUCCESS) return st;
    for (igcTensorDescriptor_t d : ins)
        if (!same_dims(d, dxDesc)) return IGC_STATUS_BAD_PARAM;
    if ((uintptr_t)y % 4 || (uintptr_t)dy % 4 || (uintptr_t)x % 4 || (uintptr_t)dx % 4) return IGC_STATUS_BAD_PARAM;
    long long strides[3][4];
    for (int t = 0; t < 3; ++t)
        for (int d = 0; d < 4; ++d) strides[t][d] = ins[t]->stride[d];
    const void *in[3] = {y, dy, x};
    return run_elementwise(handle, EW_ACT_BWD, mode, *static_cast<const float *>(alpha), *static_cast<const float *>(beta),
                           dxDesc, dx, 3, strides, in);
}

igcStatus igcAddTensor(igcHandle_t handle, const void *alpha, igcTensorDescriptor_t bDesc, const void *b, const void *beta,
                       igcTensorDescriptor_t yDesc, void *y) {
    if (!handle || !alpha || !beta || !b || !y) return IGC_STATUS_BAD_PARAM;
    igcStatus st = check_float_tensor(bDesc, false);
    if (st == IGC_STATUS_SUCCESS) st = check_float_tensor(yDesc, true);
    if (st != IGC_STATUS_SUCCESS) return st;
    long long bs[1][4];
    for (int d = 0; d < 4; ++d) {
        if (bDesc->dim[d] != 1 && bDesc->dim[d] != yDesc->dim[d]) return IGC_STATUS_BAD_PARAM;
        bs[0][d] = bDesc->dim[d] == 1 ? 0 : bDesc->stride[d];   // a broadcast dimension is not walked
    }
    if ((uintptr_t)b % 4 || (uintptr_t)y % 4) return IGC_STATUS_BAD_PARAM;
    const void *in[1] = {b};
    return run_elementwise(handle, EW_ADD, 0, *static_cast<const float *>(alpha), *static_cast<const float *>(beta), yDesc, y,
                           1, bs, in);
}

igcStatus igcSoftmaxForward(igcHandle_t handle, igcSoftmaxMode mode, const void *alpha, igcTensorDescriptor_t xDesc,
                            const void *x, const void *beta, igcTensorDescriptor_t yDesc, void *y) {
    if (!handle || !alpha || !beta || !x || !y) return IGC_STATUS_BAD_PARAM;
    if (mode != IGC_SOFTMAX_MODE_INSTANCE && mode != IGC_SOFTMAX_MODE_CHANNEL) return IGC_STATUS_BAD_PARAM;
    igcStatus st = check_float_tensor(xDesc, false);
    if (st == IGC_STATUS_SUCCESS) st = check_float_tensor(yDesc, true);
    if (st != IGC_STATUS_SUCCESS) return st;
    if (!same_dims(xDesc, yDesc) || (uintptr_t)x % 4 || (uintptr_t)y % 4) return IGC_STATUS_BAD_PARAM;
    SoftmaxArgs a{};
    a.alpha = *static_cast<const float *>(alpha);
    a.beta = *static_cast<const float *>(beta);
    a.y = static_cast<float *>(y);
    a.x = static_cast<const float *>(x);
    a.C = (uint32_t)xDesc->dim[1];
    long long stride[kMaxTensors][4] = {};
    int dim[4];
    if (mode == IGC_SOFTMAX_MODE_CHANNEL) {
        // the locations (n,h,w): the channel dimension is taken out (size 1), the rest ordered by
        // x's strides so that neighbouring threads read neighbouring addresses
        for (int d = 0; d < 4; ++d) {
            dim[d] = d == 1 ? 1 : xDesc->dim[d];
            stride[0][d] = xDesc->stride[d];   // ordering key: the input's layout
            stride[1][d] = yDesc->stride[d];
        }
        View v = make_view(dim, stride, 2, /*merge=*/true);
        // (make_view orders by tensor 0 = x here; the kernel wants tensor 0 = y)
        for (int i = 0; i < v.rank; ++i) std::swap(v.stride[0][i], v.stride[1][i]);
        a.v = v;
        a.count = 1;
        for (int i = 0; i < v.rank; ++i) a.count *= v.dim[i];
        a.xsC = (uint32_t)xDesc->stride[1];
        a.ysC = (uint32_t)yDesc->stride[1];
        return launch(&igconv_softmax_channel_kernel, "igconv_softmax_channel_kernel", a, (a.count + 255u) / 256u, handle->stream);
    }
    for (int d = 0; d < 4; ++d) {
        dim[d] = d == 0 ? 1 : xDesc->dim[d];
        stride[0][d] = xDesc->stride[d];
        stride[1][d] = yDesc->stride[d];
    }
    View v = make_view(dim, stride, 2, /*merge=*/true);
    for (int i = 0; i < v.rank; ++i) std::swap(v.stride[0][i], v.stride[1][i]);
    a.v = v;
    a.count = 1;
    for (int i = 0; i < v.rank; ++i) a.count *= v.dim[i];
    a.xsC = (uint32_t)xDesc->stride[0];
    a.ysC = (uint32_t)yDesc->stride[0];
    return launch(&igconv_softmax_instance_kernel, "igconv_softmax_instance_kernel", a, (uint32_t)xDesc->dim[0], handle->stream);
}

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

igcStatus igcPoolingForward(igcHandle_t handle, igcPoolingDescriptor_t poolDesc, const void *alpha, igcTensorDescriptor_t xDesc,
                            const void *x, const void *beta, igcTensorDescriptor_t yDesc, void *y) {
    if (!handle || !alpha || !beta || !x || !y || !poolDesc) return IGC_STATUS_BAD_PARAM;
    if (!poolDesc->set) return IGC_STATUS_NOT_INITIALIZED;
    igcStatus st = check_float_tensor(xDesc, false);
    if (st == IGC_STATUS_SUCCESS) st = check_float_tensor(yDesc, true);
    if (st != IGC_STATUS_SUCCESS) return st;
    int n, c, p, q;
    st = igcGetPooling2dForwardOutputDim(poolDesc, xDesc, &n, &c, &p, &q);
    if (st != IGC_STATUS_SUCCESS) return st;
    if (yDesc->dim[0] != n || yDesc->dim[1] != c || yDesc->dim[2] != p || yDesc->dim[3] != q) return IGC_STATUS_BAD_PARAM;
    if ((uintptr_t)x % 4 || (uintptr_t)y % 4) return IGC_STATUS_BAD_PARAM;
    PoolArgs a{};
    long long stride[kMaxTensors][4] = {};
    for (int d = 0; d < 4; ++d) stride[0][d] = yDesc->stride[d];
    a.v = make_view(yDesc->dim, stride, 1, /*merge=*/false);
    a.count = (uint32_t)((long long)n * c * p * q);
    a.mode = poolDesc->mode;
    a.H = xDesc->dim[2]; a.W = xDesc->dim[3];
    a.win_h = poolDesc->win_h; a.win_w = poolDesc->win_w;
    a.pad_h = poolDesc->pad_h; a.pad_w = poolDesc->pad_w; a.u = poolDesc->u; a.v_ = poolDesc->v;
    for (int d = 0; d < 4; ++d) a.xs[d] = (uint32_t)xDesc->stride[d];
    a.x_bytes = (uint32_t)(extent(xDesc->dim, xDesc->stride) * 4);
    a.y_bytes = (uint32_t)(extent(yDesc->dim, yDesc->stride) * 4);
    a.alpha = *static_cast<const float *>(alpha);
    a.beta = *static_cast<const float *>(beta);
    a.y = static_cast<float *>(y);
    a.x = static_cast<const float *>(x);
    const uint32_t blocks = (a.count + 255u) / 256u;
    // w stride 1 in x and y: the row-strip kernel, with as many output rows per workgroup (at most 64) as
    // fit its LDS (the rows of x they touch) within 64 KB
    if (xDesc->stride[3] == 1 && yDesc->stride[3] == 1 && !std::getenv("IGCONV_POOL_GENERAL")) {
        PoolRowsArgs r{};
        r.mode = a.mode; r.H = a.H; r.W = a.W; r.P = p; r.Q = q;
        r.win_h = a.win_h; r.win_w = a.win_w; r.pad_h = a.pad_h; r.pad_w = a.pad_w; r.u = a.u; r.v_ = a.v_;
        r.C = c;
        for (int d = 0; d < 3; ++d) {
            r.xs[d] = (uint32_t)xDesc->stride[d];
            r.ys[d] = (uint32_t)yDesc->stride[d];
        }
        r.x_bytes = a.x_bytes; r.y_bytes = a.y_bytes; r.alpha = a.alpha; r.beta = a.beta; r.y = a.y; r.x = a.x;
        for (int tp = std::min(64, p); tp >= 1; tp = tp > 1 ? (tp + 1) / 2 : 0) {
            const long long xrows = std::min<long long>((long long)(tp - 1) * r.u + r.win_h, r.H);
            const long long lds = xrows * r.W * 4;
            const int strips = (p + tp - 1) / tp;
            const long long nblocks = (long long)n * c * strips;
            if (lds > 64 * 1024 || nblocks >= (1ll << 31)) continue;
            r.TP = tp; r.strips = strips;
            if (!magic_of((uint32_t)strips, &r.mStrips) || !magic_of((uint32_t)c, &r.mC) || !magic_of((uint32_t)r.W, &r.mW) ||
                !magic_of((uint32_t)r.Q, &r.mQ))
                break;
            if (a.win_h == 3 && a.win_w == 3)
                return launch(&igconv_pooling_rows_kernel<3, 3>, "igconv_pooling_rows_kernel", r, (uint32_t)nblocks, handle->stream, (size_t)lds);
            if (a.win_h == 2 && a.win_w == 2)
                return launch(&igconv_pooling_rows_kernel<2, 2>, "igconv_pooling_rows_kernel", r, (uint32_t)nblocks, handle->stream, (size_t)lds);
            return launch(&igconv_pooling_rows_kernel<0, 0>, "igconv_pooling_rows_kernel", r, (uint32_t)nblocks, handle->stream, (size_t)lds);
        }
    }
    if (a.win_h == 3 && a.win_w == 3) return launch(&igconv_pooling_kernel<3, 3>, "igconv_pooling_kernel", a, blocks, handle->stream);
    if (a.win_h == 2 && a.win_w == 2) return launch(&igconv_pooling_kernel<2, 2>, "igconv_pooling_kernel", a, blocks, handle->stream);
    return launch(&igconv_pooling_kernel<0, 0>, "igconv_pooling_kernel", a, blocks, handle->stream);
}

igcStatus igcSoftmaxBackward(igcHandle_t handle, igcSoftmaxMode mode, const void *alpha, igcTensorDescriptor_t yDesc,
                             const void *y, igcTensorDescriptor_t dyDesc, const void *dy, const void *beta,
                             igcTensorDescriptor_t dxDesc, void *dx) {
    if (!handle || !alpha || !beta || !y || !dy || !dx) return IGC_STATUS_BAD_PARAM;
    if (mode != IGC_SOFTMAX_MODE_INSTANCE && mode != IGC_SOFTMAX_MODE_CHANNEL) return IGC_STATUS_BAD_PARAM;
    igcStatus st = check_float_tensor(yDesc, false);
    if (st == IGC_STATUS_SUCCESS) st = check_float_tensor(dyDesc, false);
    if (st == IGC_STATUS_SUCCESS) st = check_float_tensor(dxDesc, true);
    if (st != IGC_STATUS_SUCCESS) return st;
    if (!same_dims(yDesc, dxDesc) || !same_dims(dyDesc, dxDesc)) return IGC_STATUS_BAD_PARAM;
    if ((uintptr_t)y % 4 || (uintptr_t)dy % 4 || (uintptr_t)dx % 4) return IGC_STATUS_BAD_PARAM;
    SoftmaxBwdArgs a{};
    a.alpha = *static_cast<const float *>(alpha);
    a.beta = *static_cast<const float *>(beta);
    a.y = static_cast<const float *>(y);
    a.dy = static_cast<const float *>(dy);
    a.dx = static_cast<float *>(dx);
    a.C = (uint32_t)yDesc->dim[1];
    // the group's dimension(s) taken out: the channel (per location) or nothing but the image
    // index (per image); the rest ordered by y's strides
    const int out_dim = mode == IGC_SOFTMAX_MODE_CHANNEL ? 1 : 0;
    long long stride[kMaxTensors][4] = {};
    int dim[4];
    for (int d = 0; d < 4; ++d) {
        dim[d] = d == out_dim ? 1 : yDesc->dim[d];
        stride[0][d] = yDesc->stride[d];
        stride[1][d] = dxDesc->stride[d];
        stride[2][d] = dyDesc->stride[d];
    }
    a.v = make_view(dim, stride, 3, /*merge=*/true);
    a.count = 1;
    for (int i = 0; i < a.v.rank; ++i) a.count *= a.v.dim[i];
    a.sC[0] = (uint32_t)yDesc->stride[out_dim];
    a.sC[1] = (uint32_t)dxDesc->stride[out_dim];
    a.sC[2] = (uint32_t)dyDesc->stride[out_dim];
    if (mode == IGC_SOFTMAX_MODE_CHANNEL)
        return launch(&igconv_softmax_bwd_channel_kernel, "igconv_softmax_bwd_channel_kernel", a, (a.count + 255u) / 256u,
                      handle->stream);
    return launch(&igconv_softmax_bwd_instance_kernel, "igconv_softmax_bwd_instance_kernel", a, (uint32_t)yDesc->dim[0],
                  handle->stream);
}

igcStatus igcPoolingBackward(igcHandle_t handle, igcPoolingDescriptor_t poolDesc, const void *alpha, igcTensorDescriptor_t dyDesc,
                             const void *dy, igcTensorDescriptor_t xDesc, const void *x, const void *beta,
                             igcTensorDescriptor_t dxDesc, void *dx) {
    if (!handle || !alpha || !beta || !x || !dy || !dx || !poolDesc) return IGC_STATUS_BAD_PARAM;
    if (!poolDesc->set) return IGC_STATUS_NOT_INITIALIZED;
    igcStatus st = check_float_tensor(xDesc, false);
    if (st == IGC_STATUS_SUCCESS) st = check_float_tensor(dyDesc, false);
    if (st == IGC_STATUS_SUCCESS) st = check_float_tensor(dxDesc, true);
    if (st != IGC_STATUS_SUCCESS) return st;
    int n, c, p, q;
    st = igcGetPooling2dForwardOutputDim(poolDesc, xDesc, &n, &c, &p, &q);
    if (st != IGC_STATUS_SUCCESS) return st;
    if (dyDesc->dim[0] != n || dyDesc->dim[1] != c || dyDesc->dim[2] != p || dyDesc->dim[3] != q) return IGC_STATUS_BAD_PARAM;
    if (!same_dims(xDesc, dxDesc)) return IGC_STATUS_BAD_PARAM;
    if ((uintptr_t)x % 4 || (uintptr_t)dy % 4 || (uintptr_t)dx % 4) return IGC_STATUS_BAD_PARAM;
    PoolBwdArgs a{};
    long long stride[kMaxTensors][4] = {};
    for (int d = 0; d < 4; ++d) stride[0][d] = dxDesc->stride[d];
    a.v = make_view(dxDesc->dim, stride, 1, /*merge=*/false);
    a.count = (uint32_t)((long long)n * c * xDesc->dim[2] * xDesc->dim[3]);
    a.mode = poolDesc->mode;
    a.H = xDesc->dim[2]; a.W = xDesc->dim[3]; a.P = p; a.Q = q;
    a.win_h = poolDesc->win_h; a.win_w = poolDesc->win_w;
    a.pad_h = poolDesc->pad_h; a.pad_w = poolDesc->pad_w; a.u = poolDesc->u; a.v_ = poolDesc->v;
    for (int d = 0; d < 4; ++d) {
        a.xs[d] = (uint32_t)xDesc->stride[d];
        a.dys[d] = (uint32_t)dyDesc->stride[d];
    }
    a.x_bytes = (uint32_t)(extent(xDesc->dim, xDesc->stride) * 4);
    a.dy_bytes = (uint32_t)(extent(dyDesc->dim, dyDesc->stride) * 4);
    a.dx_bytes = (uint32_t)(extent(dxDesc->dim, dxDesc->stride) * 4);
    a.alpha = *static_cast<const float *>(alpha);
    a.beta = *static_cast<const float *>(beta);
    a.dx = static_cast<float *>(dx);
    a.x = static_cast<const float *>(x);
    a.dy = static_cast<const float *>(dy);
    // w stride 1 everywhere: the row-strip kernel, with as many rows per workgroup (at most 64)
    // as its LDS (rows of x, two words per covering window) allows within 64 KB
    if (xDesc->stride[3] == 1 && dyDesc->stride[3] == 1 && dxDesc->stride[3] == 1 && !std::getenv("IGCONV_POOL_GENERAL")) {
        PoolBwdRowsArgs r{};
        r.mode = a.mode; r.H = a.H; r.W = a.W; r.P = p; r.Q = q;
        r.win_h = a.win_h; r.win_w = a.win_w; r.pad_h = a.pad_h; r.pad_w = a.pad_w; r.u = a.u; r.v_ = a.v_;
        r.C = c;
        for (int d = 0; d < 3; ++d) {
            r.xs[d] = (uint32_t)xDesc->stride[d];
            r.dys[d] = (uint32_t)dyDesc->stride[d];
            r.dxs[d] = (uint32_t)dxDesc->stride[d];
        }
        r.x_bytes = a.x_bytes; r.dy_bytes = a.dy_bytes; r.dx_bytes = a.dx_bytes;
        r.alpha = a.alpha; r.beta = a.beta; r.dx = a.dx; r.x = a.x; r.dy = a.dy;
        for (int th = std::min(64, r.H); th >= 1; th = th > 1 ? (th + 1) / 2 : 0) {
            const int strips = (r.H + th - 1) / th;
            int xrows = 0, wrows = 0;
            for (int s = 0; s < strips; ++s) {
                const int h0 = s * th, h1 = std::min(h0 + th, r.H);
                const int t0 = h0 + r.pad_h - (r.win_h - 1);
                const int p_lo = t0 <= 0 ? 0 : (t0 + r.u - 1) / r.u, p_hi = std::min(p - 1, (h1 - 1 + r.pad_h) / r.u);
                if (p_hi < p_lo) continue;
                wrows = std::max(wrows, p_hi - p_lo + 1);
                xrows = std::max(xrows, std::min(p_hi * r.u - r.pad_h + r.win_h, r.H) - std::max(p_lo * r.u - r.pad_h, 0));
            }
            if (r.mode != IGC_POOLING_MAX) xrows = 0;
            const long long lds = ((long long)xrows * r.W + 2ll * wrows * r.Q) * 4;
            const long long blocks = (long long)n * c * strips;
            if (lds > 64 * 1024 || blocks >= (1ll << 31)) continue;
            r.TH = th; r.strips = strips; r.xrows_max = xrows; r.wrows_max = wrows;
            r.wpi = r.Q <= 256 ? 256 / r.Q : 0;
            r.rpi = r.W <= 256 ? 256 / r.W : 0;
            if (!magic_of((uint32_t)strips, &r.mStrips) || !magic_of((uint32_t)c, &r.mC) || !magic_of((uint32_t)r.u, &r.mu) ||
                !magic_of((uint32_t)r.v_, &r.mv) || !magic_of((uint32_t)r.W, &r.mW) || !magic_of((uint32_t)r.Q, &r.mQ))
                break;
            return launch(&igconv_pooling_bwd_rows_kernel, "igconv_pooling_bwd_rows_kernel", r, (uint32_t)blocks, handle->stream,
                          (size_t)lds);
        }
    }
    return launch(&igconv_pooling_bwd_kernel, "igconv_pooling_bwd_kernel", a, (a.count + 255u) / 256u, handle->stream);
}

igcStatus igcTransformTensor(igcHandle_t handle, const void *alpha, igcTensorDescriptor_t xDesc, const void *x, const void *beta,
                             igcTensorDescriptor_t yDesc, void *y) {
    if (!handle || !alpha || !beta || !x || !y) return IGC_STATUS_BAD_PARAM;
    igcStatus st = check_float_tensor(xDesc, false);
    if (st == IGC_STATUS_SUCCESS) st = check_float_tensor(yDesc, true);
    if (st != IGC_STATUS_SUCCESS) return st;
    if (!same_dims(xDesc, yDesc) || (uintptr_t)x % 4 || (uintptr_t)y % 4) return IGC_STATUS_BAD_PARAM;
    const float a = *static_cast<const float *>(alpha), b = *static_cast<const float *>(beta);
    // Dimensions ordered by y's strides, merged where both tensors allow.  If x is contiguous along another
    // dimension than y (a change of layout), tiles of that plane go through LDS; else element by element.
    long long stride[kMaxTensors][4] = {};
    for (int d = 0; d < 4; ++d) {
        stride[0][d] = yDesc->stride[d];
        stride[1][d] = xDesc->stride[d];
    }
    const View v = make_view(yDesc->dim, stride, 2, /*merge=*/true);
    const int B = v.rank - 1;
    int A = -1;
    for (int d = 0; d < v.rank; ++d)
        if (v.stride[1][d] == 1u && v.dim[d] > 1u) A = d;
    if (v.rank >= 2 && v.rank <= 4 && v.stride[0][B] == 1u && A >= 0 && A != B && v.dim[A] >= 16u && v.dim[B] >= 16u) {
        TransposeArgs t{};
        t.dimA = v.dim[A]; t.dimB = v.dim[B];
        t.tilesA = (t.dimA + 63u) / 64u; t.tilesB = (t.dimB + 63u) / 64u;
        t.xsB = v.stride[1][B]; t.ysA = v.stride[0][A];
        uint32_t outer[2] = {1u, 1u};
        int no = 0;
        for (int d = 0; d < v.rank; ++d)
            if (d != A && d != B) {
                outer[no] = v.dim[d];
                t.xsO[no] = v.stride[1][d];
                t.ysO[no] = v.stride[0][d];
                ++no;
            }
        t.outer1 = outer[1];
        const long long blocks = (long long)t.tilesA * t.tilesB * outer[0] * outer[1];
        if (no <= 2 && blocks < (1ll << 31) && magic_of(t.tilesA, &t.mTilesA) && magic_of(t.tilesB, &t.mTilesB) &&
            magic_of(t.outer1, &t.mOuter1)) {
            t.x_bytes = (uint32_t)(extent(xDesc->dim, xDesc->stride) * 4);
            t.y_bytes = (uint32_t)(extent(yDesc->dim, yDesc->stride) * 4);
            t.alpha = a; t.beta = b;
            t.y = static_cast<float *>(y);
            t.x = static_cast<const float *>(x);
            return launch(&igconv_transpose_kernel, "igconv_transpose_kernel", t, (uint32_t)blocks, handle->stream);
        }
    }
    const void *in[1] = {x};
    return run_elementwise(handle, EW_ADD, 0, a, b, yDesc, y, 1, &xDesc->stride, in);
}

}  // extern "C"
