// Backward-filter kernels: the generic gather with columns (c,r,s) and the reduction over
// (n,p,q), plus the kernel that adds up the ranges of a cut reduction.
#include "igconv_instantiate.hpp"
#include "igconv_kernel_wgrad.hpp"

//    name, bf16, BM, BN, BK, WM, WN, gather mode
#define IGC_WGRAD_LIST(X) \
    X("f32 64x128x32 wgrad", false, 64, 128, 32, 2, 2, GATHER_WGRAD) \
    X("f32 128x128x32 wgrad", false, 128, 128, 32, 2, 2, GATHER_WGRAD) \
    X("bf16 64x128x32 wgrad", true, 64, 128, 32, 2, 2, GATHER_WGRAD) \
    X("bf16 128x128x32 wgrad", true, 128, 128, 32, 2, 2, GATHER_WGRAD) \
    X("f32 64x64x32 wgrad tap", false, 64, 64, 32, 2, 2, GATHER_WGRAD_TAP) \
    X("f32 128x64x32 wgrad tap", false, 128, 64, 32, 2, 2, GATHER_WGRAD_TAP) \
    X("f32 64x128x32 wgrad tap", false, 64, 128, 32, 2, 2, GATHER_WGRAD_TAP) \
    X("f32 128x128x32 wgrad tap", false, 128, 128, 32, 2, 2, GATHER_WGRAD_TAP) \
    X("bf16 64x64x32 wgrad tap", true, 64, 64, 32, 2, 2, GATHER_WGRAD_TAP) \
    X("bf16 128x64x32 wgrad tap", true, 128, 64, 32, 2, 2, GATHER_WGRAD_TAP) \
    X("bf16 64x128x32 wgrad tap", true, 64, 128, 32, 2, 2, GATHER_WGRAD_TAP) \
    X("bf16 128x128x32 wgrad tap", true, 128, 128, 32, 2, 2, GATHER_WGRAD_TAP) \
    X("f32 64x128x32 wgrad nopad", false, 64, 128, 32, 2, 2, GATHER_WGRAD_NOPAD) \
    X("f32 96x128x32 wgrad nopad", false, 96, 128, 32, 1, 4, GATHER_WGRAD_NOPAD) \
    X("f32 128x128x32 wgrad nopad", false, 128, 128, 32, 2, 2, GATHER_WGRAD_NOPAD) \
    X("f32 96x128x32 wgrad tap", false, 96, 128, 32, 1, 4, GATHER_WGRAD_TAP) \
    X("f32 96x128x32 wgrad", false, 96, 128, 32, 1, 4, GATHER_WGRAD) \
    X("bf16 64x128x32 wgrad nopad", true, 64, 128, 32, 2, 2, GATHER_WGRAD_NOPAD) \
    X("bf16 128x128x32 wgrad nopad", true, 128, 128, 32, 2, 2, GATHER_WGRAD_NOPAD)

namespace igc {

template <class Cfg>
static int launch_wgrad(const ConvKernelParams &p, int grid, void *stream) {
    return launch_checked(&igconv_wgrad_kernel<Cfg>, "igconv_wgrad_kernel", p, grid, Cfg::THREADS, stream);
}

#define IGC_WGRAD_INSTANTIATE(NAME, BF16, BM, BN, BK, WM, WN, GMODE) \
    template __global__ void igconv_wgrad_kernel<WgradConfig<BF16, BM, BN, BK, WM, WN, GMODE>>(const ConvKernelParams);
IGC_WGRAD_LIST(IGC_WGRAD_INSTANTIATE)

#if !defined(__HIP_DEVICE_COMPILE__)
#define IGC_WGRAD_ROW(NAME, BF16, BM, BN, BK, WM, WN, GMODE)                                         \
    {NAME, BF16, BM, BN, BK, false, false, GMODE, 256, WgradConfig<BF16, BM, BN, BK, WM, WN, GMODE>::LDS_BYTES, \
     &launch_wgrad<WgradConfig<BF16, BM, BN, BK, WM, WN, GMODE>>},
static const KernelInfo kWgradRows[] = {IGC_WGRAD_LIST(IGC_WGRAD_ROW)};
const KernelGroup kGroupWgrad = {kWgradRows, sizeof(kWgradRows) / sizeof(kWgradRows[0])};
#endif

}  // namespace igc

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

// The same sums - the same additions in the same order, so the same bits - for at most 16 parts of whole 16-byte
// vectors: a thread takes four consecutive elements and requests all its loads before it adds.  (With few parts the
// kernel above leaves most of its threads without a load: 9 parts of 3.5 MB took 14.8 us.)
__global__ __launch_bounds__(256) void igconv_sum_few_parts_kernel(const float4 *parts, float4 *out, uint32_t n4, int count,
                                                                   uint32_t stride4, float alpha, float beta) {
    const uint32_t e = blockIdx.x * 256u + threadIdx.x;
    if (e >= n4) return;
    float4 v[16];
#pragma unroll
    for (int s = 0; s < 16; ++s)
        if (s < count) v[s] = parts[(size_t)s * stride4 + e];
    // runs of one part (count <= 8) or of two: eight runs, each added from zero, then the runs added in order
    float4 sum = {0.f, 0.f, 0.f, 0.f};
    auto add = [](float4 &a, const float4 &b) {
        a.x += b.x;
        a.y += b.y;
        a.z += b.z;
        a.w += b.w;
    };
    const bool pairs = count > 8;
#pragma unroll
    for (int g = 0; g < 8; ++g) {
        float4 acc = {0.f, 0.f, 0.f, 0.f};
        if (pairs) {
            if (2 * g < count) add(acc, v[2 * g]);
            if (2 * g + 1 < count) add(acc, v[2 * g + 1]);
        } else {
            if (g < count) add(acc, v[g]);
        }
        if (g == 0) sum = acc;
        else add(sum, acc);
    }
    float4 r = {alpha * sum.x, alpha * sum.y, alpha * sum.z, alpha * sum.w};
    if (beta != 0.f) {
        const float4 o = out[e];
        r.x += beta * o.x;
        r.y += beta * o.y;
        r.z += beta * o.z;
        r.w += beta * o.w;
    }
    out[e] = r;
}

int launch_sum_parts(const float *parts, float *out, uint32_t n, int count, uint32_t stride, float alpha, float beta,
                     void *stream) {
    if (count <= 16 && n % 4 == 0 && stride % 4 == 0 && (uintptr_t)parts % 16 == 0 && (uintptr_t)out % 16 == 0) {
        uint32_t n4 = n / 4, stride4 = stride / 4;
        void *argv4[] = {&parts, &out, &n4, &count, &stride4, &alpha, &beta};
        return static_cast<int>(hipLaunchKernel(reinterpret_cast<const void *>(&igconv_sum_few_parts_kernel), dim3((n4 + 255u) / 256u),
                                                dim3(256), argv4, 0, static_cast<hipStream_t>(stream)));
    }
    void *argv[] = {&parts, &out, &n, &count, &stride, &alpha, &beta};
    return static_cast<int>(hipLaunchKernel(reinterpret_cast<const void *>(&igconv_sum_parts_kernel), dim3((n + 31u) / 32u),
                                            dim3(256), argv, 0, static_cast<hipStream_t>(stream)));
}

// wt[k][t][c] = w[k][c][t] (float or bfloat16; t < RS): the filter with the channel index innermost, so that the tap-major
// kernels, whose step is one tap of a run of channels, read contiguous runs of a filter row instead of elements
// RS apart.  With `exchange` the roles of k and c are exchanged as well, wt[c][t][k] = w[k][c][t]: the same for
// backward data, whose rows are c and whose reduction runs over k.  A thread per element, writes contiguous.
template <class T>
__global__ __launch_bounds__(256) void igconv_filter_taps_outer_kernel(const T *w, T *wt, uint32_t total, int K, int C, int RS,
                                                                       int exchange, Magic mInner, Magic mRS) {
    const uint32_t idx = blockIdx.x * 256u + threadIdx.x;
    if (idx >= total) return;
    const uint32_t inner_n = exchange ? (uint32_t)K : (uint32_t)C;
    const uint32_t ot = (__umulhi(idx, mInner.mul) + idx) >> mInner.shift, inner = idx - ot * inner_n;
    const uint32_t outer = (__umulhi(ot, mRS.mul) + ot) >> mRS.shift, t = ot - outer * (uint32_t)RS;
    const uint32_t k = exchange ? inner : outer, c = exchange ? outer : inner;
    wt[idx] = w[((size_t)k * C + c) * RS + t];
}

int launch_filter_taps_outer(const void *w, void *wt, int elem_bytes, int K, int C, int RS, bool exchange, Magic mInner, Magic mRS,
                             void *stream) {
    uint32_t total = (uint32_t)((size_t)K * C * RS);
    int ex = exchange ? 1 : 0;
    void *argv[] = {&w, &wt, &total, &K, &C, &RS, &ex, &mInner, &mRS};
    const void *kernel = elem_bytes == 2 ? reinterpret_cast<const void *>(&igconv_filter_taps_outer_kernel<uint16_t>)
                                         : reinterpret_cast<const void *>(&igconv_filter_taps_outer_kernel<float>);
    return static_cast<int>(hipLaunchKernel(kernel, dim3((total + 255u) / 256u), dim3(256), argv, 0, static_cast<hipStream_t>(stream)));
}

// xp = x extended by its zero border, packed N,C,H+2pad_h,W+2pad_w (float).  With few channels and a zero border
// the forward pass has to test every gathered element against the window (the generic gather); over xp the same
// layer has no border and runs with the tap offsets tabulated.  A thread per element of xp.
struct PadImageArgs {
    const float *x;
    float *xp;
    uint32_t total;
    int H, W, Hp, Wp, pad_h, pad_w, C;
    uint32_t xs[4];
    Magic mWp, mHp, mC;
};

__global__ __launch_bounds__(256) void igconv_pad_image_kernel(const PadImageArgs a) {
    const uint32_t idx = blockIdx.x * 256u + threadIdx.x;
    if (idx >= a.total) return;
    auto mdiv = [](uint32_t n, Magic m) { return (__umulhi(n, m.mul) + n) >> m.shift; };
    uint32_t rest = mdiv(idx, a.mWp);
    const uint32_t wp = idx - rest * (uint32_t)a.Wp;
    uint32_t q = mdiv(rest, a.mHp);
    const uint32_t hp = rest - q * (uint32_t)a.Hp;
    const uint32_t n = mdiv(q, a.mC), c = q - n * (uint32_t)a.C;
    const uint32_t h = hp - (uint32_t)a.pad_h, w = wp - (uint32_t)a.pad_w;   // (wrap below zero: fail the test)
    float v = 0.f;
    if (h < (uint32_t)a.H && w < (uint32_t)a.W) v = a.x[(size_t)n * a.xs[0] + (size_t)c * a.xs[1] + (size_t)h * a.xs[2] + (size_t)w * a.xs[3]];
    a.xp[idx] = v;
}

int launch_pad_image(const float *x, float *xp, int N, int C, int H, int W, int pad_h, int pad_w, const long long xs[4], Magic mWp,
                     Magic mHp, Magic mC, void *stream) {
    const int Hp = H + 2 * pad_h, Wp = W + 2 * pad_w;
    PadImageArgs a{x, xp, (uint32_t)((size_t)N * C * Hp * Wp), H, W, Hp, Wp, pad_h, pad_w, C,
                   {(uint32_t)xs[0], (uint32_t)xs[1], (uint32_t)xs[2], (uint32_t)xs[3]}, mWp, mHp, mC};
    void *argv[] = {&a};
    return static_cast<int>(hipLaunchKernel(reinterpret_cast<const void *>(&igconv_pad_image_kernel), dim3((a.total + 255u) / 256u),
                                            dim3(256), argv, 0, static_cast<hipStream_t>(stream)));
}

// ---- backward data of a strided layer with few channels, as ONE forward pass ------------------
// Per axis the rows of dx split into u phases: with g = h + pad, a = g mod u and i = g div u, row h
// meets exactly the taps e = a + u*t (e counted in reading direction) and those read dy row i - t.
// All phases share the tap grid t < R' = ceil(R/u) once a missing tap (e >= R) counts as a zero
// weight, so that
//   y'[n, (a,b,c), i, j] = sum_{k,t,t'} W(k,c,a+u*t,b+v*t') * dy[n,k,i-t,j-t']
// is a stride-1 forward pass over dy with u*v*C output maps and the filter below, and
//   dx[n,c,h,w] = y'[n, (a,b,c), i, j].
// A first layer's three channels thus fill 48 rows of the MFMA tiles instead of 3 of 32 in each of 16
// launches.  F[m][k][tau][sigma], m = (a*v + b)*C + c, holds W(k, c, a + u*(R'-1-tau), b + v*(S'-1-sigma))
// - the forward kernels read tap tau at row i - (R'-1) + tau - or zero past the filter's end.
struct PhaseFilterArgs {
    const float *w;
    float *f;
    uint32_t total;          // elements of F
    int K, C, R, S, u, v, Rp, Sp, flip;
    Magic mSp, mRp, mK, mC, mv;
};

__global__ __launch_bounds__(256) void igconv_pack_phase_filter_kernel(const PhaseFilterArgs a) {
    const uint32_t idx = blockIdx.x * 256u + threadIdx.x;
    if (idx >= a.total) return;
    auto mdiv = [](uint32_t n, Magic m) { return (__umulhi(n, m.mul) + n) >> m.shift; };
    uint32_t rest = mdiv(idx, a.mSp);
    const uint32_t sigma = idx - rest * (uint32_t)a.Sp;
    uint32_t q = mdiv(rest, a.mRp);
    const uint32_t tau = rest - q * (uint32_t)a.Rp;
    rest = q;
    q = mdiv(rest, a.mK);
    const uint32_t k = rest - q * (uint32_t)a.K;
    const uint32_t m = q;
    const uint32_t ab = mdiv(m, a.mC), c = m - ab * (uint32_t)a.C;
    const uint32_t pa = mdiv(ab, a.mv), pb = ab - pa * (uint32_t)a.v;
    const int e = (int)pa + a.u * (a.Rp - 1 - (int)tau), f = (int)pb + a.v * (a.Sp - 1 - (int)sigma);
    float val = 0.f;
    if (e < a.R && f < a.S) {
        const int r = a.flip ? a.R - 1 - e : e, sx = a.flip ? a.S - 1 - f : f;
        val = a.w[(((size_t)k * a.C + c) * a.R + r) * a.S + sx];
    }
    a.f[idx] = val;
}

int launch_pack_phase_filter(const float *w, float *f, int K, int C, int R, int S, int u, int v, int Rp, int Sp, bool flip,
                             Magic mSp, Magic mRp, Magic mK, Magic mC, Magic mv, void *stream) {
    PhaseFilterArgs a{w, f, (uint32_t)((size_t)u * v * C * K * Rp * Sp), K, C, R, S, u, v, Rp, Sp, flip ? 1 : 0, mSp, mRp, mK, mC, mv};
    void *argv[] = {&a};
    return static_cast<int>(hipLaunchKernel(reinterpret_cast<const void *>(&igconv_pack_phase_filter_kernel),
                                            dim3((a.total + 255u) / 256u), dim3(256), argv, 0, static_cast<hipStream_t>(stream)));
}

// dx[n,c,h,w] = alpha * y'[n,(a,b,c),i,j] + beta * dx[n,c,h,w] (y' packed N, u*v*C, I, J; rows i >= I or columns
// j >= J belong to input rows no window reaches: zero).  A thread per column w of four consecutive rows of dx (lanes
// along w): the decode of (n, c, first row, w) and of the column's phase serves the four elements, and their four
// loads are requested together.
struct PhaseScatterArgs {
    const float *y;
    float *dx;
    uint32_t total;          // N*C*ceil(H/4)*W
    int C, H, W, HB, I, J, u, v, pad_h, pad_w;
    uint32_t dxs[4];         // strides of dx in elements
    Magic mW, mHB, mC, mu, mv;
    float alpha, beta;
};

__global__ __launch_bounds__(256) void igconv_phase_scatter_kernel(const PhaseScatterArgs a) {
    const uint32_t idx = blockIdx.x * 256u + threadIdx.x;
    if (idx >= a.total) return;
    auto mdiv = [](uint32_t n, Magic m) { return (__umulhi(n, m.mul) + n) >> m.shift; };
    uint32_t rest = mdiv(idx, a.mW);
    const uint32_t w = idx - rest * (uint32_t)a.W;
    uint32_t q = mdiv(rest, a.mHB);
    const uint32_t h0 = (rest - q * (uint32_t)a.HB) * 4u;
    const uint32_t n = mdiv(q, a.mC), c = q - n * (uint32_t)a.C;
    const uint32_t gw = w + (uint32_t)a.pad_w;
    const uint32_t j = mdiv(gw, a.mv), pb = gw - j * (uint32_t)a.v;
    const uint32_t maps = (uint32_t)(a.u * a.v * a.C);
    float val[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const uint32_t gh = h0 + (uint32_t)e + (uint32_t)a.pad_h;
        const uint32_t i = mdiv(gh, a.mu), pa = gh - i * (uint32_t)a.u;
        val[e] = 0.f;
        if (h0 + (uint32_t)e < (uint32_t)a.H && i < (uint32_t)a.I && j < (uint32_t)a.J) {
            const uint32_t m = (pa * (uint32_t)a.v + pb) * (uint32_t)a.C + c;
            val[e] = a.y[(((size_t)n * maps + m) * a.I + i) * a.J + j];
        }
    }
    float *dst = a.dx + (size_t)n * a.dxs[0] + (size_t)c * a.dxs[1] + (size_t)h0 * a.dxs[2] + (size_t)w * a.dxs[3];
    float old[4] = {0.f, 0.f, 0.f, 0.f};
    if (a.beta != 0.f) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (h0 + (uint32_t)e < (uint32_t)a.H) old[e] = dst[(size_t)e * a.dxs[2]];
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        if (h0 + (uint32_t)e >= (uint32_t)a.H) break;
        float r = a.alpha * val[e];
        if (a.beta != 0.f) r += a.beta * old[e];
        dst[(size_t)e * a.dxs[2]] = r;
    }
}

int launch_phase_scatter(const float *y, float *dx, int N, int C, int H, int W, int I, int J, int u, int v, int pad_h, int pad_w,
                         const long long dxs[4], Magic mW, Magic mH, Magic mC, Magic mu, Magic mv, float alpha, float beta,
                         void *stream) {
    (void)mH;
    const int HB = (H + 3) / 4;
    Magic mHB;
    if (!magic_for((uint32_t)HB, &mHB)) return 1;
    PhaseScatterArgs a{y, dx, (uint32_t)((size_t)N * C * HB * W), C, H, W, HB, I, J, u, v, pad_h, pad_w,
                       {(uint32_t)dxs[0], (uint32_t)dxs[1], (uint32_t)dxs[2], (uint32_t)dxs[3]}, mW, mHB, mC, mu, mv,
                       alpha, beta};
    void *argv[] = {&a};
    return static_cast<int>(hipLaunchKernel(reinterpret_cast<const void *>(&igconv_phase_scatter_kernel),
                                            dim3((a.total + 255u) / 256u), dim3(256), argv, 0, static_cast<hipStream_t>(stream)));
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

// The same for whole blocks (K and C multiples of 16) and 4-byte aligned buffers, moved as dwords: a run of 16 pairs
// is 8 * taps dwords on both sides; an output dword takes its two halves from LDS.  Half as many memory
// instructions as the element-wise form.
template <int taps>
__global__ __launch_bounds__(256) void igconv_filter_exchange_dwords_kernel(const uint32_t *w, uint32_t *wt, int K, int C) {
    constexpr int ROW = 8 * taps, TOTAL = 16 * ROW, PER = (TOTAL + 255) / 256;
    __shared__ uint32_t blk32[TOTAL];
    const int k0 = blockIdx.x * 16, c0 = blockIdx.y * 16;
    uint32_t v[PER];
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        const int e = (int)threadIdx.x + 256 * i;
        const int k = e / ROW, d = e - k * ROW;
        v[i] = e < TOTAL ? w[(((size_t)(k0 + k) * C + c0) * taps) / 2 + d] : 0u;
    }
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        const int e = (int)threadIdx.x + 256 * i;
        if (e < TOTAL) blk32[e] = v[i];
    }
    __syncthreads();
    const uint16_t *blk = reinterpret_cast<const uint16_t *>(blk32);   // [k][c][t]
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        const int e = (int)threadIdx.x + 256 * i;
        if (e >= TOTAL) break;
        const int c = e / ROW, d = e - c * ROW;   // halves 2 d and 2 d + 1 of the run (k_local, t) of channel c
        const int ka = (2 * d) / taps, ta = 2 * d - ka * taps, kb = (2 * d + 1) / taps, tb = 2 * d + 1 - kb * taps;
        const uint32_t lo = blk[(ka * 16 + c) * taps + ta], hi = blk[(kb * 16 + c) * taps + tb];
        wt[(((size_t)(c0 + c) * K + k0) * taps) / 2 + d] = lo | (hi << 16);
    }
}

int launch_filter_exchange(const void *w, void *wt, int K, int C, int taps, void *stream) {
    void *argv[] = {&w, &wt, &K, &C};
    const bool dwords = K % 16 == 0 && C % 16 == 0 && (uintptr_t)w % 4 == 0 && (uintptr_t)wt % 4 == 0;
    const void *kernel = taps == 9 ? (dwords ? reinterpret_cast<const void *>(&igconv_filter_exchange_dwords_kernel<9>)
                                             : reinterpret_cast<const void *>(&igconv_filter_exchange_kernel<9>))
                                   : (dwords ? reinterpret_cast<const void *>(&igconv_filter_exchange_dwords_kernel<1>)
                                             : reinterpret_cast<const void *>(&igconv_filter_exchange_kernel<1>));
    return static_cast<int>(hipLaunchKernel(kernel,
                                            dim3((K + 15) / 16, (C + 15) / 16), dim3(256), argv, 0,
                                            static_cast<hipStream_t>(stream)));
}

}  // namespace igc
