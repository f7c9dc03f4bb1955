// Double-precision implicit-GEMM convolution (paper, Section 2: every routine exists in
// single and double precision; Section 3: the lowered matrix D_m is formed tile by tile in
// on-chip memory only).  One kernel serves the forward pass, backward data and backward
// filter: all three are products O (rows x columns) = A (rows x reduction) . B (reduction x
// columns) in which an element of B is an element of an image picked by TWO index sets,
//
//   column  j  -> (j0, j1, j2) by division through (PQ, Q): base j0*xsN, window origin
//                 (j1*u - pad_h, j2*v - pad_w)
//   reduction k -> (i0, i1, i2) by division through (RS, S): offset i0*xsC, window offset
//                 (dh, dw) = (i1, i2)            [forward, backward data; reversed for eq. 2]
//                         or (i1*redMulH, i2*redMulW)   [backward filter]
//   B[k][j] = image[base + offset + (h0+dh)*xsH + (w0+dw)*xsW], zero outside the image,
//
// and an element of A is a[m*wsRow + i0*wsRed + wTap0 + i1*wsTapR + i2*wsTapS].  The host
// names the sets: forward j = (n,p,q), k = (c,r,s), a = filter; backward data the same over
// dy per stride phase with the filter's strides exchanged; backward filter j = (c,r,s),
// k = (n,p,q), a = dy.
//
// Tile 64 x 64 x 16, 256 threads = 2 x 2 wavefronts of 32 x 32, v_mfma_f64_16x16x4_f64
// (64 cycles each on this chip, so a plain double-buffered loop keeps the matrix pipe the
// bottleneck).  LDS holds both operands k-major ([k][row]) so that the 16 lanes sharing a k
// read 16 consecutive doubles.  One workgroup per (tile, reduction range).
#ifndef IGCONV_KERNEL_F64_HPP_
#define IGCONV_KERNEL_F64_HPP_

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "igconv_params.h"

namespace igc {

typedef double f64x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kF64BM = 64, kF64BN = 64, kF64BK = 16;
constexpr int kF64LdsBytes = 2 * kF64BK * (kF64BM + kF64BN) * 8;
constexpr uint32_t kF64OutOfRange = 0x80000000u;   // a byte offset no buffer reaches: reads as zero

__device__ __forceinline__ uint32_t f64_mdiv(uint32_t n, Magic m) { return (__umulhi(n, m.mul) + n) >> m.shift; }

__device__ __forceinline__ double f64_load(__amdgpu_buffer_rsrc_t buf, uint32_t byte_off) {
    const u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(buf, byte_off, 0, 0);
    return __builtin_bit_cast(double, v);
}

// WGRAD: the reduction index moves the window by (i1*redMulH, i2*redMulW) (backward filter);
// otherwise by the tap (i1, i2) itself, reversed when p.flip is set.
template <bool WGRAD>
__global__ __launch_bounds__(256) void igconv_f64_kernel(const ConvKernelParams p) {
    constexpr int BM = kF64BM, BN = kF64BN, BK = kF64BK;
    __shared__ double As[2][BK][BM];
    __shared__ double Bs[2][BK][BN];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int l16 = lane & 15, lq = lane >> 4;

    // (tile, range) of this workgroup: numbered in contiguous ranges per XCD
    const int tiles = p.tilesM * p.tilesN;
    const int item = (int)(blockIdx.x % 8u) * p.tilesPerXcd + (int)(blockIdx.x / 8u);
    if (item >= tiles * p.splits) return;
    const int split = item / tiles, tile = item - split * tiles;
    const int m0 = (tile % p.tilesM) * BM, n0 = (tile / p.tilesM) * BN;
    const int s_begin = split * p.stepsPerSplit, s_end = min(p.ksteps, s_begin + p.stepsPerSplit);

    const __amdgpu_buffer_rsrc_t xbuf = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p.x), 0, p.x_bytes, 0x00020000u);
    const __amdgpu_buffer_rsrc_t wbuf = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p.w), 0, p.w_bytes, 0x00020000u);
    const __amdgpu_buffer_rsrc_t ybuf = __builtin_amdgcn_make_buffer_rsrc(
        static_cast<uint8_t *>(p.y) + (size_t)split * p.ySplitBytes, 0, p.y_bytes, 0x00020000u);

    // ---- B role: one column, four consecutive reduction indices per step
    const int b_col = tid & 63, b_kq = (tid >> 6) * 4;
    const int j = n0 + b_col;
    const bool b_ok = j < p.NPQ;
    int b_base = 0, b_h0 = 0, b_w0 = 0;
    {
        const uint32_t jj = b_ok ? (uint32_t)j : 0u;
        const uint32_t j0 = f64_mdiv(jj, p.mPQ), rem = jj - j0 * (uint32_t)p.PQ;
        const uint32_t j1 = f64_mdiv(rem, p.mQ), j2 = rem - j1 * (uint32_t)p.Q;
        b_base = (int)j0 * p.xsN;
        b_h0 = (int)j1 * p.u - p.pad_h;
        b_w0 = (int)j2 * p.v - p.pad_w;
    }
    // ---- A role: one row, four consecutive reduction indices per step
    const int a_row = tid >> 2, a_kq = (tid & 3) * 4;
    const int m = m0 + a_row;
    const bool a_ok = m < p.K;
    const int a_base = a_ok ? m * p.wsRow + p.wTap0 : 0;

    double a_reg[4], b_reg[4];
    auto fetch = [&](int step) {
        {   // B
            const uint32_t k0 = (uint32_t)(step * BK + b_kq);
            uint32_t i0 = f64_mdiv(k0, p.mRS), rem = k0 - i0 * (uint32_t)p.RS;
            uint32_t i1 = f64_mdiv(rem, p.mS), i2 = rem - i1 * (uint32_t)p.S;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                int dh, dw;
                if (WGRAD) {
                    dh = (int)i1 * p.redMulH;
                    dw = (int)i2 * p.redMulW;
                } else {
                    dh = p.flip ? p.R - 1 - (int)i1 : (int)i1;
                    dw = p.flip ? p.S - 1 - (int)i2 : (int)i2;
                }
                const int h = b_h0 + dh, w = b_w0 + dw;
                const bool ok = b_ok && (int)(k0 + e) < p.CRS && (uint32_t)h < (uint32_t)p.H && (uint32_t)w < (uint32_t)p.W;
                const uint32_t off = (uint32_t)(b_base + (int)i0 * p.xsC + h * p.xsH + w * p.xsW) * 8u;
                b_reg[e] = f64_load(xbuf, ok ? off : kF64OutOfRange);
                ++i2; ++rem;
                if (i2 == (uint32_t)p.S) { i2 = 0; ++i1; }
                if (rem == (uint32_t)p.RS) { rem = 0; i1 = 0; i2 = 0; ++i0; }
            }
        }
        {   // A
            const uint32_t k0 = (uint32_t)(step * BK + a_kq);
            uint32_t i0 = f64_mdiv(k0, p.mRS), rem = k0 - i0 * (uint32_t)p.RS;
            uint32_t i1 = f64_mdiv(rem, p.mS), i2 = rem - i1 * (uint32_t)p.S;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const bool ok = a_ok && (int)(k0 + e) < p.CRS;
                const uint32_t off = (uint32_t)(a_base + (int)i0 * p.wsRed + (int)i1 * p.wsTapR + (int)i2 * p.wsTapS) * 8u;
                a_reg[e] = f64_load(wbuf, ok ? off : kF64OutOfRange);
                ++i2; ++rem;
                if (i2 == (uint32_t)p.S) { i2 = 0; ++i1; }
                if (rem == (uint32_t)p.RS) { rem = 0; i1 = 0; i2 = 0; ++i0; }
            }
        }
    };
    auto stage = [&](int buf) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            As[buf][a_kq + e][a_row] = a_reg[e];
            Bs[buf][b_kq + e][b_col] = b_reg[e];
        }
    };

    f64x4 acc[2][2];
#pragma unroll
    for (int bi = 0; bi < 2; ++bi)
#pragma unroll
        for (int bj = 0; bj < 2; ++bj) acc[bi][bj] = f64x4{0.0, 0.0, 0.0, 0.0};

    if (s_begin < s_end) {
        fetch(s_begin);
        stage(0);
    }
    __syncthreads();
    int cur = 0;
    for (int s = s_begin; s < s_end; ++s) {
        const bool more = s + 1 < s_end;
        if (more) fetch(s + 1);
#pragma unroll
        for (int kg = 0; kg < BK / 4; ++kg) {
            const int kk = kg * 4 + lq;
            const double a0 = As[cur][kk][wm * 32 + l16], a1 = As[cur][kk][wm * 32 + 16 + l16];
            const double b0 = Bs[cur][kk][wn * 32 + l16], b1 = Bs[cur][kk][wn * 32 + 16 + l16];
            acc[0][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b0, acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b1, acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b0, acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b1, acc[1][1], 0, 0, 0);
        }
        if (more) stage(cur ^ 1);
        __syncthreads();
        cur ^= 1;
    }

    // ---- epilogue: lane (l16, lq), value v of block (bi, bj) is row 4*v + lq, column l16
    const double alpha = p.alpha64, beta = p.beta64;
#pragma unroll
    for (int bj = 0; bj < 2; ++bj) {
        const int col = n0 + wn * 32 + bj * 16 + l16;
        if (col >= p.NPQ) continue;
        const uint32_t j0 = f64_mdiv((uint32_t)col, p.mPQ), rem = (uint32_t)col - j0 * (uint32_t)p.PQ;
        const uint32_t j1 = f64_mdiv(rem, p.mQ), j2 = rem - j1 * (uint32_t)p.Q;
        const int ycol = (int)j0 * p.ysN + (int)j1 * p.ysP + (int)j2 * p.ysQ;
#pragma unroll
        for (int bi = 0; bi < 2; ++bi)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = m0 + wm * 32 + bi * 16 + 4 * v + lq;
                if (row >= p.K) continue;
                const uint32_t off = (uint32_t)(ycol + row * p.ysK) * 8u;
                double r = alpha * acc[bi][bj][v];
                if (beta != 0.0) r += beta * f64_load(ybuf, off);
                __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2, r), ybuf, off, 0, 0);
            }
    }
}

}  // namespace igc
#endif
