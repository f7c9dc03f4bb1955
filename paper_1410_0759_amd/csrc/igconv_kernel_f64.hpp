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
// Tile (32 NB) x (32 NB) x 16 (NB = 2 is built: 64 x 64), 512 threads: wavefronts 0-3 multiply (2 x 2 of them,
// NB x NB blocks of v_mfma_f64_16x16x4_f64 each), wavefronts 4-7 move the operands from global memory into
// LDS, requested two steps ahead of the multiplication (two register sets), one barrier per step; four
// workgroups per compute unit (64 registers).  Backward filter, 64 x 128 x 28 x 28 -> 128, 3 x 3: 54 TFLOP/s;
// as one instruction stream per wavefront with the loads one step ahead, two workgroups per compute unit:
// 31.  What the steps to 54 were worth: the second pair of workgroups 31 -> 42 (a step waited for its loads);
// keeping the compiler from branching around the loads of a step past the end of the reduction - it waited
// for every outstanding load inside the branches - and pinning the requests before the staging: 42 -> 54.
// With the moving wavefronts idle the multiplying ones reach 68: on this chip the vector instructions of one
// wavefront and the double-precision MFMAs of another do not overlap (the movers alone take half of the
// multipliers' time, and the times add), so what is left is the movers' instruction count - about 60 vector
// instructions per step and thread.  Stepping the decoded index by additions instead of decoding it with
// integer multiplications was measured: no fewer instructions, no faster.  Tiles of 64 x 128 and 128 x 64 (two
// workgroups per compute unit) were measured too: no faster.  LDS holds both operands k-major ([k][row]) so that the 16 lanes sharing a k read
// 16 consecutive doubles.  One workgroup per (tile, reduction range).
#ifndef IGCONV_KERNEL_F64_HPP_
#define IGCONV_KERNEL_F64_HPP_

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "igconv_params.h"

namespace igc {

typedef double f64x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kF64BK = 16;
constexpr int kF64Threads = 512;
constexpr int f64_lds_bytes(int nb) { return 2 * kF64BK * (64 * nb + 4) * 8; }
constexpr uint32_t kF64OutOfRange = 0x80000000u;   // a byte offset no buffer reaches: reads as zero

__device__ __forceinline__ uint32_t f64_mdiv(uint32_t n, Magic m) { return (__umulhi(n, m.mul) + n) >> m.shift; }

__device__ __forceinline__ double f64_load(__amdgpu_buffer_rsrc_t buf, uint32_t byte_off) {
    const u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(buf, byte_off, 0, 0);
    return __builtin_bit_cast(double, v);
}

// WGRAD: the reduction index moves the window by (i1*redMulH, i2*redMulW) (backward filter);
// otherwise by the tap (i1, i2) itself, reversed when p.flip is set.
// (64 registers: four workgroups per compute unit)
template <bool WGRAD, int NB>
__global__ __launch_bounds__(kF64Threads) __attribute__((amdgpu_waves_per_eu(8, 8))) void igconv_f64_kernel(const ConvKernelParams p) {
    constexpr int BM = 32 * NB, BN = 32 * NB, BK = kF64BK;
    constexpr int KPT = BK * BM / 256;   // consecutive reduction indices per thread and operand
    constexpr int ALD = BM + 2;          // row stride of As: the 16 lanes that write one row of A land in 16 banks
    constexpr int ROWS = BM / 16;        // rows of A per thread
    constexpr int BLD = BN + 2;          // the same for Bs (backward filter writes it with lanes along the reduction too)
    __shared__ double As[2][BK][ALD];
    __shared__ double Bs[2][BK][BLD];

    const int tid = threadIdx.x & 255, lane = tid & 63, wave = tid >> 6;
    const bool mover = threadIdx.x >= 256;
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

    // ---- B role.  Forward / backward data: one column, KPT consecutive reduction indices per step (lanes along
    // the columns, which are contiguous in the image).  Backward filter: one reduction index - the A role's -
    // and the columns b_col0 + 16 e: there the reduction (n, p, q) is what is contiguous in the image, and 16
    // lanes along it read one or two cache lines where lanes along (c, r, s) touched a line per filter row.
    const int b_col = WGRAD ? (tid >> 4) : (tid & (BN - 1)), b_kq = WGRAD ? (tid & 15) : (tid / BN) * KPT;
    constexpr int BCOLS = WGRAD ? BN / 16 : 1;
    static_assert(BN / 16 == KPT, "one register per column (backward filter) or per reduction index");
    bool b_ok = false;
    int b_base = 0, b_h0 = 0, b_w0 = 0;
    int c_base[BCOLS], c_h0[BCOLS], c_w0[BCOLS];
#pragma unroll
    for (int e = 0; e < BCOLS; ++e) {
        const int j = n0 + b_col + 16 * e;
        const bool ok = j < p.NPQ;
        const uint32_t jj = ok ? (uint32_t)j : 0u;
        const uint32_t j0 = f64_mdiv(jj, p.mPQ), rem = jj - j0 * (uint32_t)p.PQ;
        const uint32_t j1 = f64_mdiv(rem, p.mQ), j2 = rem - j1 * (uint32_t)p.Q;
        const int h0 = (int)j1 * p.u - p.pad_h, w0 = (int)j2 * p.v - p.pad_w;
        if (WGRAD) {
            c_h0[e] = ok ? h0 : -(1 << 30);   // (a column past the end fails every window test)
            c_w0[e] = w0;
            c_base[e] = (int)j0 * p.xsN + h0 * p.xsH + w0 * p.xsW;
        } else {
            b_ok = ok;
            b_base = (int)j0 * p.xsN;
            b_h0 = h0;
            b_w0 = w0;
        }
    }
    // ---- A role: one reduction index per step (lanes along the reduction: where A is
    // contiguous in it, 16 lanes read one 128-byte line), rows a_row0 + 16 e
    const int a_k = tid & 15, a_row0 = tid >> 4;

    // Steps past the end of this range load nothing (a buffer load with its offset out of range brings zero).
    const int k_end = min(p.CRS, s_end * BK);

    auto fetch = [&](int step, double (&a_reg)[ROWS], double (&b_reg)[KPT]) {
        if (WGRAD) {   // B, lanes along the reduction
            // (A reduction index past the end moves the window out of the image: one select per step.  Tested
            // per element, the compiler turned the test into branches around the loads, with waits for every
            // outstanding load inside them.)
            const uint32_t k = (uint32_t)(step * BK + b_kq);
            const uint32_t i0 = f64_mdiv(k, p.mRS), rem = k - i0 * (uint32_t)p.RS;
            const uint32_t i1 = f64_mdiv(rem, p.mS), i2 = rem - i1 * (uint32_t)p.S;
            const int dh0 = (int)i1 * p.redMulH, dw = (int)i2 * p.redMulW;
            const int kterm = (int)i0 * p.xsC + dh0 * p.xsH + dw * p.xsW;
            const int dh = (int)k < k_end ? dh0 : -(1 << 29);
#pragma unroll
            for (int e = 0; e < BCOLS; ++e) {
                const bool ok = (uint32_t)(c_h0[e] + dh) < (uint32_t)p.H && (uint32_t)(c_w0[e] + dw) < (uint32_t)p.W;
                b_reg[e] = f64_load(xbuf, ok ? (uint32_t)(c_base[e] + kterm) * 8u : kF64OutOfRange);
            }
        } else {   // B, lanes along the columns
            const uint32_t k0 = (uint32_t)(step * BK + b_kq);
            uint32_t i0 = f64_mdiv(k0, p.mRS), rem = k0 - i0 * (uint32_t)p.RS;
            uint32_t i1 = f64_mdiv(rem, p.mS), i2 = rem - i1 * (uint32_t)p.S;
#pragma unroll
            for (int e = 0; e < KPT; ++e) {
                int dh, dw;
                if (WGRAD) {
                    dh = (int)i1 * p.redMulH;
                    dw = (int)i2 * p.redMulW;
                } else {
                    dh = p.flip ? p.R - 1 - (int)i1 : (int)i1;
                    dw = p.flip ? p.S - 1 - (int)i2 : (int)i2;
                }
                const int h = b_h0 + dh, w = b_w0 + dw;
                const bool ok = b_ok && (int)(k0 + e) < k_end && (uint32_t)h < (uint32_t)p.H && (uint32_t)w < (uint32_t)p.W;
                const uint32_t off = (uint32_t)(b_base + (int)i0 * p.xsC + h * p.xsH + w * p.xsW) * 8u;
                b_reg[e] = f64_load(xbuf, ok ? off : kF64OutOfRange);
                ++i2; ++rem;
                if (i2 == (uint32_t)p.S) { i2 = 0; ++i1; }
                if (rem == (uint32_t)p.RS) { rem = 0; i1 = 0; i2 = 0; ++i0; }
            }
        }
        {   // A
            const uint32_t k = (uint32_t)(step * BK + a_k);
            const uint32_t i0 = f64_mdiv(k, p.mRS), rem = k - i0 * (uint32_t)p.RS;
            const uint32_t i1 = f64_mdiv(rem, p.mS), i2 = rem - i1 * (uint32_t)p.S;
            const int koff = p.wTap0 + (int)i0 * p.wsRed + (int)i1 * p.wsTapR + (int)i2 * p.wsTapS;
            const uint32_t k_bit = (int)k < k_end ? 0u : kF64OutOfRange;   // (or-ed in: no branch to form)
#pragma unroll
            for (int e = 0; e < ROWS; ++e) {
                const int m = m0 + a_row0 + 16 * e;
                const uint32_t off = (uint32_t)(m * p.wsRow + koff) * 8u;
                a_reg[e] = f64_load(wbuf, (m < p.K ? off : kF64OutOfRange) | k_bit);
            }
        }
    };
    auto stage = [&](int buf, const double (&a_reg)[ROWS], const double (&b_reg)[KPT]) {
#pragma unroll
        for (int e = 0; e < ROWS; ++e) As[buf][a_k][a_row0 + 16 * e] = a_reg[e];
#pragma unroll
        for (int e = 0; e < KPT; ++e) {
            if (WGRAD)
                Bs[buf][b_kq][b_col + 16 * e] = b_reg[e];
            else
                Bs[buf][b_kq + e][b_col] = b_reg[e];
        }
    };

    // Both kinds of wavefront meet at one barrier before the first step and at one after every step; an odd
    // number of steps is rounded up (the extra step multiplies zeros: k_end).
    const int nsteps = (max(s_end - s_begin, 0) + 1) & ~1;
    if (mover) {
        double a0[ROWS], b0[KPT], a1[ROWS], b1[KPT];
        fetch(s_begin, a0, b0);
        fetch(s_begin + 1, a1, b1);
        stage(0, a0, b0);
        __syncthreads();
        // (enter the loop with no load outstanding: merging this path with the loop's back edge, the compiler
        // otherwise waits for every load at the top of each step)
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
        __builtin_amdgcn_sched_barrier(0);
        for (int i = 0; i < nsteps; i += 2) {
            // while buffer 0 is multiplied (step i): request step i + 2, stage step i + 1
            fetch(s_begin + i + 2, a0, b0);
            __builtin_amdgcn_sched_barrier(0);   // (requests first: otherwise they are issued behind the wait)
            stage(1, a1, b1);
            __syncthreads();
            // while buffer 1 is multiplied (step i + 1): request step i + 3, stage step i + 2
            fetch(s_begin + i + 3, a1, b1);
            __builtin_amdgcn_sched_barrier(0);
            stage(0, a0, b0);
            __syncthreads();
        }
        return;
    }

    f64x4 acc[NB][NB];
#pragma unroll
    for (int bi = 0; bi < NB; ++bi)
#pragma unroll
        for (int bj = 0; bj < NB; ++bj) acc[bi][bj] = f64x4{0.0, 0.0, 0.0, 0.0};

    __syncthreads();
    int cur = 0;
    for (int i = 0; i < nsteps; ++i) {
#pragma unroll
        for (int kg = 0; kg < BK / 4; ++kg) {
            const int kk = kg * 4 + lq;
            double av[NB], bv[NB];
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                av[b] = As[cur][kk][wm * (16 * NB) + b * 16 + l16];
                bv[b] = Bs[cur][kk][wn * (16 * NB) + b * 16 + l16];
            }
#pragma unroll
            for (int bi = 0; bi < NB; ++bi)
#pragma unroll
                for (int bj = 0; bj < NB; ++bj)
                    acc[bi][bj] = __builtin_amdgcn_mfma_f64_16x16x4f64(av[bi], bv[bj], acc[bi][bj], 0, 0, 0);
        }
        __syncthreads();
        cur ^= 1;
    }

    // ---- epilogue: lane (l16, lq), value v of block (bi, bj) is row 4*v + lq, column l16
    const double alpha = p.alpha64, beta = p.beta64;
#pragma unroll
    for (int bj = 0; bj < NB; ++bj) {
        const int col = n0 + wn * (16 * NB) + bj * 16 + l16;
        if (col >= p.NPQ) continue;
        const uint32_t j0 = f64_mdiv((uint32_t)col, p.mPQ), rem = (uint32_t)col - j0 * (uint32_t)p.PQ;
        const uint32_t j1 = f64_mdiv(rem, p.mQ), j2 = rem - j1 * (uint32_t)p.Q;
        const int ycol = (int)j0 * p.ysN + (int)j1 * p.ysP + (int)j2 * p.ysQ;
#pragma unroll
        for (int bi = 0; bi < NB; ++bi)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = m0 + wm * (16 * NB) + bi * 16 + 4 * v + lq;
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
