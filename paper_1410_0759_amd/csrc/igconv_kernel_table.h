// Table of compiled kernel variants and the host-side launcher.  Internal.
#ifndef IGCONV_KERNEL_TABLE_H_
#define IGCONV_KERNEL_TABLE_H_

#include "igconv_params.h"

namespace igc {

struct KernelInfo {
    const char *name;
    bool bf16;      // input data type: bfloat16 (else float)
    int BM, BN, BK; // tile of O_m per workgroup and reduction elements per step
    bool swap;      // lanes run along output channels in the epilogue
    bool veca;      // filter rows fetched with 16-byte loads (needs CRS % VEC == 0, aligned w)
    int gmode;      // gather mode: 0 generic, 1 tap-major reduction order, 2 unpadded, 3 nine-tap table,
                    // 4 channel vectors (bf16, nine taps, unit channel stride), 5 the same from a staged image patch,
                    // 6 backward-filter (generic gather, roles of columns and reduction exchanged),
                    // 7 unpadded with the tap offsets in an LDS table (short reductions),
                    // 8 backward-filter with columns (tap, channel), one tap per tile,
                    // 9 backward-filter without padding, few channels,
                    // 11 mode 7 with a last step of half the k-groups,
                    // 13 mode 7 for an odd number of steps (the step that rounds the count up is not multiplied),
                    // 12 1x1 filters over channel vectors (bf16, unit channel stride): both operands loaded as they are,
                    // 10 backward-filter over channel vectors (bf16, unit channel strides), tiles transposed in registers,
                    // 14 filter order with the tap tracked by the scalar unit and the window test in a bit mask (R*S <= 63)
                    // 15 unpadded, 32 x 32 tiles, the reduction cut among the wavefronts, operands straight from global memory
                    // 16 mode 15 with a zero border: the window test from a mask with a bit per tap (R*S <= 31)
    int threads;
    int ldsBytes;
    // Enqueue on `stream` (a hipStream_t); returns the runtime's error code (0 = ok).
    int (*launch)(const ConvKernelParams &, int grid, void *stream);
    int variant = 0;  // 1: (gather modes 15, 16) the filter rows staged in LDS;
                      // 2: `threads` / 256 teams of four wavefronts per workgroup, each on its share of the steps;
                      // 3: wavefronts that move tiles beside wavefronts that multiply (gather mode 5)
    bool f64 = false; // double precision in and out (alpha64 / beta64 of the parameters apply)
    int patchPixels = 512;  // gather mode 5: pixels of the zero-extended image a tile's staged patch can hold
};

struct KernelGroup {
    const KernelInfo *kernels;
    int count;
};

// One group per translation unit of kernel instantiations.
extern const KernelGroup kGroupF32Taps9, kGroupF32TapMajor, kGroupF32Nopad, kGroupF32Generic, kGroupF32Swap, kGroupBF16,
    kGroupBF16Channels, kGroupWgrad, kGroupF64, kGroupWgradBF16Channels, kGroupBF16Pointwise, kGroupF32Teams, kGroupF32Masked, kGroupF64Masked, kGroupF32Direct;

// Adds up `count` partial results (`stride` floats apart) into out = alpha*sum + beta*out;
// returns the runtime's error code.
int launch_sum_parts(const float *parts, float *out, uint32_t n, int count, uint32_t stride, float alpha, float beta,
                     void *stream);

// wt[c][k][t] = w[k][c][t] for 2-byte elements, t < taps, taps 9 or 1 (the filter with its first two
// dimensions exchanged, each pair's taps kept in order); returns the runtime's error code.
int launch_filter_exchange(const void *w, void *wt, int K, int C, int taps, void *stream);

// wt[k][t][c] = w[k][c][t] for elements of 4 or 2 bytes (t < RS), or with `exchange` wt[c][t][k]: the filter as the
// tap-major kernels like to read it in the forward pass resp. in backward data.  mInner: the divisor C resp. K.
int launch_filter_taps_outer(const void *w, void *wt, int elem_bytes, int K, int C, int RS, bool exchange, Magic mInner, Magic mRS,
                             void *stream);

// xp = x with its zero border written out, packed N,C,H+2pad_h,W+2pad_w (float; x read through the strides xs).
int launch_pad_image(const float *x, float *xp, int N, int C, int H, int W, int pad_h, int pad_w, const long long xs[4], Magic mWp,
                     Magic mHp, Magic mC, void *stream);

// Backward data of a strided layer with few channels as one forward pass (see igconv_kernels_wgrad.hip): the
// filter of that pass, f[(a*v + b)*C + c][k][Rp][Sp], and the move of its result y' (N, u*v*C, I, J, packed)
// to dx = alpha * y'(...) + beta * dx.  The divisors are the launch-time multiply+shift forms of the named sizes.
int launch_pack_phase_filter(const float *w, float *f, int K, int C, int R, int S, int u, int v, int Rp, int Sp, bool flip,
                             Magic mSp, Magic mRp, Magic mK, Magic mC, Magic mv, void *stream);
int launch_phase_scatter(const float *y, float *dx, int N, int C, int H, int W, int I, int J, int u, int v, int pad_h, int pad_w,
                         const long long dxs[4], Magic mW, Magic mH, Magic mC, Magic mu, Magic mv, float alpha, float beta,
                         void *stream);

// The same for the channel-vector backward-filter kernels, whose parts are stored as [tap][row position][column
// position] (KP x CP positions per tap, tiles of BM x BN): see igconv_kernel_wgrad_bf16c.hpp.
int launch_sum_positions(const float *parts, float *out, uint32_t n, int count, uint32_t stride, float alpha, float beta, int C,
                         int RS, int BM, int BN, int KP, int CP, void *stream);
int launch_sum_parts_f64(const double *parts, double *out, uint32_t n, int count, uint32_t stride, double alpha, double beta,
                         void *stream);

// Compute units of the current device, 0 when the runtime finds none (igconv_probe.hip).
int query_compute_units();

int kernel_count();
const KernelInfo *kernel_info(int id);  // nullptr when out of range

}  // namespace igc
#endif
