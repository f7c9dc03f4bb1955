// Launch-time constants handed from the host part of the library to the kernels.
// Internal to the library (not part of the C ABI).
#ifndef IGCONV_PARAMS_H_
#define IGCONV_PARAMS_H_

#include <stdint.h>

namespace igc {

// floor(n / d) for 0 <= n < 2^31 as (umulhi(n, mul) + n) >> shift: division by a
// launch-time constant turned into multiply + shift (paper, Section 3.1, last
// paragraph).  shift = ceil(log2 d), mul = ceil(2^(32+shift) / d) - 2^32.
struct Magic {
    uint32_t mul;
    uint32_t shift;
};

// (mul, shift) for a divisor 1 <= d < 2^31; false outside that range.  Host code.
inline bool magic_for(uint32_t d, Magic *m) {
    if (d < 1u || d >= (1u << 31)) return false;
    uint32_t shift = 0;
    while ((1ull << shift) < d) ++shift;  // ceil(log2 d)
    const unsigned __int128 one = 1;
    const unsigned __int128 q = ((one << (32 + shift)) + d - 1) / d;  // ceil(2^(32+shift) / d), in [2^32, 2^33)
    m->mul = (uint32_t)(q - (one << 32));
    m->shift = shift;
    return true;
}

// The kernels that feed the MFMAs straight from global memory (igconv_kernel_f32d.hpp): entries of their LDS table of
// tap offsets (one per reduction index), and how many steps ahead their requests run (as many register sets).
constexpr int kDirectTableEntries = 16384;
constexpr int direct_depth(int bk, bool staged_rows = false) { return staged_rows ? 4 : (bk >= 32 ? 2 : 3); }   // (bk: reduction indices per step)

struct ConvKernelParams {
    const void *x;   // input tensor D (device)
    const void *w;   // filters F, packed K,C,R,S (device)
    void *y;         // output tensor O (device)
    uint32_t x_bytes, w_bytes, y_bytes;  // extents, used as buffer-descriptor limits
    int32_t N, C, H, W, K, R, S, P, Q;
    int32_t pad_h, pad_w, u, v;
    int32_t flip;    // 1: eq. 2 (tap r reads row R-1-r), 0: cross-correlation
    int32_t CRS, NPQ, PQ, RS;
    Magic mPQ, mQ, mRS, mS;
    int32_t xsN, xsC, xsH, xsW;  // element strides of x
    int32_t ysN, ysK, ysP, ysQ;  // element strides of y
    float alpha, beta;
    double alpha64 = 0.0, beta64 = 0.0;   // the same for the double-precision kernels
    const float *bias = nullptr;   // K floats added per output feature map before the activation, or null
    int32_t act = -1;    // activation applied last: 0 sigmoid, 1 rectified linear, 2 tanh, -1 none
    int32_t tilesM, tilesN;
    int32_t tilesPerXcd;  // ceil(tilesM * tilesN / 8): tiles are dealt to the 8 XCDs in contiguous ranges
    int32_t wgsPerXcd;    // workgroups launched per XCD (grid = 8 * wgsPerXcd); each takes every wgsPerXcd-th tile of its range
    int32_t ksteps;  // reduction steps of the chosen kernel (depends on its reduction order)
    int32_t tail_step;  // first step in which the reduction range ends inside the step, else -1
    // Where the filter element (row m, reduction channel c, tap (r,s)) lives, in elements:
    // m*wsRow + c*wsRed + wTap0 + r*wsTapR + s*wsTapS (tap-major kernels only; the others
    // read the packed K,C,R,S order directly).  Forward: (C*R*S, R*S, 0, S, 1).  Backward-data
    // exchanges the roles of k and c and walks a subset of the taps backwards.
    // Backward-filter reuses them for its first operand dy[n,k,p,q]: row (k) stride wsRow, and
    // n, p, q strides in wsRed, wsTapR, wsTapS.
    int32_t wsRow, wsRed, wTap0, wsTapR, wsTapS;
    // Backward-filter: window coordinates of reduction index (n,p,q) are (p*redMulH, q*redMulW);
    // the reduction is cut into `splits` ranges of stepsPerSplit (even) steps, range s writing
    // its result at y + s*ySplitBytes.
    int32_t redMulH, redMulW, splits, stepsPerSplit;
    uint32_t ySplitBytes;
    // zero-extended image: Wp = W + 2 pad_w pixels per row, HpWp = (H + 2 pad_h) * Wp per image
    int32_t Wp, HpWp;
    Magic mWp, mHpWp;
};

}  // namespace igc
#endif
