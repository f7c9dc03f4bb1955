// Backward filter for bf16 tensors whose channels are contiguous (x and dy with unit channel
// stride), paper Section 2.1.1 (the backward forms are products of the same kind):
//
//   dw[k, c, r, s] = sum over pixels i = (n,p,q) of dy[i][k] * x[pixel(i) + tap(r,s)][c]
//
// rows k, columns c of ONE tap per tile, reduction over the pixels.  Both operands have the
// reduction index as their SLOW dimension in memory (a pixel holds its channels
// contiguously), while v_mfma_f32_32x32x16_bf16 wants 8 consecutive reduction elements per
// lane.  So the tiles are transposed on their way into LDS: a thread loads the 16-byte
// channel vectors (8 channels) of 8 consecutive pixels - 16 neighbouring lanes read 256
// contiguous bytes of one pixel -, transposes the 8 x 8 block of 16-bit values in registers
// (32 v_perm_b32) and writes 8 rows of "8 pixels of one channel" (16 bytes each).
//
// LDS: [stage][row position][64 pixels + 8 of padding]; the row position of channel
// cv*8 + ch (cv: 16-byte vector, ch: channel in it) is ch*(rows/8) + cv, so that the 16
// lanes writing one ch land in 16 consecutive rows (row stride 9 x 16 bytes: all banks once)
// and an MFMA block reads 32 consecutive rows.  MFMA row i of block b therefore stands for
// the channel at position 32 b + i; the epilogue undoes that.
//
// The byte offset of a pixel in dy and in x (tap added, zero border and range end folded in
// as an out-of-range offset) is the same for every channel, so one wavefront per operand
// computes the 64 offsets of a step, one pixel per lane, two steps ahead, into a small LDS
// table; the loading threads fetch their 8 offsets with two 16-byte LDS reads.
//
// A workgroup has eight wavefronts: four movers (the 256 loading threads above, one 8 x 8 block each per operand
// and step) and four multipliers that only read fragments and issue MFMAs; they meet at one barrier per step, the
// movers filling the LDS stage the multipliers read next.
//
// One workgroup per (tile, reduction range).  With a workspace the results are stored in
// the order the accumulators have them, [range][tap][row position][column position] padded
// to whole tiles (32 lanes write 128 contiguous bytes), and igconv_sum_positions_kernel adds
// the ranges in order while it moves the sums to dw[k][c][r][s]; dw itself has one tap's
// elements 4*R*S bytes apart, and writing it from here (no workspace) costs as much as the
// whole reduction.
#ifndef IGCONV_KERNEL_WGRAD_BF16C_HPP_
#define IGCONV_KERNEL_WGRAD_BF16C_HPP_

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "igconv_params.h"

namespace igc {

typedef float wg_f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 wg_bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t wg_u32x4 __attribute__((ext_vector_type(4)));

constexpr int kWgcBK = 64;                    // pixels per step
constexpr int kWgcRowBytes = kWgcBK * 2 + 16; // LDS row: 64 pixels + padding to an odd number of 16-byte units
constexpr uint32_t kWgcOutOfRange = 0x80000000u;

template <int BM_, int BN_>
struct WgradBf16cConfig {
    static constexpr int BM = BM_, BN = BN_, BK = kWgcBK;
    // Eight wavefronts: four that only read operand fragments from LDS and issue MFMAs, four that load, transpose and
    // write the tiles of the steps ahead (as in igconv_kernel_bf16s.hpp).  A wavefront issues in order: with the loads,
    // 32 permutes and LDS writes of a step in the same stream as its 16 MFMAs the MFMA pipe waited for them (the bf16
    // workload: 54 -> 49 us, 306 -> 277 at a mini-batch of 256; every tile shape gained).
    static constexpr int THREADS = 512;
    static constexpr int STAGE_BYTES = (BM + BN) * kWgcRowBytes;
    static constexpr int TABLE_BYTES = 2 * 4 * kWgcBK * 4;   // [slot][wavefront][pixel]: wavefronts 0, 1 hold dy's and x's offsets
    static constexpr int LDS_BYTES = 2 * STAGE_BYTES + TABLE_BYTES;
    static_assert(BM % 64 == 0 && BN % 64 == 0 && BM + BN <= 256, "one 8x8 block per thread");
    // (with BM + BN < 256 the last wavefronts repeat blocks of the x operand: same loads, same values written)
};

__device__ __forceinline__ uint32_t wgc_mdiv(uint32_t n, Magic m) { return (__umulhi(n, m.mul) + n) >> m.shift; }

template <class Cfg>
__global__ __launch_bounds__(Cfg::THREADS) void igconv_wgrad_bf16c_kernel(const ConvKernelParams p) {
    constexpr int BM = Cfg::BM, BN = Cfg::BN, BK = Cfg::BK;
    constexpr int MB = BM / 64, NB = BN / 64;      // 32x32 blocks per wavefront (2 x 2 wavefronts)
    constexpr int RB = kWgcRowBytes;
    __shared__ __attribute__((aligned(16))) uint8_t lds[Cfg::LDS_BYTES];
    uint32_t *const table = reinterpret_cast<uint32_t *>(lds + 2 * Cfg::STAGE_BYTES);   // [2][4][64]

    const int lane = threadIdx.x & 63;
    const int wave_all = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    // wavefronts 0-3 multiply, 4-7 move; both kinds number themselves 0-3 (and the moving threads 0-255)
    const bool mover = wave_all >= 4;
    const int wave = wave_all & 3;
    const int tid = (int)threadIdx.x & 255;
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, half = lane >> 5;

    // (tile, range): numbered in contiguous ranges per XCD
    const int tiles = p.tilesM * p.tilesN;
    const int item = (int)(blockIdx.x % 8u) * p.tilesPerXcd + (int)(blockIdx.x / 8u);
    if (item >= tiles * p.splits) return;
    const int split = item / tiles, tile = item - split * tiles;
    const int m0 = (tile % p.tilesM) * BM;
    // column tile -> (tap, channel block): PQ = channel blocks per tap, Q and R the filter's S and R
    const uint32_t tn = (uint32_t)(tile / p.tilesM);
    const uint32_t tap = wgc_mdiv(tn, p.mPQ);
    const uint32_t tr = wgc_mdiv(tap, p.mQ), ts = tap - tr * (uint32_t)p.Q;
    const int tap_h = (int)(p.flip ? (uint32_t)p.R - 1u - tr : tr) - p.pad_h;
    const int tap_w = (int)(p.flip ? (uint32_t)p.Q - 1u - ts : ts) - p.pad_w;
    const int n0 = (int)(tn - tap * (uint32_t)p.PQ) * BN;
    const int s_begin = split * p.stepsPerSplit, s_end = min(p.ksteps, s_begin + p.stepsPerSplit);

    const __amdgpu_buffer_rsrc_t xbuf = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p.x), 0, p.x_bytes, 0x00020000u);
    const __amdgpu_buffer_rsrc_t dybuf = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p.w), 0, p.w_bytes, 0x00020000u);
    const __amdgpu_buffer_rsrc_t ybuf = __builtin_amdgcn_make_buffer_rsrc(
        static_cast<uint8_t *>(p.y) + (size_t)split * p.ySplitBytes, 0, p.y_bytes, 0x00020000u);

    // ---- offsets of the 64 pixels of a step: wavefront 0 for dy, wavefront 1 for x, one pixel per lane.
    // (Wavefronts 2 and 3 do the same into slots nobody reads: the loop stays free of branches, which
    // keeps the compiler from waiting for all outstanding loads at block boundaries.)
    const bool table_dy = (wave & 1) == 0;
    auto fill_table = [&](int step) {
        const uint32_t i = (uint32_t)step * BK + (uint32_t)lane;
        const uint32_t n = wgc_mdiv(i, p.mRS), rem = i - n * (uint32_t)p.RS;
        const uint32_t pp = wgc_mdiv(rem, p.mS), qq = rem - pp * (uint32_t)p.S;
        const bool live = i < (uint32_t)p.CRS && step < s_end;
        const uint32_t hh = table_dy ? pp : pp * (uint32_t)p.redMulH + (uint32_t)tap_h;   // (wraps below zero: fails the test)
        const uint32_t ww = table_dy ? qq : qq * (uint32_t)p.redMulW + (uint32_t)tap_w;
        const bool ok = live && (table_dy || (hh < (uint32_t)p.H && ww < (uint32_t)p.W));
        const uint32_t sn = table_dy ? (uint32_t)p.wsRed : (uint32_t)p.xsC, sh = table_dy ? (uint32_t)p.wsTapR : (uint32_t)p.xsH,
                       sw = table_dy ? (uint32_t)p.wsTapS : (uint32_t)p.xsW;
        table[((step & 1) * 4 + wave) * BK + lane] = ok ? (n * sn + hh * sh + ww * sw) * 2u : kWgcOutOfRange;
    };

    // ---- loading role: thread -> (operand, channel vector cv, pixel group pg)
    const bool role_a = wave < BM / 64;      // (uniform over a wavefront: the buffer descriptor is chosen by a scalar select)
    const int blk = role_a ? tid : (tid - BM) % BN;
    constexpr int NVA = BM / 8, NVB = BN / 8;
    const int cv = role_a ? blk % NVA : blk % NVB;
    const int pg = role_a ? blk / NVA : blk / NVB;     // 0..7
    // byte offset of the channel vector inside a pixel; out of range when the tile overhangs K resp. C
    const int ch0 = (role_a ? m0 : n0) + cv * 8;
    const uint32_t vec_off = ch0 < (role_a ? p.K : p.NPQ) ? (uint32_t)ch0 * 2u : kWgcOutOfRange;
    // LDS: row position of channel (cv, ch) is ch*NV + cv (B rows follow the BM rows of A)
    const int row0 = role_a ? cv : BM + cv;
    const int row_step = role_a ? NVA : NVB;

    // two register sets: the loads of step t go to set (t - first step) & 1
    wg_u32x4 ld0[8], ld1[8];
    auto fetch = [&](int step, wg_u32x4 (&ld)[8]) {
        const uint32_t *t = table + ((step & 1) * 4 + (role_a ? 0 : 1)) * BK + pg * 8;
        const wg_u32x4 o0 = *reinterpret_cast<const wg_u32x4 *>(t), o1 = *reinterpret_cast<const wg_u32x4 *>(t + 4);
        const uint32_t offs[8] = {o0[0], o0[1], o0[2], o0[3], o1[0], o1[1], o1[2], o1[3]};
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            // (either part out of range keeps the sum at or above 2^31: reads as zero)
            const uint32_t off = (offs[j] | vec_off) >= kWgcOutOfRange ? kWgcOutOfRange : offs[j] + vec_off;
            ld[j] = __builtin_amdgcn_raw_buffer_load_b128(role_a ? dybuf : xbuf, off, 0, 0);
        }
    };
    // 8 pixels x 8 channels -> 8 channels x 8 pixels, one 16-byte LDS row piece per channel
    auto stage = [&](int buf, const wg_u32x4 (&ld)[8]) {
        uint8_t *base = lds + buf * Cfg::STAGE_BYTES + pg * 16;
#pragma unroll
        for (int ch = 0; ch < 8; ++ch) {
            const uint32_t sel = (ch & 1) ? 0x07060302u : 0x05040100u;
            wg_u32x4 o;
#pragma unroll
            for (int pp = 0; pp < 4; ++pp) o[pp] = __builtin_amdgcn_perm(ld[2 * pp + 1][ch >> 1], ld[2 * pp][ch >> 1], sel);
            *reinterpret_cast<wg_u32x4 *>(base + (row0 + ch * row_step) * RB) = o;
        }
    };

    wg_f32x16 acc[MB][NB];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // ---- pipeline: global loads two steps ahead (their transposition into LDS, one step later, then never waits), offset
    // table three steps ahead.  In step s the multipliers compute from LDS stage `cur` while the movers put the loaded
    // data of step s+1 into the other stage and request step s+2; one barrier per step for all eight wavefronts.  Past
    // the range's end the table holds out-of-range offsets, so the extra step of an odd range and the look-ahead load zeros.
    if (mover) {
        auto move = [&](int s, int cur, wg_u32x4 (&ld_new)[8], const wg_u32x4 (&ld_next)[8]) {
            fetch(s + 2, ld_new);
            fill_table(s + 3);
            stage(cur ^ 1, ld_next);
            __syncthreads();
        };
        fill_table(s_begin);
        fill_table(s_begin + 1);
        __syncthreads();
        fetch(s_begin, ld0);
        fetch(s_begin + 1, ld1);
        __syncthreads();
        fill_table(s_begin + 2);
        stage(0, ld0);
        __syncthreads();
        for (int s = s_begin; s < s_end; s += 2) {
            move(s, 0, ld0, ld1);
            move(s + 1, 1, ld1, ld0);
        }
        return;
    } else {
        auto multiply = [&](int cur) {
            const uint8_t *a_base = lds + cur * Cfg::STAGE_BYTES + (wm * (BM / 2) + l32) * RB + half * 16;
            const uint8_t *b_base = lds + cur * Cfg::STAGE_BYTES + (BM + wn * (BN / 2) + l32) * RB + half * 16;
#pragma unroll
            for (int ks = 0; ks < BK / 16; ++ks) {
                wg_bf16x8 av[MB], bv[NB];
#pragma unroll
                for (int i = 0; i < MB; ++i) av[i] = *reinterpret_cast<const wg_bf16x8 *>(a_base + i * 32 * RB + ks * 32);
#pragma unroll
                for (int j = 0; j < NB; ++j) bv[j] = *reinterpret_cast<const wg_bf16x8 *>(b_base + j * 32 * RB + ks * 32);
#pragma unroll
                for (int i = 0; i < MB; ++i)
#pragma unroll
                    for (int j = 0; j < NB; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[i], bv[j], acc[i][j], 0, 0, 0);
            }
            __syncthreads();
        };
        __syncthreads();
        __syncthreads();
        __syncthreads();
        for (int s = s_begin; s < s_end; s += 2) {
            multiply(0);
            multiply(1);
        }
    }

    // ---- epilogue.  Workspace (ysN != 0): [tap][row position][column position], ysP x ysK positions per tap.
    if (p.ysN != 0) {
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            const uint32_t col = (uint32_t)(n0 + wn * (BN / 2) + j * 32 + l32);
#pragma unroll
            for (int i = 0; i < MB; ++i)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const uint32_t row = (uint32_t)(m0 + wm * (BM / 2) + i * 32 + 8 * (v / 4) + 4 * half + (v % 4));
                    const uint32_t off = ((tap * (uint32_t)p.ysP + row) * (uint32_t)p.ysK + col) * 4u;
                    // (alpha is 1 here; the product keeps the store's source in an ordinary vector register -
                    // storing the accumulator element directly was compiled into 16 stores of element 0)
                    const float r = p.alpha * acc[i][j][v];
                    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, r), ybuf, off, 0, 0);
                }
        }
        return;
    }
    // Straight into dw[k*ysK + c*ysQ + tap]; MFMA row/column index -> channel through the LDS row positions
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        const int posc = wn * (BN / 2) + j * 32 + l32;
        const int c = n0 + (posc % NVB) * 8 + posc / NVB;
        if (c >= p.NPQ) continue;
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int posr = wm * (BM / 2) + i * 32 + 8 * (v / 4) + 4 * half + (v % 4);
                const int k = m0 + (posr % NVA) * 8 + posr / NVA;
                if (k >= p.K) continue;
                const uint32_t off = ((uint32_t)k * (uint32_t)p.ysK + (uint32_t)c * (uint32_t)p.ysQ + tap) * 4u;
                float r = p.alpha * acc[i][j][v];
                if (p.beta != 0.f) r += p.beta * __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(ybuf, off, 0, 0));
                __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, r), ybuf, off, 0, 0);
            }
    }
}

}  // namespace igc
#endif
