// Forward convolution with 1x1 filters for bf16 tensors whose channels are contiguous in x
// (paper, Section 3: with R = S = 1 the lowered matrix D_m is x itself, read through strides):
//
//   y[n,k,p,q] = sum_c w[k][c] * x[n, p*u - pad_h, q*v - pad_w, c]
//
// a plain product of two operands that are both contiguous along the reduction (the filter
// row of k, the channel vector of a pixel), so both go to LDS as they are loaded, 16 bytes =
// 8 channels per load, 8 neighbouring lanes reading 128 contiguous bytes of one row.
// Tile BM x BN x 64 channels, 2 x 2 wavefronts, v_mfma_f32_32x32x16_bf16; LDS rows of
// 64 channels + 16 bytes (an odd number of 16-byte units: conflict-free 16-byte accesses);
// global loads two steps ahead in two register sets, one barrier per step; moving and multiplying wavefronts apart.  Persistent workgroups whose loads run on across the tile boundary.  The epilogue is the shared one (alpha/beta, bias,
// activation, either orientation of the output).
#ifndef IGCONV_KERNEL_BF16_PW_HPP_
#define IGCONV_KERNEL_BF16_PW_HPP_

#include "igconv_kernel.hpp"

namespace igc {

constexpr int kPwBK = 64;                     // channels per step
constexpr int kPwRowBytes = kPwBK * 2 + 16;

template <int BM_, int BN_, bool SWAP_>
struct Bf16PwConfig {
    static constexpr int BM = BM_, BN = BN_, BK = kPwBK;
    static constexpr bool SWAP = SWAP_;
    // eight wavefronts: four that load the tiles of the steps ahead and write them to LDS, four that read fragments and
    // issue MFMAs (and store the finished tile); one barrier per step
    static constexpr int THREADS = 512;
    static constexpr int STAGE_BYTES = (BM + BN) * kPwRowBytes;
    static constexpr int LDS_BYTES = 2 * STAGE_BYTES;
    static_assert(BM % 64 == 0 && BN % 64 == 0, "2 x 2 wavefronts of whole 32 x 32 blocks");
};

template <class Cfg>
__global__ __launch_bounds__(Cfg::THREADS) void igconv_fwd_bf16_pw_kernel(const ConvKernelParams p) {
    constexpr int BM = Cfg::BM, BN = Cfg::BN, BK = Cfg::BK;
    constexpr int MB = BM / 64, NB = BN / 64;
    constexpr int RB = kPwRowBytes;
    constexpr int NA = BM / 32, NBV = BN / 32;      // 16-byte loads per thread and step: rows tid/8 + 32 i
    typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
    __shared__ __attribute__((aligned(16))) uint8_t lds[Cfg::LDS_BYTES];

    const int lane = threadIdx.x & 63;
    const int wave_all = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    const bool mover = wave_all >= 4;            // wavefronts 4-7 move, 0-3 multiply; both kinds number themselves 0-3
    const int wave = wave_all & 3, tid = (int)threadIdx.x & 255;
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, half = lane >> 5;

    // Persistent: the workgroup takes every wgsPerXcd-th tile of its XCD's contiguous range, and the load pipeline runs
    // on across the tile boundary - the last steps of a tile request the first two of the next one, which are on their
    // way while the finished tile's epilogue stores (a layer with few channels is a tile of one or two steps: its
    // whole life was a wait for those loads).
    const int tiles = p.tilesM * p.tilesN;
    const int xcd = (int)(blockIdx.x % 8u), slot = (int)(blockIdx.x / 8u);
    const int range_end = (xcd + 1) * p.tilesPerXcd < tiles ? (xcd + 1) * p.tilesPerXcd : tiles;
    int tile = xcd * p.tilesPerXcd + slot;
    if (tile >= range_end) return;

    const __amdgpu_buffer_rsrc_t xbuf = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p.x), 0, p.x_bytes, kBufferWord3);
    const __amdgpu_buffer_rsrc_t wbuf = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p.w), 0, p.w_bytes, kBufferWord3);
    const __amdgpu_buffer_rsrc_t ybuf = __builtin_amdgcn_make_buffer_rsrc(p.y, 0, p.y_bytes, kBufferWord3);

    // ---- loading role: channel vector vec of the step, rows (filter rows / pixels) tid/8 + 32 i
    const int vec = tid & 7, row = tid >> 3;
    // byte offsets of the rows' first channel, or the out-of-range marker (everything, for a tile that does not exist)
    auto tile_offsets = [&](int t, uint32_t (&a_off)[NA], uint32_t (&b_off)[NBV]) {
        const bool live = t < range_end;
        const int m0 = (t % p.tilesM) * BM, n0 = (t / p.tilesM) * BN;
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            const int m = m0 + row + 32 * i;
            a_off[i] = live && m < p.K ? (uint32_t)m * (uint32_t)p.C * 2u : kOutOfRange;
        }
#pragma unroll
        for (int i = 0; i < NBV; ++i) {
            const int j = n0 + row + 32 * i;
            const uint32_t jj = live && j < p.NPQ ? (uint32_t)j : 0u;
            const uint32_t n = magic_div(jj, p.mPQ), rem = jj - n * (uint32_t)p.PQ;
            const uint32_t pp = magic_div(rem, p.mQ), qq = rem - pp * (uint32_t)p.Q;
            const uint32_t h = pp * (uint32_t)p.u - (uint32_t)p.pad_h, w = qq * (uint32_t)p.v - (uint32_t)p.pad_w;   // (wrap below zero: fail the test)
            const bool ok = live && j < p.NPQ && h < (uint32_t)p.H && w < (uint32_t)p.W;
            b_off[i] = ok ? (n * (uint32_t)p.xsN + h * (uint32_t)p.xsH + w * (uint32_t)p.xsW) * 2u : kOutOfRange;
        }
    };
    uint32_t a_off[NA], b_off[NBV], a_nxt[NA], b_nxt[NBV];   // of the current tile and of the next one
    u32x4_t a0[NA], b0[NBV], a1[NA], b1[NBV];
    auto fetch_from = [&](int step, const uint32_t (&ao)[NA], const uint32_t (&bo)[NBV], u32x4_t (&a)[NA], u32x4_t (&b)[NBV]) {
        const int ch = step * BK + vec * 8;
        const uint32_t co = ch < p.C ? (uint32_t)ch * 2u : kOutOfRange;     // (also the step that makes an odd count even)
#pragma unroll
        for (int i = 0; i < NA; ++i)
            a[i] = __builtin_amdgcn_raw_buffer_load_b128(wbuf, (ao[i] | co) >= kOutOfRange ? kOutOfRange : ao[i] + co, 0, 0);
#pragma unroll
        for (int i = 0; i < NBV; ++i)
            b[i] = __builtin_amdgcn_raw_buffer_load_b128(xbuf, (bo[i] | co) >= kOutOfRange ? kOutOfRange : bo[i] + co, 0, 0);
    };
    auto stage = [&](int buf, const u32x4_t (&a)[NA], const u32x4_t (&b)[NBV]) {
        uint8_t *base = lds + buf * Cfg::STAGE_BYTES + row * RB + vec * 16;
#pragma unroll
        for (int i = 0; i < NA; ++i) *reinterpret_cast<u32x4_t *>(base + 32 * i * RB) = a[i];
#pragma unroll
        for (int i = 0; i < NBV; ++i) *reinterpret_cast<u32x4_t *>(base + (BM + 32 * i) * RB) = b[i];
    };

    f32x16 acc[MB][NB];
    const int steps = (p.ksteps + 1) & ~1;   // per tile, an even number: the step added to an odd count reads zeros

    // In step s the multipliers compute from LDS stage `cur` while the movers put the loaded data of step s+1 into the
    // other stage and request step s+2 - of this tile, or step s+2-steps of the next one; one barrier per step.
    if (mover) {
        auto move = [&](int s, int cur, u32x4_t (&a_new)[NA], u32x4_t (&b_new)[NBV], const u32x4_t (&a_next)[NA],
                        const u32x4_t (&b_next)[NBV]) __attribute__((always_inline)) {
            if (s + 2 < steps) fetch_from(s + 2, a_off, b_off, a_new, b_new);
            else fetch_from(s + 2 - steps, a_nxt, b_nxt, a_new, b_new);
            stage(cur ^ 1, a_next, b_next);
            __syncthreads();
        };
        tile_offsets(tile, a_off, b_off);
        fetch_from(0, a_off, b_off, a0, b0);
        fetch_from(1, a_off, b_off, a1, b1);
        stage(0, a0, b0);
        __syncthreads();
        for (; tile < range_end; tile += p.wgsPerXcd) {
            tile_offsets(tile + p.wgsPerXcd, a_nxt, b_nxt);
            for (int s = 0; s < steps; s += 2) {
                move(s, 0, a0, b0, a1, b1);
                move(s + 1, 1, a1, b1, a0, b0);
            }
#pragma unroll
            for (int i = 0; i < NA; ++i) a_off[i] = a_nxt[i];
#pragma unroll
            for (int i = 0; i < NBV; ++i) b_off[i] = b_nxt[i];
        }
        return;
    }
    auto multiply = [&](int cur) __attribute__((always_inline)) {
        const uint8_t *a_base = lds + cur * Cfg::STAGE_BYTES + (wm * (BM / 2) + l32) * RB + half * 16;
        const uint8_t *b_base = lds + cur * Cfg::STAGE_BYTES + (BM + wn * (BN / 2) + l32) * RB + half * 16;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8 av[MB], bv[NB];
#pragma unroll
            for (int i = 0; i < MB; ++i) av[i] = *reinterpret_cast<const bf16x8 *>(a_base + i * 32 * RB + ks * 32);
#pragma unroll
            for (int j = 0; j < NB; ++j) bv[j] = *reinterpret_cast<const bf16x8 *>(b_base + j * 32 * RB + ks * 32);
#pragma unroll
            for (int i = 0; i < MB; ++i)
#pragma unroll
                for (int j = 0; j < NB; ++j) {
                    if constexpr (Cfg::SWAP)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bv[j], av[i], acc[i][j], 0, 0, 0);
                    else
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[i], bv[j], acc[i][j], 0, 0, 0);
                }
        }
        __syncthreads();
    };
    __syncthreads();
    for (; tile < range_end; tile += p.wgsPerXcd) {
        const int m0 = (tile % p.tilesM) * BM, n0 = (tile / p.tilesM) * BN;
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
            for (int j = 0; j < NB; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
        float bias[MB];
        load_bias<MB>(p, m0 + wm * (BM / 2), l32, bias);
        for (int s = 0; s < steps; s += 2) {
            multiply(0);
            multiply(1);
        }
        // (the movers are already on the next tile's first steps)
        store_tile<Cfg::SWAP, MB, NB>(p, ybuf, acc, bias, m0 + wm * (BM / 2), n0 + wn * (BN / 2), half, l32);
    }
}

}  // namespace igc
#endif
