// bf16 kernel for nine-tap filters and channel-contiguous (NHWC-style) inputs with the two
// halves of the work - moving tiles into LDS, multiplying them - in different wavefronts.
//
// Same method as igconv_kernel_bf16c.hpp (Section 3.1 of the paper: the lowered input exists
// only as LDS tiles, the next tiles are fetched while the current ones are multiplied; the
// D_m side is a patch of the zero-extended image staged once per step and read by every
// tap).  What was measured on that kernel: with its loads, byte permutes, LDS writes and
// MFMAs in ONE instruction stream per wavefront, the MFMA pipe is busy 37 % of the time on a
// full chip; the same stream without the global loads 56 %, the MFMAs alone 81 %.  A
// wavefront issues in order: every wait for a load, every permute, every LDS write and every
// 16-byte LDS read (about 15 cycles of issue each) sits between two MFMAs of 32 cycles.
// Here a workgroup has 4 * GROUPS + 4 wavefronts:
//  * 4 * GROUPS "multipliers" do nothing but read operand fragments from LDS and issue MFMAs.
//    Each group of four owns the whole BM x BN tile of O_m (wavefront = 64 x 64 of it, as in
//    the other kernels) for ITS 16 of the 16 * GROUPS channels of a reduction step; with two
//    groups every SIMD holds two multipliers, whose LDS reads and MFMAs interleave, and the
//    second group's sums are added to the first's through LDS before the epilogue (a fixed
//    order: deterministic);
//  * 4 "movers" fetch the tiles of the steps ahead.  F_m: thread = (channel group, row,
//    channel half) loads its 8 channels x 9 taps (144 contiguous bytes of the packed K,C,R,S
//    filter), transposes them in registers into nine "8 channels of tap t" vectors and writes
//    them to the tap planes, as before.  D_m: the patch goes from global memory straight into
//    LDS (buffer loads with the LDS bit: 16 bytes per lane, a wavefront fills 1 KB; a pixel
//    outside the image is requested out of range and arrives as zeros), no registers, no
//    LDS write instructions.
// The two kinds meet at one workgroup barrier per reduction step.  With the multipliers on
// step t, the movers' interval tau = t + PRE (PRE intervals run before the first step):
//  * request the filter rows of step tau into register set tau mod DA;
//  * transpose the rows of step tau - DA (requested DA intervals ago) and write them to plane
//    stage (tau - DA) mod SA; they are read from step tau - DA on, i.e. PRE - DA intervals
//    later: with SLACK = 1 the movers run one interval ahead of need, with 0 just in time;
//  * request the patch of step tau - EB into patch stage (tau - EB) mod SB, EB = PRE - 2, and
//    before the barrier wait until the patch requested DB = 1 interval ago has arrived: it is
//    the one of step t + 1, which the barrier publishes.
// A plane stage is written again SA steps later and a patch stage requested again SB steps
// later, both after the barrier at which the multipliers are done with it: SA = 2 + SLACK,
// SB = 3 (read now, published next, on its way).  The filter rows wait in registers, so their
// depth DA costs no LDS.  The movers are hidden behind the multipliers: with LDS filled once
// with pseudo-random values and no loads at all the multipliers alone take the complete
// kernel's time (with LDS left at zero a third less: the matrix pipes draw less power on
// operands that do not change, and the chip clocks higher - a register-only loop of this MFMA
// reaches 2478 TFLOP/s on uniform and 1753 on changing operands).  A multiplier reads its fragments two taps ahead (three register
// sets), one read per MFMA slot; its barrier sits before the last two taps of a step, after
// which it reads the first fragments of the next stage.
//
// LDS layouts.  Filter planes: [channel group][tap][row][2 x 16 bytes], the two halves of a
// row swapped on every other group of 8 rows (conflict-free 16-byte reads of 32 consecutive
// rows).  Patch: [channel group][pixel][2 x 16 bytes] with the same swap by pixel number,
// pixel = flat index in the zero-extended images minus the tile's first; the operand of lane
// (column, half) for tap (r,s) is the 16 bytes of pixel b(column) - b(first) + r*Wp + s.
#ifndef IGCONV_KERNEL_BF16S_HPP_
#define IGCONV_KERNEL_BF16S_HPP_

#include "igconv_kernel.hpp"

namespace igc {

template <int BM_, int BN_, bool SWAP_, int GROUPS_, int PATCH_PIX_, int DA_, int SLACK_>
struct Bf16sConfig {
    static constexpr int BM = BM_, BN = BN_;
    static constexpr bool SWAP = SWAP_;
    static constexpr int GROUPS = GROUPS_;                // groups of four multipliers, each on its 16 channels of a step
    static constexpr int DA = DA_;                        // register sets for filter rows = intervals between request and use
    static constexpr int SLACK = SLACK_;
    static constexpr int PRE = DA_ + 1 + SLACK_;          // intervals before the multipliers' first step
    static constexpr int SA = 2 + SLACK_;                 // stages of filter planes
    static constexpr int EB = PRE - 2;                    // the patch of step tau - EB is requested in interval tau ...
    static constexpr int SB = PRE - EB + 1;               // ... so the patch has three stages (read, published next, on its way)
    static constexpr int DB = PRE - 1 - EB;               // intervals between a patch request and the wait for it
    static constexpr int MULT_THREADS = 256 * GROUPS_;
    static constexpr int THREADS = MULT_THREADS + 256;
    static constexpr int WAVES_PER_SIMD = THREADS / 256;
    static constexpr int TAPS = 9, CH = 16, BK = TAPS * CH * GROUPS_;   // reduction elements per step
    static constexpr int PATCH_PIX = PATCH_PIX_;          // pixels of the zero-extended image per tile
    static constexpr int A_GROUP_BYTES = TAPS * BM * 32, A_BYTES = GROUPS_ * A_GROUP_BYTES;
    static constexpr int B_GROUP_BYTES = PATCH_PIX * 32, B_BYTES = GROUPS_ * B_GROUP_BYTES;
    static constexpr int B_BASE = SA * A_BYTES;           // LDS: the plane stages, then the patch stages
    static constexpr int LDS_BYTES = SA * A_BYTES + SB * B_BYTES;
    static constexpr int WM = 1, WN = 4;                  // a group's four wavefronts side by side
    static constexpr int TM = BM / WM, TN = BN / WN;
    static constexpr int MB = TM / 32, NB = TN / 32;
    // movers: one (channel group, row, half) block of the filter per thread; the patch's 1 KB requests are dealt
    // to the wavefronts that stage no filter rows, or to all four when all four do
    static constexpr int A_WAVES = GROUPS_ * BM / 32;
    static constexpr bool B_ALL = A_WAVES == 4;
    static constexpr int B_WAVES = B_ALL ? 4 : 4 - A_WAVES;
    static constexpr int B_TOTAL = GROUPS_ * PATCH_PIX / 32;   // 1 KB requests per step
    static constexpr int B_LOADS = B_TOTAL / B_WAVES;          // ... per patch-moving wavefront
    static_assert(BM % 32 == 0 && BN % 128 == 0, "wave blocks are 32x32 multiples");
    static_assert(A_WAVES == 2 || A_WAVES == 4, "filter rows: two or four moving wavefronts");
    static_assert(PATCH_PIX % 32 == 0 && B_TOTAL % B_WAVES == 0, "patch requests divide among the wavefronts");
    static_assert(DA_ >= 1 && DA_ <= 3 && (SLACK_ == 0 || SLACK_ == 1) && DB >= 1 && EB >= 1, "depths");
    static_assert(GROUPS_ == 1 || (GROUPS_ == 2 && BM * BN * 4 <= LDS_BYTES), "two groups: the second group's sums pass through LDS");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget");
};

template <class Cfg>
__global__ __launch_bounds__(Cfg::THREADS, Cfg::WAVES_PER_SIMD) void igconv_fwd_bf16s_kernel(const ConvKernelParams p) {
#if defined(__HIP_DEVICE_COMPILE__)   // (the host pass needs the kernel's name and signature only)
    constexpr int BM = Cfg::BM, BN = Cfg::BN, MB = Cfg::MB, NB = Cfg::NB, GROUPS = Cfg::GROUPS;
    constexpr int TAPS = Cfg::TAPS, DA = Cfg::DA, SA = Cfg::SA, SB = Cfg::SB, DB = Cfg::DB, PRE = Cfg::PRE;

    __shared__ __attribute__((aligned(1024))) uint8_t lds[Cfg::LDS_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5;
    const int l32 = lane & 31;

    // tile numbering: see igconv_kernel.hpp (contiguous ranges of tiles per XCD)
    const int tile = (int)(blockIdx.x % 8u) * p.tilesPerXcd + (int)(blockIdx.x / 8u);
    if (tile >= p.tilesM * p.tilesN) return;
    const int m0 = (tile % p.tilesM) * BM;
    const int n0 = (tile / p.tilesM) * BN;
    const int T = p.ksteps;   // steps of 16 * GROUPS channels (the host offers the kernel when C is a multiple of that)

    // tap t of the reduction order -> (row, column) of the window, eq. 2 inverting the filter
    auto tap_rs = [&](int t, uint32_t &tr, uint32_t &ts) {
        const uint32_t r = magic_div((uint32_t)t, p.mS);
        const uint32_t sx = (uint32_t)t - r * (uint32_t)p.S;
        tr = p.flip ? (uint32_t)p.R - 1u - r : r;
        ts = p.flip ? (uint32_t)p.S - 1u - sx : sx;
    };
    // first pixel of column j's window as a flat index into the zero-extended images
    auto window_start = [&](uint32_t j) {
        const uint32_t n = magic_div(j, p.mPQ);
        const uint32_t rem = j - n * (uint32_t)p.PQ;
        const uint32_t pp = magic_div(rem, p.mQ);
        const uint32_t qq = rem - pp * (uint32_t)p.Q;
        return n * (uint32_t)p.HpWp + pp * (uint32_t)(p.u * p.Wp) + qq * (uint32_t)p.v;
    };
    const uint32_t g_first = __builtin_amdgcn_readfirstlane(window_start((uint32_t)n0));
    // byte offset of (row or pixel number, 16-byte half) in a plane resp. the patch
    auto swz = [](int idx, int hf) { return idx * 32 + ((hf ^ ((idx >> 3) & 1)) << 4); };
    // Workgroup barrier after this wavefront's LDS reads and writes are done.  Written out by hand: a release
    // fence would also wait for every outstanding global request of the wavefront (the requests into LDS count
    // as LDS writes for it), and the point of the stages ahead is that those stay in flight across barriers;
    // the movers wait for exactly the requests a barrier publishes before they reach it.
    auto lds_barrier = [&]() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); };

    if (wave >= 4 * GROUPS) {
        // ================================ movers ================================
        const int pw = wave - 4 * GROUPS;
        const int ptid = tid - Cfg::MULT_THREADS;
        const __amdgpu_buffer_rsrc_t xbuf = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p.x), 0, p.x_bytes, kBufferWord3);
        const __amdgpu_buffer_rsrc_t wbuf = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p.w), 0, p.w_bytes, kBufferWord3);
        const bool does_a = pw < Cfg::A_WAVES;
        const bool does_b = Cfg::B_ALL || pw >= Cfg::A_WAVES;
        const int bw = Cfg::B_ALL ? pw : pw - Cfg::A_WAVES;   // number among the patch-moving wavefronts

        // F_m: thread = (channel group, row, channel half); its block starts 16 * group + 8 * half channels
        // into the step's channels of its row
        const int a_grp = ptid / (2 * BM), a_row = (ptid % (2 * BM)) >> 1, ha = ptid & 1;
        const uint32_t a_voff = (a_grp < GROUPS && m0 + a_row < p.K)
                                    ? ((uint32_t)(m0 + a_row) * (uint32_t)p.CRS + (uint32_t)(a_grp * 144 + ha * 72)) * 2u
                                    : kOutOfRange;
        const int a_woff = (a_grp < GROUPS ? a_grp : 0) * Cfg::A_GROUP_BYTES + swz(a_row, ha);
        u32x4 a_reg[DA][TAPS];
#pragma unroll
        for (int d = 0; d < DA; ++d)
#pragma unroll
            for (int q = 0; q < TAPS; ++q) a_reg[d][q] = u32x4{0u, 0u, 0u, 0u};

        // D_m: request i of this wavefront fills the 1 KB number L = bw * B_LOADS + i of a patch stage: channel
        // group L / (PATCH_PIX / 32), pixels [32 L', 32 L' + 32) of it; lane = (pixel, 16-byte slot), the slot
        // holding the half the swap puts there
        uint32_t b_voff[Cfg::B_LOADS];
        {
            const int j_last = n0 + BN - 1 < p.NPQ ? n0 + BN - 1 : p.NPQ - 1;
            const uint32_t g_end = __builtin_amdgcn_readfirstlane(window_start((uint32_t)j_last)) +
                                   (uint32_t)((p.R - 1) * p.Wp + p.S);   // one past the tile's last pixel
#pragma unroll
            for (int i = 0; i < Cfg::B_LOADS; ++i) {
                const int L = bw * Cfg::B_LOADS + i;
                const int grp = L / (Cfg::PATCH_PIX / 32);
                const int pix = (L % (Cfg::PATCH_PIX / 32)) * 32 + (lane >> 1);
                const int hf = (lane & 1) ^ ((pix >> 3) & 1);
                const uint32_t g = g_first + (uint32_t)pix;
                const uint32_t n = magic_div(g, p.mHpWp);
                const uint32_t rem = g - n * (uint32_t)p.HpWp;
                const uint32_t hp = magic_div(rem, p.mWp);
                const uint32_t wp = rem - hp * (uint32_t)p.Wp;
                const uint32_t h = hp - (uint32_t)p.pad_h, w = wp - (uint32_t)p.pad_w;  // wrap below 0 -> huge
                const bool ok = g < g_end && h < (uint32_t)p.H && w < (uint32_t)p.W;   // (g < g_end implies n < N)
                b_voff[i] = ok ? (n * (uint32_t)p.xsN + h * (uint32_t)p.xsH + w * (uint32_t)p.xsW) * 2u +
                                     (uint32_t)(grp * 32 + hf * 16)
                               : kOutOfRange;
            }
        }
        // scalar offsets of reduction step `step` (the buffer size for a step that does not exist: everything reads as zero)
        auto a_soff = [&](int step) {
            const uint32_t live = mask_lt((uint32_t)step, (uint32_t)T);   // (step >= 0 here)
            return (((uint32_t)step * (uint32_t)(Cfg::BK * 2)) & live) | (p.w_bytes & ~live);
        };
        auto b_soff = [&](int step) {
            const uint32_t live = mask_lt((uint32_t)step, (uint32_t)T);
            return (((uint32_t)step * (uint32_t)(Cfg::CH * GROUPS * 2) * (uint32_t)p.xsC) & live) | (p.x_bytes & ~live);
        };
        // Tap t of the thread's 8 channels: element (c, t) sits at position c*9 + t of the 72 loaded ones, i.e.
        // 16-bit half (c*9+t)&1 of dword (c*9+t)>>1.
        auto write_a = [&](int set, int stage, int t) {
            u32x4 o;
#pragma unroll
            for (int jd = 0; jd < 4; ++jd) {
                const int e_lo = 18 * jd + t, e_hi = 18 * jd + 9 + t;      // channels 2jd, 2jd+1
                const uint32_t lo = a_reg[set][(e_lo >> 1) >> 2][(e_lo >> 1) & 3];
                const uint32_t hi = a_reg[set][(e_hi >> 1) >> 2][(e_hi >> 1) & 3];
                o[jd] = __builtin_amdgcn_perm(hi, lo, (t & 1) ? 0x05040302u : 0x07060100u);
            }
            *reinterpret_cast<u32x4 *>(lds + stage * Cfg::A_BYTES + t * (BM * 32) + a_woff) = o;
        };
        // One interval (see the head of the file); the register set is a compile-time constant.
        auto interval = [&](auto set_c, int tau) __attribute__((always_inline)) {
            constexpr int set = decltype(set_c)::value;
            if (does_a) {
                const int sw = tau - DA;            // step whose planes are written now (its rows sit in this set)
                if (sw >= 0) {
                    const int stage = sw % SA;
#pragma unroll
                    for (int t = 0; t < TAPS; ++t) write_a(set, stage, t);
                }
                const uint32_t so = a_soff(tau);
#pragma unroll
                for (int q = 0; q < TAPS; ++q)
                    a_reg[set][q] = __builtin_amdgcn_raw_buffer_load_b128(wbuf, a_voff + (uint32_t)q * 16u, so, 0);
            }
            if (does_b) {
                const int sb = tau - Cfg::EB;      // step whose patch is requested now
                if (sb >= 0) {
                    const int stage = sb % SB;
                    const uint32_t so = b_soff(sb);
                    uint8_t *const dst = lds + Cfg::B_BASE + stage * Cfg::B_BYTES + bw * (Cfg::B_LOADS * 1024);
#pragma unroll
                    for (int i = 0; i < Cfg::B_LOADS; ++i)
                        __builtin_amdgcn_raw_ptr_buffer_load_lds(xbuf, (__attribute__((address_space(3))) void *)(dst + i * 1024), 16,
                                                                 b_voff[i], so, 0, 0);
                }
                // Everything this wavefront has requested after the patch of DB intervals ago may stay in flight: per
                // interval B_LOADS patch requests, and TAPS filter loads when it also stages filter rows.
                constexpr int later = DB * (Cfg::B_LOADS + (Cfg::B_ALL ? TAPS : 0));
                static_assert(later < 64, "vmcnt is a 6-bit counter");
                __builtin_amdgcn_s_waitcnt(0x0F70 | (later & 15) | ((later >> 4) << 14));
            }
            lds_barrier();
        };
        const int total = T + PRE;
        for (int tau = 0; tau < total; tau += DA) {
            interval(std::integral_constant<int, 0>{}, tau);
            if constexpr (DA > 1) if (tau + 1 < total) interval(std::integral_constant<int, 1>{}, tau + 1);
            if constexpr (DA > 2) if (tau + 2 < total) interval(std::integral_constant<int, 2>{}, tau + 2);
        }
        // no request of this wavefront may still be on its way into LDS when the workgroup's LDS is given away
        __builtin_amdgcn_s_waitcnt(0x0F70);
        if constexpr (GROUPS > 1) {   // (the multipliers' exchange of sums below has two more barriers)
            lds_barrier();
            lds_barrier();
        }
        return;
    }

    // ================================ multipliers ================================
    const __amdgpu_buffer_rsrc_t ybuf = __builtin_amdgcn_make_buffer_rsrc(p.y, 0, p.y_bytes, kBufferWord3);
    const int grp = GROUPS > 1 ? wave >> 2 : 0;   // which 16 channels of a step
    const int wn = wave & 3;                      // which 64 columns of the tile
    f32x16 acc[MB][NB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mb][nb][v] = 0.f;
    float bvec[MB];   // bias of the wavefront's rows, fetched long before the epilogue
    load_bias<MB>(p, m0, l32, bvec);
    const int fa_off = grp * Cfg::A_GROUP_BYTES + swz(l32, half);
    int fb_off[NB][TAPS];   // LDS offset of the lane's patch operand per column block and tap
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const int j = n0 + wn * Cfg::TN + nb * 32 + l32;
        // columns past the end are never stored; let them read the last column's window
        const uint32_t rel = window_start((uint32_t)(j < p.NPQ ? j : p.NPQ - 1)) - g_first;
#pragma unroll
        for (int t = 0; t < TAPS; ++t) {
            uint32_t tr, ts;
            tap_rs(t, tr, ts);
            fb_off[nb][t] = grp * Cfg::B_GROUP_BYTES + swz((int)(rel + tr * (uint32_t)p.Wp + ts), half);
        }
    }
    constexpr int G = TAPS, MPG = MB * NB, NM = G * MPG;
    static_assert(G % 3 == 0, "tap g uses fragment set g mod 3 in every step");
    u32x4 fragA[3][MB], fragB[3][NB];
    // item i of the fragments of tap g: the MB filter fragments, then the NB patch fragments
    auto read_item = [&](const uint8_t *planes, const uint8_t *patch, int g, int fs, int i) {
        if (i < MB)
            fragA[fs][i] = *reinterpret_cast<const u32x4 *>(planes + g * (BM * 32) + fa_off + i * 1024);
        else
            fragB[fs][i - MB] = *reinterpret_cast<const u32x4 *>(patch + fb_off[i - MB][g]);
    };
    auto mfma = [&](int fs, int j) {
        const int mb = j / NB, nb = j % NB;
        const bf16x8 fa = __builtin_bit_cast(bf16x8, fragA[fs][mb]);
        const bf16x8 fb = __builtin_bit_cast(bf16x8, fragB[fs][nb]);
        if constexpr (Cfg::SWAP)
            acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb, fa, acc[mb][nb], 0, 0, 0);
        else
            acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, acc[mb][nb], 0, 0, 0);
    };
    __builtin_amdgcn_s_setprio(2);   // the MFMA stream goes first where both kinds of wavefront want to issue
    // the movers fill the first stages
    for (int i = 0; i < PRE; ++i) lds_barrier();
#pragma unroll
    for (int i = 0; i < MB + NB; ++i) read_item(lds, lds + Cfg::B_BASE, 0, 0, i);
#pragma unroll
    for (int i = 0; i < MB + NB; ++i) read_item(lds, lds + Cfg::B_BASE, 1, 1, i);
    int sa = 0, sb = 0;   // plane and patch stage of the current step
    for (int t = 0; t < T; ++t) {
        const int sa1 = sa + 1 == SA ? 0 : sa + 1, sb1 = sb + 1 == SB ? 0 : sb + 1;
        const uint8_t *const planes = lds + sa * Cfg::A_BYTES, *const patch = lds + Cfg::B_BASE + sb * Cfg::B_BYTES;
        const uint8_t *const planes1 = lds + sa1 * Cfg::A_BYTES, *const patch1 = lds + Cfg::B_BASE + sb1 * Cfg::B_BYTES;
        // Nine taps; the fragments of tap g+2 are requested while tap g multiplies, one per MFMA slot, so that what
        // is issued between two MFMAs fits in the time one takes.  Before the last two taps the barrier:
        // everything this wavefront needs from the stage is in registers or on its way (the barrier waits for
        // it), and the next stage is complete; the last two taps request its first two.
        static_for<NM>([&](auto mc) {
            constexpr int m = decltype(mc)::value;
            constexpr int g = m / MPG, j = m % MPG;
            if constexpr (j == 0 && g == G - 2) lds_barrier();
            constexpr int r0 = j * (MB + NB) / MPG, r1 = (j + 1) * (MB + NB) / MPG;
            static_for<r1 - r0>([&](auto ic) {
                constexpr int i = r0 + decltype(ic)::value;
                if constexpr (g + 2 < G) read_item(planes, patch, g + 2, (g + 2) % 3, i);
                else read_item(planes1, patch1, g + 2 - G, (g + 2) % 3, i);
            });
            mfma(g % 3, j);
            __builtin_amdgcn_sched_barrier(0);
        });
        sa = sa1;
        sb = sb1;
    }
    __builtin_amdgcn_s_setprio(0);
    if constexpr (GROUPS > 1) {
        // The second group's sums go to the first through LDS (nothing in it is needed any more once every
        // wavefront has passed the first barrier), 16 bytes per lane and piece: lane-contiguous, conflict-free.
        lds_barrier();
        f32x4 *const xch = reinterpret_cast<f32x4 *>(lds) + (wn * MB * NB * 4) * 64 + lane;
        if (grp == 1) {
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                    for (int c = 0; c < 4; ++c)
                        xch[((mb * NB + nb) * 4 + c) * 64] =
                            f32x4{acc[mb][nb][4 * c], acc[mb][nb][4 * c + 1], acc[mb][nb][4 * c + 2], acc[mb][nb][4 * c + 3]};
        }
        lds_barrier();
        if (grp == 1) return;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const f32x4 o = xch[((mb * NB + nb) * 4 + c) * 64];
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[mb][nb][4 * c + e] += o[e];
                }
    }
    store_tile<Cfg::SWAP, MB, NB>(p, ybuf, acc, bvec, m0, n0 + wn * Cfg::TN, half, l32);
#endif
}

}  // namespace igc
#endif
