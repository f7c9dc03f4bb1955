// bf16 kernel for nine-tap filters and channel-contiguous (NHWC-style) inputs.
//
// Same method as igconv_kernel.hpp (Section 3.1 of the paper: the lowered input exists
// only as LDS tiles; the next tiles are fetched while the current ones are multiplied),
// rearranged for the bf16 MFMA rate, which is 16 times the fp32 one: an element-wise gather
// cannot feed it.  With channels contiguous in x, 8 channels of one tap of one output pixel
// are one 16-byte load - exactly what one lane feeds to v_mfma_f32_32x32x16_bf16.  So:
//  * a reduction step is 16 channels x 9 taps (144 elements of the reduction, ordered tap,
//    channel); k-group t of the step is tap t, its 16 channels split over the two halves of
//    the wavefront;
//  * D_m tile: thread = (column j, channel half), the half in the lowest lane bit; its nine loads use the nine per-column tap
//    offsets built once per tile (window test folded in, as in the fp32 nine-tap kernels)
//    plus the step's channel offset as a scalar: no vector instruction;
//  * F_m tile: the filter is packed K,C,R,S, so for one row the step is 144 contiguous
//    elements ordered (channel, tap).  Thread = (row, channel half) loads its 72 elements with
//    nine 16-byte loads and transposes them in registers (36 byte-permutes) into nine vectors
//    "8 channels of tap t", i.e. the order the MFMA wants, before writing them to LDS;
//  * LDS: [stage][tap][row][2 x 16 bytes]; the two 16-byte halves of a row are swapped on
//    every other group of 8 rows, which makes the 16-byte reads of 16 consecutive rows
//    bank-conflict free without padding.  Two stages of 9*(BM+BN)*32 bytes.
// PATCH variant of the D_m side.  The nine taps of neighbouring columns read the same pixels:
// in the zero-extended image (H+2pad_h rows of W+2pad_w pixels, all images in one flat
// index g) column j = (n,p,q) starts at b(j) = n*Hp*Wp + p*u*Wp + q*v and tap (r,s) adds
// r*Wp + s.  The pixels a tile needs are therefore the range [b(first column),
// b(last column) + (R-1)*Wp + S-1] of g: a few hundred pixels instead of 9*BN.  That range
// (16 channels of each pixel per step) is staged once per step; the MFMA operand of lane
// (column, half) for tap t is the 16 bytes at patch[half][b(column) - b(first) + r*Wp + s],
// read straight from the patch.  The host offers this variant only when the range of every
// tile fits the patch.
// The pipeline (two register sets, LDS-only barrier before the last k-group, one burst of
// side work per MFMA, single-block loop) is the one of igconv_kernel.hpp.
#ifndef IGCONV_KERNEL_BF16C_HPP_
#define IGCONV_KERNEL_BF16C_HPP_

#include "igconv_kernel.hpp"

namespace igc {

template <int BM_, int BN_, int WM_, int WN_, bool SWAP_, bool PATCH_ = false, int TEAMS_ = 1>
struct Bf16cConfig {
    static constexpr bool PATCH = PATCH_;
    // TEAMS = 2: a workgroup of 512 threads, two teams of four wavefronts, each running the whole
    // pipeline below in its own half of LDS over its half of the reduction steps; the second team's
    // accumulators are added to the first's through LDS before the epilogue (a fixed order).  For
    // problems with fewer tiles than compute units, where one workgroup per compute unit spends most
    // of a step waiting for its loads: two teams keep twice as many loads in flight.
    static constexpr int TEAMS = TEAMS_;
    static constexpr int PATCH_PIX = 512;                   // pixels of the zero-extended image per tile
    static constexpr int PATCH_PLANE = PATCH_PIX * 16 + 128;  // one channel half; +128 B: halves on disjoint banks
    static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_;
    static constexpr bool SWAP = SWAP_;
    static constexpr int TEAM_THREADS = 256;
    static constexpr int THREADS = TEAM_THREADS * TEAMS_;
    static constexpr int TAPS = 9, CH = 16;                 // per reduction step
    static constexpr int BK = TAPS * CH;
    static constexpr int ROW_BYTES = CH * 2;                // one row of one tap: two 16-byte halves
    // Every thread stages filter rows, so that the main loop has no divergent code: the
    // F_m planes always hold TEAM_THREADS/2 rows, of which the first BM are used.
    // (one thread per half row: with fewer than TEAM_THREADS/2 rows the idle threads load nothing and
    // write to 16 spare rows past the tile's - a two-way bank conflict on writes nobody reads -
    // so that two workgroups fit a compute unit)
    static constexpr int AR = BM_ < TEAM_THREADS / 2 ? BM_ + 16 : TEAM_THREADS / 2;
    static constexpr int A_BYTES = TAPS * AR * ROW_BYTES;
    static constexpr int B_BYTES = PATCH ? 2 * PATCH_PLANE : TAPS * BN * ROW_BYTES;
    static constexpr int TEAM_LDS_BYTES = 2 * (A_BYTES + B_BYTES);
    static constexpr int LDS_BYTES = TEAMS_ * TEAM_LDS_BYTES;
    static constexpr int TM = BM / WM, TN = BN / WN;
    static constexpr int MB = TM / 32, NB = TN / 32;
    static_assert(WM * WN == 4, "four wavefronts per workgroup");
    static_assert(BM % (32 * WM) == 0 && BN % (32 * WN) == 0, "wave blocks are 32x32 multiples");
    static_assert(BM <= AR && (PATCH || 2 * BN == TEAM_THREADS), "thread = (row or column, channel half)");
    static_assert(TEAMS_ == 1 || (TEAMS_ == 2 && BM_ * BN_ * 4 <= TEAM_LDS_BYTES), "two teams: the second team's results pass through its LDS");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget");
};

template <class Cfg>
__global__ __launch_bounds__(Cfg::THREADS) void igconv_fwd_bf16c_kernel(const ConvKernelParams p) {
    constexpr int BM = Cfg::BM, BN = Cfg::BN, MB = Cfg::MB, NB = Cfg::NB;
    constexpr int TAPS = Cfg::TAPS;

    __shared__ __attribute__((aligned(16))) uint8_t lds[Cfg::LDS_BYTES];
    // (two teams: `tid` is the thread's number within its team, `wave` the wavefront's)
    const int team = Cfg::TEAMS > 1 ? __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 8) : 0;
    uint8_t *const ldsA = lds + team * Cfg::TEAM_LDS_BYTES;   // [2][TAPS][AR][32]
    uint8_t *const ldsB = ldsA + 2 * Cfg::A_BYTES;            // [2][TAPS][BN][32]

    const int tid = threadIdx.x & 255;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5;
    const int l32 = lane & 31;

    // tile numbering: see igconv_kernel.hpp (contiguous ranges of tiles per XCD)
    const int tile = (int)(blockIdx.x % 8u) * p.tilesPerXcd + (int)(blockIdx.x / 8u);
    if (tile >= p.tilesM * p.tilesN) return;
    const int m0 = (tile % p.tilesM) * BM;
    const int n0 = (tile / p.tilesM) * BN;

    const __amdgpu_buffer_rsrc_t xbuf = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p.x), 0, p.x_bytes, kBufferWord3);
    const __amdgpu_buffer_rsrc_t wbuf = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p.w), 0, p.w_bytes, kBufferWord3);
    const __amdgpu_buffer_rsrc_t ybuf = __builtin_amdgcn_make_buffer_rsrc(p.y, 0, p.y_bytes, kBufferWord3);

    // ---- D_m role -------------------------------------------------------------------
    // Both variants: thread = (jl, hb) with the channel half hb in the lowest lane bit, so that
    // neighbouring lanes read the two halves of one 32-byte run; NBL 16-byte loads per step
    // whose per-thread offsets are built once per tile (validity folded in), the step's
    // channel offset being added as a scalar.
    constexpr bool PATCH = Cfg::PATCH;
    constexpr int NBL = PATCH ? Cfg::PATCH_PIX / 128 : TAPS;
    const int jl = tid >> 1, hb = tid & 1;
    uint32_t b_voff[NBL];
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
    uint32_t g_first = 0;  // PATCH: flat index of the tile's first pixel
    if constexpr (PATCH) {
        // thread stages pixels g_first + jl + 128*i, i < NBL
        g_first = __builtin_amdgcn_readfirstlane(window_start((uint32_t)n0));
        const int j_last = n0 + BN - 1 < p.NPQ ? n0 + BN - 1 : p.NPQ - 1;
        const uint32_t g_end = __builtin_amdgcn_readfirstlane(window_start((uint32_t)j_last)) +
                               (uint32_t)((p.R - 1) * p.Wp + p.S);   // one past the tile's last pixel
#pragma unroll
        for (int i = 0; i < NBL; ++i) {
            const uint32_t g = g_first + (uint32_t)(jl + 128 * i);
            const uint32_t n = magic_div(g, p.mHpWp);
            const uint32_t rem = g - n * (uint32_t)p.HpWp;
            const uint32_t hp = magic_div(rem, p.mWp);
            const uint32_t wp = rem - hp * (uint32_t)p.Wp;
            const uint32_t h = hp - (uint32_t)p.pad_h, w = wp - (uint32_t)p.pad_w;  // wrap below 0 -> huge
            const bool ok = g < g_end && h < (uint32_t)p.H && w < (uint32_t)p.W;   // (g < g_end implies n < N)
            b_voff[i] = ok ? (n * (uint32_t)p.xsN + h * (uint32_t)p.xsH + w * (uint32_t)p.xsW) * 2u + (uint32_t)hb * 16u
                           : kOutOfRange;
        }
    } else {
        // thread stages the nine taps of column n0 + jl
        const int j = n0 + jl;
        const bool cv = j < p.NPQ;
        const uint32_t jj = cv ? (uint32_t)j : 0u;
        const uint32_t n = magic_div(jj, p.mPQ);
        const uint32_t rem = jj - n * (uint32_t)p.PQ;
        const uint32_t pp = magic_div(rem, p.mQ);
        const uint32_t qq = rem - pp * (uint32_t)p.Q;
        const int h0 = (int)pp * p.u - p.pad_h;
        const int w0 = (int)qq * p.v - p.pad_w;
        const uint32_t colbase_b = (n * (uint32_t)p.xsN + (uint32_t)h0 * (uint32_t)p.xsH + (uint32_t)w0 * (uint32_t)p.xsW) * 2u;
        u16x2 hw0, hw_max;  // packed 16-bit window test, see igconv_kernel.hpp
        hw0[1] = cv ? (uint16_t)h0 : (uint16_t)0x8000;
        hw0[0] = (uint16_t)w0;
        hw_max[1] = (uint16_t)(p.H - 1);
        hw_max[0] = (uint16_t)(p.W - 1);
#pragma unroll
        for (int t = 0; t < TAPS; ++t) {
            uint32_t tr, ts;
            tap_rs(t, tr, ts);
            const u16x2 tap = __builtin_bit_cast(u16x2, (tr << 16) | ts);
            const u16x2 hw = hw0 + tap;
            const u16x2 cl = __builtin_elementwise_min(hw, hw_max);
            const bool ok = __builtin_bit_cast(uint32_t, cl) == __builtin_bit_cast(uint32_t, hw);
            b_voff[t] = ok ? colbase_b + (tr * (uint32_t)p.xsH + ts * (uint32_t)p.xsW) * 2u + (uint32_t)hb * 16u : kOutOfRange;
        }
    }
    // LDS byte offset of (row, 16-byte half) inside one tap plane, halves swapped on every
    // other group of 8 rows
    auto plane_off = [](int row, int hf) { return row * 32 + ((hf ^ ((row >> 3) & 1)) << 4); };
    const int b_woff = PATCH ? hb * Cfg::PATCH_PLANE + jl * 16 : plane_off(jl, hb);

    // ---- F_m role: thread = (row, channel half ha) -----------------------------------
    const int a_row = tid >> 1, ha = tid & 1;
    const uint32_t a_voff = (a_row < BM && m0 + a_row < p.K)
                                ? ((uint32_t)(m0 + a_row) * (uint32_t)p.CRS + (uint32_t)ha * 72u) * 2u
                                : kOutOfRange;
    const int a_woff = plane_off(a_row < BM ? a_row : BM + (a_row & 15), ha);

    constexpr int NAL = TAPS;      // filter loads per thread and step

    // registers holding the tiles in flight (two sets)
    u32x4 a_reg[2][NAL], b_reg[2][NBL];
    uint32_t sc_asoff = 0, sc_bsoff = 0;

    // Steps of this team: [s_begin, s_end); every team runs `team_steps` of them (the workgroup's
    // barriers are common), the ones past s_end on zeros.
    const int team_steps = Cfg::TEAMS > 1 ? ((p.ksteps + Cfg::TEAMS - 1) / Cfg::TEAMS + 1) & ~1 : p.ksteps;
    const int s_begin = team * team_steps;
    const int s_end = Cfg::TEAMS > 1 ? min(p.ksteps, s_begin + team_steps) : p.ksteps;
    auto decode = [&](int tau) {
        const uint32_t ut = __builtin_amdgcn_readfirstlane((uint32_t)(s_begin + tau));
        const uint32_t live = mask_lt(ut, (uint32_t)max(s_end, 0));
        sc_asoff = ((ut * (uint32_t)(Cfg::BK * 2)) & live) | (p.w_bytes & ~live);   // 16 channels x 9 taps of a row
        sc_bsoff = ((ut * (uint32_t)(Cfg::CH * 2) * (uint32_t)p.xsC) & live) | (p.x_bytes & ~live);
    };
    auto load_a = [&](int set, int q) {   // q-th 16 bytes of this thread's 72 elements
        a_reg[set][q] = __builtin_amdgcn_raw_buffer_load_b128(wbuf, a_voff + (uint32_t)q * 16u, sc_asoff, 0);
    };
    auto load_b = [&](int set, int i) {
        b_reg[set][i] = __builtin_amdgcn_raw_buffer_load_b128(xbuf, b_voff[i], sc_bsoff, 0);
    };
    // Tap t of the thread's 8 channels: element (c, t) sits at position c*9 + t of the 72
    // loaded ones, i.e. 16-bit half (c*9+t)&1 of dword (c*9+t)>>1.
    auto write_a = [&](int set, int buf, int t) {
        u32x4 o;
#pragma unroll
        for (int jd = 0; jd < 4; ++jd) {
            const int e_lo = 18 * jd + t, e_hi = 18 * jd + 9 + t;      // channels 2jd, 2jd+1
            const uint32_t lo = a_reg[set][(e_lo >> 1) >> 2][(e_lo >> 1) & 3];
            const uint32_t hi = a_reg[set][(e_hi >> 1) >> 2][(e_hi >> 1) & 3];
            // result = {16-bit half e_lo&1 of lo, 16-bit half e_hi&1 of hi}; e_hi&1 != e_lo&1
            o[jd] = __builtin_amdgcn_perm(hi, lo, (t & 1) ? 0x05040302u : 0x07060100u);
        }
        *reinterpret_cast<u32x4 *>(ldsA + buf * Cfg::A_BYTES + t * (Cfg::AR * 32) + a_woff) = o;
    };
    auto write_b = [&](int set, int buf, int i) {
        constexpr int kStride = PATCH ? 128 * 16 : BN * 32;  // 128 pixels further / next tap plane
        *reinterpret_cast<u32x4 *>(ldsB + buf * Cfg::B_BYTES + i * kStride + b_woff) = b_reg[set][i];
    };
    constexpr int NL = 1 + NAL + NBL, NW = NAL + NBL;
    auto load_item = [&](int i, int set, int tau) {
        if (i == 0) decode(tau);
        else if (i <= NAL) load_a(set, i - 1);
        else load_b(set, i - 1 - NAL);
    };
    auto write_item = [&](int i, int set, int buf) {
        if (i < NAL) write_a(set, buf, i);
        else write_b(set, buf, i - NAL);
    };

    // ---- MFMA role -------------------------------------------------------------------
    const int wm = wave % Cfg::WM, wn = wave / Cfg::WM;
    f32x16 acc[MB][NB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mb][nb][v] = 0.f;
    float bvec[MB];   // bias of the wavefront's rows, fetched long before the epilogue
    load_bias<MB>(p, m0 + wm * Cfg::TM, l32, bvec);
    constexpr int G = TAPS, MPG = MB * NB, NM = G * MPG, SB = NM - MPG;
    u32x4 fragA[2][MB], fragB[2][NB];
    // (wm*TM + mb*32 and wn*TN + nb*32 are multiples of 16, so the half swap depends on l32 only)
    const int fa_off = (wm * Cfg::TM) * 32 + plane_off(l32, half);
    const int fb_off = (wn * Cfg::TN) * 32 + plane_off(l32, half);
    // PATCH: LDS offset of the lane's operand per column block and tap
    int fb_patch[PATCH ? NB : 1][PATCH ? TAPS : 1];
    if constexpr (PATCH) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            const int j = n0 + wn * Cfg::TN + nb * 32 + l32;
            // columns past the end are never stored; let them read the last column's window
            const uint32_t rel = window_start((uint32_t)(j < p.NPQ ? j : p.NPQ - 1)) - g_first;
#pragma unroll
            for (int t = 0; t < TAPS; ++t) {
                uint32_t tr, ts;
                tap_rs(t, tr, ts);
                fb_patch[nb][t] = half * Cfg::PATCH_PLANE + (int)(rel + tr * (uint32_t)p.Wp + ts) * 16;
            }
        }
    }
    auto read_frags = [&](int buf, int g, int fs) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
            fragA[fs][mb] = *reinterpret_cast<const u32x4 *>(ldsA + buf * Cfg::A_BYTES + g * (Cfg::AR * 32) + fa_off + mb * 1024);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            if constexpr (PATCH)
                fragB[fs][nb] = *reinterpret_cast<const u32x4 *>(ldsB + buf * Cfg::B_BYTES + fb_patch[nb][g]);
            else
                fragB[fs][nb] = *reinterpret_cast<const u32x4 *>(ldsB + buf * Cfg::B_BYTES + g * (BN * 32) + fb_off + nb * 1024);
        }
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
    auto lds_barrier = [&]() {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
    };

    // ---- main loop (see igconv_kernel.hpp) -----------------------------------------------
    auto step = [&](auto parity, int t) {
        constexpr int cur = decltype(parity)::value, nxt = cur ^ 1;
        constexpr int fs0 = cur;  // G = 9 is odd: the fragment sets keep alternating across steps
        const int k2 = t + 2;
        static_for<NM>([&](auto mc) {
            constexpr int m = decltype(mc)::value;
            constexpr int g = m / MPG, j = m % MPG;
            constexpr int fs = (fs0 + g) & 1;
            if constexpr (j == 0 && g + 1 < G) read_frags(cur, g + 1, fs ^ 1);
            if constexpr (m == SB) {
                lds_barrier();
                read_frags(nxt, 0, fs ^ 1);
            }
            // Loads go out in two bursts (filter rows, then pixels): a thread's loads hit the same
            // few cache lines, which a 32 KB L1 only keeps if nothing else comes between them.
            constexpr int l0 = m == 0 ? 0 : (m == 1 ? 1 + NAL : NL), l1 = m == 0 ? 1 + NAL : NL;
            static_for<(l1 > l0 ? l1 - l0 : 0)>([&](auto ic) { load_item(l0 + decltype(ic)::value, cur, k2); });
            constexpr int WS = NW < SB ? NW : SB;
            if constexpr (m >= SB - WS && m < SB) {
                constexpr int q = m - (SB - WS);
                constexpr int w0 = (q * NW + WS - 1) / WS, w1 = ((q + 1) * NW + WS - 1) / WS;
                static_for<w1 - w0>([&](auto ic) { write_item(w0 + decltype(ic)::value, nxt, nxt); });
            }
            mfma(fs, j);
            __builtin_amdgcn_sched_barrier(0);
        });
    };
    static_for<NL>([&](auto ic) { load_item(decltype(ic)::value, 0, 0); });
    static_for<NL>([&](auto ic) { load_item(decltype(ic)::value, 1, 1); });
    static_for<NW>([&](auto ic) { write_item(decltype(ic)::value, 0, 0); });
    lds_barrier();
    read_frags(0, 0, 0);
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): enter the loop with no load outstanding
    __builtin_amdgcn_sched_barrier(0);
    for (int t = 0; t < team_steps; t += 2) {
        step(std::integral_constant<int, 0>{}, t);
        step(std::integral_constant<int, 1>{}, t + 1);
    }

    if constexpr (Cfg::TEAMS > 1) {
        // the second team's sums go to the first through the second team's LDS (all of its reads
        // are done: barrier), 16 bytes per lane and piece: lane-contiguous, conflict-free
        __syncthreads();
        f32x4 *const xch = reinterpret_cast<f32x4 *>(lds + Cfg::TEAM_LDS_BYTES) + (wave * MB * NB * 4) * 64 + lane;
        if (team == 1) {
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                    for (int c = 0; c < 4; ++c)
                        xch[((mb * NB + nb) * 4 + c) * 64] =
                            f32x4{acc[mb][nb][4 * c], acc[mb][nb][4 * c + 1], acc[mb][nb][4 * c + 2], acc[mb][nb][4 * c + 3]};
        }
        __syncthreads();
        if (team == 1) return;
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
    store_tile<Cfg::SWAP, MB, NB>(p, ybuf, acc, bvec, m0 + wm * Cfg::TM, n0 + wn * Cfg::TN, half, l32);
}

}  // namespace igc
#endif
