// Backward-filter kernels for gfx950 (paper, Section 2.1: the gradient with respect to the
// filters is one of the convolution's three forms; Section 3.1: the lowered operand exists only
// as on-chip tiles).  dw (K x CRS) = dy (K x NPQ) . D_m^T: rows are output channels k, columns
// filter elements (c,r,s), and the reduction runs over the output pixels (n,p,q).  The software
// pipeline, the LDS layout, the MFMA role and the epilogue are those of igconv_kernel.hpp (whose
// helpers this file uses); what differs is where the two operands come from:
//  * the first operand is dy, read element by element through its strides with one decode of the
//    thread's reduction index (n,p,q) per step;
//  * the gathered operand is x at (n, c, p*u + r - pad_h, q*v + s - pad_w), in one of three ways:
//    GATHER_WGRAD      columns (c,r,s) one per lane, the window test per element on packed 16-bit
//                      coordinates (any problem);
//    GATHER_WGRAD_TAP  columns ordered (tap, channel), one tap per column tile: lanes run along the
//                      reduction index (consecutive pixels: coalesced loads), decode it and test the
//                      window once per step - the tile's tap is a scalar - and a thread's elements
//                      are channels reached through a scalar offset (wants C to fill a column tile);
//    GATHER_WGRAD_NOPAD  no padding, few channels: lanes along the reduction index as above,
//                      columns in filter order; a thread keeps the offsets of its columns in
//                      registers for the whole tile and a gathered element costs one addition.
// The reduction is cut into ranges (p.splits), one "tile" per (tile, range); each range writes its
// own copy of the output, summed in order afterwards (igconv_kernels_wgrad.hip).
#ifndef IGCONV_KERNEL_WGRAD_HPP_
#define IGCONV_KERNEL_WGRAD_HPP_

#include "igconv_kernel.hpp"

namespace igc {

template <bool BF16_, int BM_, int BN_, int BK_, int WM_, int WN_, int GMODE_>
struct WgradConfig {
    static constexpr int GMODE = GMODE_;
    static constexpr bool BF16 = BF16_;
    static constexpr int BM = BM_, BN = BN_, BK = BK_, WM = WM_, WN = WN_;
    static constexpr bool SWAP = false;  // lanes run along the columns (c,r,s) in the epilogue
    static constexpr int THREADS = 256;
    static constexpr int ESIZE = BF16 ? 2 : 4;
    static constexpr int VEC = 16 / ESIZE;           // elements per 16-byte LDS access
    static constexpr int KG = 2 * VEC;               // reduction elements per k-group
    static constexpr int REM = 0;                    // (no partial k-group: BK is a multiple of KG)
    static constexpr int LDV = (BK / VEC + 1) | 1;   // LDS row stride in 16-byte units (odd: see igconv_kernel.hpp)
    static constexpr int LD = LDV * VEC;
    static constexpr int A_ELEMS = BM * LD, B_ELEMS = BN * LD;
    static constexpr int LDS_BYTES = 2 * (A_ELEMS + B_ELEMS) * ESIZE;
    static constexpr int MIN_WAVES = LDS_BYTES <= 80 * 1024 ? 2 : 1;   // waves per SIMD the registers must allow
    static constexpr int TM = BM / WM, TN = BN / WN; // per-wave output block
    static constexpr int MB = TM / 32, NB = TN / 32; // 32x32 MFMA blocks per wave
    static constexpr int CG = BN / 64;               // column groups of 64 lanes
    static constexpr int KPARTS = 4 / CG;            // wavefronts sharing one column group
    static constexpr int KPT = BK / KPARTS;          // reduction indices gathered per thread (GATHER_WGRAD)
    static_assert(WM * WN == 4, "four wavefronts per workgroup");
    static_assert(BM % (32 * WM) == 0 && BN % (32 * WN) == 0, "wave blocks are 32x32 multiples");
    static_assert(BN == 64 || BN == 128 || BN == 256, "column tile is 1, 2 or 4 wavefronts wide");
    static_assert(BK % KG == 0 && BK % KPARTS == 0 && KPT % 2 == 0 && 256 % BK == 0, "k tile granularity; one reduction index per thread");
    static_assert(GMODE == GATHER_WGRAD || GMODE == GATHER_WGRAD_TAP || GMODE == GATHER_WGRAD_NOPAD, "a backward-filter gather");
    static_assert(GMODE == GATHER_WGRAD || BK == 32, "a half wavefront spans the reduction indices of a step");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget");
};

template <class Cfg>
__global__ __launch_bounds__(Cfg::THREADS, Cfg::MIN_WAVES) void igconv_wgrad_kernel(const ConvKernelParams p) {
    constexpr int BM = Cfg::BM, BN = Cfg::BN, BK = Cfg::BK, LD = Cfg::LD;
    constexpr int VEC = Cfg::VEC, KG = Cfg::KG, ES = Cfg::ESIZE;
    constexpr int MB = Cfg::MB, NB = Cfg::NB, KPT = Cfg::KPT;
    constexpr int GM = Cfg::GMODE;
    constexpr bool WGN = GM == GATHER_WGRAD_NOPAD;
    constexpr bool WGT = GM == GATHER_WGRAD_TAP || WGN;   // lanes along the reduction index
    using elem_t = typename std::conditional<Cfg::BF16, uint16_t, float>::type;

    __shared__ __attribute__((aligned(16))) elem_t lds[2 * (Cfg::A_ELEMS + Cfg::B_ELEMS)];
    elem_t *const ldsA = lds;                        // [2][BM][LD]
    elem_t *const ldsB = ldsA + 2 * Cfg::A_ELEMS;    // [2][BN][LD]

    const int tid = threadIdx.x & 255;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5;   // which half of the k-group this lane feeds
    const int l32 = lane & 31;

    // persistent workgroups, tiles numbered in contiguous ranges per XCD (see igconv_kernel.hpp); above one range
    // the tile numbers repeat once per range of the reduction
    const int wg_xcd = (int)(blockIdx.x % 8u), wg_local = (int)(blockIdx.x / 8u);
    const int tiles_mn = p.tilesM * p.tilesN;
    const int tiles_total = tiles_mn * p.splits;
    auto tile_number = [&](int i) {
        const int local = wg_local + i * p.wgsPerXcd;
        const int t = wg_xcd * p.tilesPerXcd + local;
        return local < p.tilesPerXcd && t < tiles_total ? t : tiles_total;
    };
    if (tile_number(0) >= tiles_total) return;
    // The tile whose loads are being issued.  A tile number of tiles_total stands for "no tile": its reduction
    // range lies beyond the end, so that all it gathers is zeros.
    int m0 = 0, n0 = 0, split = 0, t_begin = 0;

    const __amdgpu_buffer_rsrc_t xbuf = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p.x), 0, p.x_bytes, kBufferWord3);
    const __amdgpu_buffer_rsrc_t wbuf = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p.w), 0, p.w_bytes, kBufferWord3);
    // ---- GATHER_WGRAD: this lane's column j -> (c,r,s) (divisors PQ = R*S and Q = S of the filter) ---------------
    // hw0 packs the window origin (tap_r - pad_h, tap_s - pad_w) as two 16-bit fields; adding the packed window
    // coordinates (p*u, q*v) of a reduction index gives the input coordinates, inside the image iff both fields are
    // <= (H-1, W-1) as unsigned 16-bit numbers.
    const int cg = wave % Cfg::CG;
    const int kpart = wave / Cfg::CG;
    const int jl = cg * 64 + lane;
    u16x2 hw0;
    uint32_t colbase_b = 0;
    auto setup_column = [&]() {
        const int j = n0 + jl;
        const bool cv = j < p.NPQ;
        const uint32_t jj = cv ? (uint32_t)j : 0u;
        const uint32_t n = magic_div(jj, p.mPQ);
        const uint32_t rem = jj - n * (uint32_t)p.PQ;
        const uint32_t pp = magic_div(rem, p.mQ);
        const uint32_t qq = rem - pp * (uint32_t)p.Q;
        const int h0 = (int)pp * p.u - p.pad_h;
        const int w0 = (int)qq * p.v - p.pad_w;
        colbase_b = (n * (uint32_t)p.xsN + (uint32_t)h0 * (uint32_t)p.xsH + (uint32_t)w0 * (uint32_t)p.xsW) * ES;
        hw0[1] = (uint16_t)h0;
        hw0[0] = (uint16_t)w0;
        if (!cv) {
            hw0[1] = 0x8000;           // no element of a column beyond the end is ever in range
        }
    };
    u16x2 hw_max;
    hw_max[1] = (uint16_t)(p.H - 1);
    hw_max[0] = (uint16_t)(p.W - 1);

    // ---- first operand (dy): BM*BK elements, one reduction index per thread (the same in all its passes) -----
    constexpr int A_TOTAL = BM * BK;
    constexpr int A_PASSES = (A_TOTAL + 255) / 256;
    constexpr bool A_PARTIAL = A_TOTAL % 256 != 0;
    int a_row[A_PASSES], a_kk[A_PASSES];
#pragma unroll
    for (int ps = 0; ps < A_PASSES; ++ps) {
        const int idx = tid + ps * 256;
        a_row[ps] = idx / BK;
        a_kk[ps] = idx % BK;
    }

    // Registers holding the tiles in flight between HBM and LDS: two sets, tile T uses set T&1.
    elem_t a_sca[2][A_PASSES];
    elem_t b_val[2][KPT > BN / 8 ? KPT : BN / 8];
    // GATHER_WGRAD: per-lane decode, lane L standing for element L of this wavefront's run of the step: byte offset
    // of the element's window coordinates (dec_so) and the packed coordinates (dec_tap).
    uint32_t dec_il = 0, dec_c = 0, dec_rs = 0, dec_so = 0, dec_tap = 0;
    int sc_tau = 0;
    uint32_t a_jo = 0;  // offset of this thread's reduction index in the first operand
    // GATHER_WGRAD_TAP / _NOPAD: this thread's reduction index of a step is lane % 32; its columns are BN/8
    // consecutive ones starting at wave*(BN/4) + (lane/32)*(BN/8) of the tile.  Per tile: the tap's window offset and
    // the scalar offset of the wavefront's first channel; per step: the pixel's offset for this tap (window test
    // folded in).
    constexpr int WT_E = BN / 8;
    const int wt_kk = lane & 31;
    const int wt_col = wave * (BN / 4) + half * WT_E;
    const uint32_t wt_laneoff = (uint32_t)(half * WT_E) * (uint32_t)p.xsN * ES;
    int sc_tap_h = 0, sc_tap_w = 0, sc_tapidx = 0;
    uint32_t wn_col[WGN ? WT_E : 1];   // GATHER_WGRAD_NOPAD: offsets of this thread's columns (c,r,s) in x
    uint32_t sc_colso = 0, wt_pix = kOutOfRange, wt_n = 0, wt_rem = 0, wt_j = 0;

    // (rows beyond K are never stored: they may read row 0; the reduction index's part of the offset, which also
    // carries the out-of-range marker, is added per step)
    uint32_t a_voff[A_PASSES];
    auto setup_rows = [&]() {
#pragma unroll
      for (int ps = 0; ps < A_PASSES; ++ps) {
        const int row = m0 + a_row[ps];
        a_voff[ps] = (uint32_t)(row < p.K ? row : 0) * (uint32_t)p.wsRow * ES;
      }
    };
    // Everything the loads of a tile depend on.
    auto setup_tile = [&](int tile) {
        if (p.splits > 1) {
            split = tile / tiles_mn;
            tile -= split * tiles_mn;
            t_begin = split * p.stepsPerSplit;
        }
        m0 = (tile % p.tilesM) * BM;
        if constexpr (WGN) {
            n0 = (tile / p.tilesM) * BN;
#pragma unroll
            for (int e = 0; e < WT_E; ++e) {
                // column i -> (c, r, s) with PQ = R*S and Q = S of the filter; tap in reading direction
                const uint32_t i = (uint32_t)(n0 + wt_col + e);
                const uint32_t c = magic_div(i, p.mPQ);
                const uint32_t rs = i - c * (uint32_t)p.PQ;
                const uint32_t r = magic_div(rs, p.mQ);
                const uint32_t sx = rs - r * (uint32_t)p.Q;
                const uint32_t tr = p.flip ? (uint32_t)p.R - 1u - r : r, ts = p.flip ? (uint32_t)p.Q - 1u - sx : sx;
                wn_col[e] = i < (uint32_t)p.NPQ ? (c * (uint32_t)p.xsN + tr * (uint32_t)p.xsH + ts * (uint32_t)p.xsW) * ES : kOutOfRange;
            }
        } else if constexpr (WGT) {
            // column tile -> (tap, channel block); PQ holds the channel blocks per tap, Q and P
            // the filter's S and R
            const uint32_t tn = (uint32_t)(tile / p.tilesM);
            const uint32_t tap = magic_div(tn, p.mPQ);
            const uint32_t r = magic_div(tap, p.mQ);
            const uint32_t sx = tap - r * (uint32_t)p.Q;
            sc_tapidx = (int)tap;
            sc_tap_h = (int)(p.flip ? (uint32_t)p.R - 1u - r : r) - p.pad_h;
            sc_tap_w = (int)(p.flip ? (uint32_t)p.Q - 1u - sx : sx) - p.pad_w;
            n0 = (int)(tn - tap * (uint32_t)p.PQ) * BN;   // first channel of the tile
            sc_colso = (uint32_t)(n0 + wave * (BN / 4)) * (uint32_t)p.xsN * ES;
        } else {
            n0 = (tile / p.tilesM) * BN;
            setup_column();
        }
        setup_rows();
    };

    // Start of the load of reduction step tau, in two halves so that each fits between two MFMAs.
    auto decode1 = [&](int tau) {
        if constexpr (WGT) {
            sc_tau = __builtin_amdgcn_readfirstlane(tau);
            wt_j = (uint32_t)(sc_tau * BK + wt_kk);
            wt_n = magic_div(wt_j, p.mRS);
            wt_rem = wt_j - wt_n * (uint32_t)p.RS;
        } else {
            // i -> (n, p*Q+q) for i = first index of the run + lane
            sc_tau = __builtin_amdgcn_readfirstlane(tau);
            dec_il = (uint32_t)(tau * BK + kpart * KPT) + (uint32_t)lane;
            dec_c = magic_div(dec_il, p.mRS);
            dec_rs = dec_il - dec_c * (uint32_t)p.RS;
        }
    };
    auto decode2 = [&]() {
        if constexpr (WGT) {
            const uint32_t pp = magic_div(wt_rem, p.mS);
            const uint32_t qq = wt_rem - pp * (uint32_t)p.S;
            const bool live = wt_j < (uint32_t)p.CRS;
            const uint32_t hh = pp * (uint32_t)p.redMulH + (uint32_t)sc_tap_h;   // (wraps below zero: fails the test)
            const uint32_t ww = qq * (uint32_t)p.redMulW + (uint32_t)sc_tap_w;
            const bool ok = live && (WGN || (hh < (uint32_t)p.H && ww < (uint32_t)p.W));   // (no padding: always inside)
            wt_pix = ok ? (wt_n * (uint32_t)p.xsC + hh * (uint32_t)p.xsH + ww * (uint32_t)p.xsW) * ES + (WGN ? 0u : wt_laneoff) : kOutOfRange;
            a_jo = live ? (wt_n * (uint32_t)p.wsRed + pp * (uint32_t)p.wsTapR + qq * (uint32_t)p.wsTapS) * ES : kOutOfRange;
        } else {
            const uint32_t r = magic_div(dec_rs, p.mS);
            const uint32_t sx = dec_rs - r * (uint32_t)p.S;
            // window coordinates of the element: the reduction index is an output pixel and they are (p*u, q*v)
            const uint32_t tr = (p.flip ? (uint32_t)p.R - 1u - r : r) * (uint32_t)p.redMulH;
            const uint32_t ts = (p.flip ? (uint32_t)p.S - 1u - sx : sx) * (uint32_t)p.redMulW;
            const uint32_t so = (dec_c * (uint32_t)p.xsC + tr * (uint32_t)p.xsH + ts * (uint32_t)p.xsW) * ES;
            const bool live = dec_il < (uint32_t)p.CRS;
            // first operand: this thread's reduction index (the same in all its passes)
            const uint32_t ja = (uint32_t)(sc_tau * BK + a_kk[0]);
            const uint32_t n = magic_div(ja, p.mRS);
            const uint32_t rem = ja - n * (uint32_t)p.RS;
            const uint32_t pp = magic_div(rem, p.mS);
            const uint32_t qq = rem - pp * (uint32_t)p.S;
            a_jo = ja < (uint32_t)p.CRS
                       ? (n * (uint32_t)p.wsRed + pp * (uint32_t)p.wsTapR + qq * (uint32_t)p.wsTapS) * ES
                       : kOutOfRange;
            dec_so = so;
            dec_tap = live ? ((tr << 16) | ts) : 0x80000000u;  // i >= CRS: never in range
        }
    };
    auto load_a = [&](int set, int tau, int ps) {
        const uint32_t voffa = a_voff[ps] + a_jo;
        if constexpr (Cfg::BF16) {
            a_sca[set][ps] = __builtin_amdgcn_raw_buffer_load_b16(wbuf, voffa, 0, 0);
        } else {
            a_sca[set][ps] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(wbuf, voffa, 0, 0));
        }
    };
    // Gathered tile, element e of this thread.
    auto load_b = [&](int set, int e) __attribute__((always_inline)) {
        uint32_t vo, so;
        if constexpr (WGN) {
            // (a dead reduction index or a column past the end carries the out-of-range marker; when
            // both do, the sum wraps to a valid offset, but such a column is never stored)
            vo = wt_pix + wn_col[e];
            so = 0;
        } else if constexpr (WGT) {
            vo = wt_pix;
            so = sc_colso + (uint32_t)e * (uint32_t)p.xsN * ES;
        } else {
            // lane e's decode as scalars, then the window test
            const uint32_t d = __builtin_amdgcn_readlane(dec_so, e);
            const u16x2 tap = __builtin_bit_cast(u16x2, (uint32_t)__builtin_amdgcn_readlane(dec_tap, e));
            const u16x2 hw = hw0 + tap;
            const u16x2 cl = __builtin_elementwise_min(hw, hw_max);
            const bool ok = __builtin_bit_cast(uint32_t, cl) == __builtin_bit_cast(uint32_t, hw);
            vo = ok ? colbase_b + d : kOutOfRange;
            so = 0;
        }
        if constexpr (Cfg::BF16) {
            b_val[set][e] = __builtin_amdgcn_raw_buffer_load_b16(xbuf, vo, so, 0);
        } else {
            b_val[set][e] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(xbuf, vo, so, 0));
        }
    };
    auto write_a = [&](int set, int buf, int ps) {
        elem_t *const A = ldsA + buf * Cfg::A_ELEMS + a_row[ps] * LD + a_kk[ps];
        if (A_PARTIAL && ps == A_PASSES - 1 && a_row[ps] >= BM) return;  // threads beyond the tile
        *A = a_sca[set][ps];
    };
    // Chunk q of this lane's run of the gathered tile: 16 bytes, or 8 where the run does not
    // start on a 16-byte boundary; lanes along the reduction index write one element.
    constexpr bool B_W16 = (KPT * ES) % 16 == 0;
    constexpr int B_WE = B_W16 ? VEC : VEC / 2;  // elements per write
    auto write_b = [&](int set, int buf, int q) {
        if constexpr (WGT) {   // one element: column wt_col + q, this thread's reduction index
            ldsB[buf * Cfg::B_ELEMS + (wt_col + q) * LD + wt_kk] = b_val[set][q];
            return;
        }
        elem_t *const dst = ldsB + buf * Cfg::B_ELEMS + jl * LD + kpart * KPT + q * B_WE;
        uint32_t v[4];
        if constexpr (Cfg::BF16) {
#pragma unroll
            for (int d = 0; d < B_WE / 2; ++d)
                v[d] = (uint32_t)b_val[set][q * B_WE + 2 * d] | ((uint32_t)b_val[set][q * B_WE + 2 * d + 1] << 16);
        } else {
#pragma unroll
            for (int d = 0; d < B_WE; ++d) v[d] = __builtin_bit_cast(uint32_t, b_val[set][q * B_WE + d]);
        }
        if constexpr (B_W16) {
            u32x4 o = {v[0], v[1], v[2], v[3]};
            *reinterpret_cast<u32x4 *>(dst) = o;
        } else {
            u32x2 o = {v[0], v[1]};
            *reinterpret_cast<u32x2 *>(dst) = o;
        }
    };

    // Moving one tile is a list of small items: NL load items (decode halves, loads of the first operand, gathered
    // elements) and NW LDS-write items.
    constexpr int NB_ELEMS = WGT ? WT_E : KPT;   // gathered elements per thread and step
    constexpr int NW_A = A_PASSES, NW_B = WGT ? WT_E : KPT / B_WE, NW = NW_A + NW_B;
    constexpr int NL = 2 + A_PASSES + NB_ELEMS;
    auto load_item = [&](int i, int set, int tau) __attribute__((always_inline)) {
        if (i == 0) decode1(tau);
        else if (i == 1) decode2();
        else if (i < 2 + A_PASSES) load_a(set, tau, i - 2);
        else load_b(set, i - 2 - A_PASSES);
    };
    auto write_item = [&](int i, int set, int buf) {
        if (i < NW_A) write_a(set, buf, i);
        else write_b(set, buf, i - NW_A);
    };

    // ---- MFMA role -------------------------------------------------------------------
    const int wm = wave % Cfg::WM;
    const int wn = wave / Cfg::WM;
    f32x16 acc[MB][NB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mb][nb][v] = 0.f;

    // A step's BK reduction elements are fed to the MFMAs in k-groups: a full group is
    // 16 bytes of k per lane (the two halves of the wavefront hold different k), i.e. four
    // fp32 MFMAs (one bf16 MFMA) per 32x32 block; a last group of half that size takes
    // 8 bytes per lane.
    constexpr int G_FULL = BK / KG, REM = Cfg::REM, G = G_FULL + (REM ? 1 : 0);
    constexpr int EPG_FULL = Cfg::BF16 ? 1 : 4, EPG_LAST = REM ? REM / 2 : EPG_FULL;
    constexpr int MPG_FULL = EPG_FULL * MB * NB, MPG_LAST = EPG_LAST * MB * NB;
    constexpr int NM = G_FULL * MPG_FULL + (REM ? MPG_LAST : 0);  // MFMAs per step
    constexpr int SB = NM - MPG_LAST;                             // first MFMA of the last group
    // Operand fragments in two register sets, alternating from group to group (and on
    // across steps when G is odd), so that the next group's fragments load while this
    // group multiplies.
    u32x4 fragA[2][MB], fragB[2][NB];
    const int fa_off = (wm * Cfg::TM + l32) * LD;
    const int fb_off = (wn * Cfg::TN + l32) * LD;
    auto read_frags = [&](int buf, int g, int fs) {
        const bool full = g < G_FULL;
        const int koff = full ? g * KG + half * VEC : G_FULL * KG + half * (REM / 2);
        const elem_t *const A = ldsA + buf * Cfg::A_ELEMS + fa_off + koff;
        const elem_t *const B = ldsB + buf * Cfg::B_ELEMS + fb_off + koff;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            if (full) {
                fragA[fs][mb] = *reinterpret_cast<const u32x4 *>(A + mb * 32 * LD);
            } else {
                const u32x2 t2 = *reinterpret_cast<const u32x2 *>(A + mb * 32 * LD);
                fragA[fs][mb][0] = t2[0];
                fragA[fs][mb][1] = t2[1];
            }
        }
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            if (full) {
                fragB[fs][nb] = *reinterpret_cast<const u32x4 *>(B + nb * 32 * LD);
            } else {
                const u32x2 t2 = *reinterpret_cast<const u32x2 *>(B + nb * 32 * LD);
                fragB[fs][nb][0] = t2[0];
                fragB[fs][nb][1] = t2[1];
            }
        }
    };
    // MFMA number j of a k-group whose fragments sit in set fs.  Consecutive MFMAs go to
    // different accumulators.
    auto mfma = [&](int fs, int j) {
        const int e = j / (MB * NB), mb = (j / NB) % MB, nb = j % NB;
        if constexpr (Cfg::BF16) {
            const bf16x8 fa = __builtin_bit_cast(bf16x8, fragA[fs][mb]);
            const bf16x8 fb = __builtin_bit_cast(bf16x8, fragB[fs][nb]);
            if constexpr (Cfg::SWAP)
                acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb, fa, acc[mb][nb], 0, 0, 0);
            else
                acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, acc[mb][nb], 0, 0, 0);
        } else {
            // (whole-vector casts: a bit_cast applied to a single vector element reads
            // element 0 with this compiler)
            const f32x4 va = __builtin_bit_cast(f32x4, fragA[fs][mb]);
            const f32x4 vb = __builtin_bit_cast(f32x4, fragB[fs][nb]);
            if constexpr (Cfg::SWAP)
                acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(vb[e], va[e], acc[mb][nb], 0, 0, 0);
            else
                acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(va[e], vb[e], acc[mb][nb], 0, 0, 0);
        }
    };
    // Workgroup barrier that orders LDS traffic only: global loads stay in flight.
    auto lds_barrier = [&]() {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
    };

    // ---- main loop: the software pipeline of igconv_kernel.hpp ------------------------------
    // During step t, which multiplies LDS stage t&1: the loads of step t+2 are issued into register set t&1, one item
    // per MFMA; step t+1, requested a whole step earlier into the other set, is written to LDS stage (t+1)&1 in the
    // slots just before the barrier; before the last k-group the workgroup synchronises and the first fragments of
    // step t+1 are read.  The order is pinned with scheduling barriers.  Steps beyond a range's end read zeros.
    auto step = [&](auto parity, int k2) __attribute__((always_inline)) {   // k2: the step whose tiles are requested during this one
        constexpr int cur = decltype(parity)::value, nxt = cur ^ 1;
        constexpr int fs0 = (G & 1) ? cur : 0;  // fragment set of this step's group 0
        static_for<NM>([&](auto mc) {
            constexpr int m = decltype(mc)::value;
            constexpr int g = m / MPG_FULL < G - 1 ? m / MPG_FULL : G - 1;
            constexpr int j = m - g * MPG_FULL;
            constexpr int fs = (fs0 + g) & 1;
            if constexpr (j == 0 && g + 1 < G) read_frags(cur, g + 1, fs ^ 1);
            if constexpr (m == SB) {
                lds_barrier();
                read_frags(nxt, 0, fs ^ 1);
            }
            // load items i with floor(i * NM / NL) == m: step t+2 -> set cur
            constexpr int l0 = (m * NL + NM - 1) / NM, l1 = ((m + 1) * NL + NM - 1) / NM;
            static_for<l1 - l0>([&](auto ic) { load_item(l0 + decltype(ic)::value, cur, k2); });
            // write items, packed into the slots before the barrier: step t+1, set nxt -> stage nxt
            constexpr int WS = NW < SB ? NW : SB;   // slots used for writes
            if constexpr (m >= SB - WS && m < SB) {
                constexpr int q = m - (SB - WS);
                constexpr int w0 = (q * NW + WS - 1) / WS, w1 = ((q + 1) * NW + WS - 1) / WS;
                static_for<w1 - w0>([&](auto ic) { write_item(w0 + decltype(ic)::value, nxt, nxt); });
            }
            mfma(fs, j);
            __builtin_amdgcn_sched_barrier(0);
        });
    };

    // A tile is one range of the reduction and takes `nsteps` steps, a whole number of pairs, so that the loop body
    // stays a single basic block; a range that reaches past the last step reads zeros there.
    const int nsteps = p.stepsPerSplit;   // (even; the host rounds an odd number of steps up)
    setup_tile(tile_number(0));
    float bias_cur[MB], bias_next[MB];   // (no bias in this pass: zeros, for the shared epilogue)
    load_bias<MB>(p, m0 + wm * Cfg::TM, l32, bias_cur);
    // Prologue: request the first two steps back to back, then write the first to LDS stage 0 as it arrives.
    static_for<NL>([&](auto ic) { load_item(decltype(ic)::value, 0, t_begin); });
    static_for<NL>([&](auto ic) { load_item(decltype(ic)::value, 1, t_begin + 1); });
    static_for<NW>([&](auto ic) { write_item(decltype(ic)::value, 0, 0); });
    lds_barrier();
    read_frags(0, 0, 0);
    // Enter the loop with no load outstanding: otherwise the compiler, merging this path
    // with the loop's back edge, waits for every load at the top of each step.
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
    __builtin_amdgcn_sched_barrier(0);
    for (int it = 1;; ++it) {
        for (int t = 2; t < nsteps; t += 2) {
            step(std::integral_constant<int, 0>{}, t_begin + t);
            step(std::integral_constant<int, 1>{}, t_begin + t + 1);
        }
        // The last two steps of this tile request the first two steps of the workgroup's next tile (of "no tile"
        // after the last one).
        const int out_m0 = m0, out_n0 = n0, out_split = split, out_tap = sc_tapidx;
        const int next = tile_number(it);
        setup_tile(next);
        load_bias<MB>(p, m0 + wm * Cfg::TM, l32, bias_next);
        step(std::integral_constant<int, 0>{}, t_begin);
        step(std::integral_constant<int, 1>{}, t_begin + 1);
        // (each range of a cut reduction writes its own copy of the output, y_bytes long; GATHER_WGRAD_TAP: the
        // columns are channels, R*S elements apart, and the tile's tap moves the base)
        const uint32_t ytap = GM == GATHER_WGRAD_TAP ? (uint32_t)out_tap * 4u : 0u;
        const uint32_t ybase = (uint32_t)out_split * p.ySplitBytes + ytap;
        const __amdgpu_buffer_rsrc_t ybuf = __builtin_amdgcn_make_buffer_rsrc(
            static_cast<char *>(p.y) + ybase, 0, p.y_bytes - ytap, kBufferWord3);
        store_tile<false, MB, NB, WGT>(p, ybuf, acc, bias_cur, out_m0 + wm * Cfg::TM, out_n0 + wn * Cfg::TN, half, l32);
        if (next >= tiles_total) break;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) bias_cur[mb] = bias_next[mb];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[mb][nb][v] = 0.f;
    }
}

}  // namespace igc
#endif
