// Double-precision implicit-GEMM convolution with the software pipeline of the fp32 kernels
// (paper, Section 2: every routine in single and double precision; Section 3.1: the lowered
// input exists only as on-chip tiles, the next tiles are fetched while the current ones are
// multiplied).  Serves the forward pass and the phases of backward data for filters of up to
// 63 taps; anything else, and backward filter, runs with igconv_kernel_f64.hpp.
//
// What igconv_kernel_f64.hpp spends per reduction step of its 64 x 64 x 16 tile - about 185
// vector instructions per thread for the window test and address of every gathered element,
// all issued in one clump before the step's 16 MFMAs, and a barrier that also waits for the
// global loads - is what keeps it at half of the rate of v_mfma_f64_16x16x4_f64.  Here:
//  * the gather is the masked one of igconv_kernel.hpp (GATHER_MASKED): the reduction runs in
//    the filter's own order (c,r,s); a wavefront owns a run of consecutive indices of a step,
//    whose tap (position in the window, offset from the window origin, bit number) is tracked
//    in scalar registers and stepped by ten scalar instructions per element; whether tap t of
//    a column's window lies inside the image is bit t of a 64-bit mask per lane, built once
//    per tile.  A gathered element costs three vector instructions and one load;
//  * filter rows are read with 16-byte loads where the reduction index is contiguous in the
//    filter (forward pass), else (backward data: the filter through its row / reduction / tap
//    strides) element by element with one decode per thread and step;
//  * loads run two steps ahead in two register sets, LDS holds two stages, the only barrier
//    of a step orders LDS traffic alone, and every piece of side work sits between two MFMAs
//    (the order is pinned, as in igconv_kernel.hpp);
//  * workgroups are persistent and walk the tiles of their XCD's range; the first loads of
//    the next tile are issued during the last two steps of the current one.
//
// Tile BM x BN x 16, 256 threads = 2 x 2 wavefronts, each with (BM/32) x (BN/32) blocks of
// 16 x 16.  LDS rows are [row][k], 16 doubles plus 16 bytes: lane (l16, lq) of a wavefront
// reads the two doubles k = 8g + 2lq, 8g + 2lq + 1 of its row with one 16-byte read and
// feeds them to two MFMAs (both operands use the same assignment of k to lanes, and the sum
// over k commutes); a row stride of 9 x 16 bytes puts 16 consecutive rows on distinct banks.
#ifndef IGCONV_KERNEL_F64M_HPP_
#define IGCONV_KERNEL_F64M_HPP_

#include "igconv_kernel.hpp"

namespace igc {

typedef double f64x4m __attribute__((ext_vector_type(4)));
typedef double f64x2m __attribute__((ext_vector_type(2)));

template <int BM_, int BN_, bool VECA_>
struct F64mConfig {
    static constexpr int BM = BM_, BN = BN_, BK = 16;
    static constexpr bool VECA = VECA_;            // filter rows fetched with 16-byte loads
    static constexpr int LD = BK + 2;              // doubles per LDS row
    static constexpr int A_ELEMS = BM * LD, B_ELEMS = BN * LD;
    static constexpr int LDS_BYTES = 2 * (A_ELEMS + B_ELEMS) * 8;
    static constexpr int WM = 2, WN = 2, TM = BM / WM, TN = BN / WN;
    static constexpr int MB = TM / 16, NB = TN / 16;
    static constexpr int CG = BN / 64, KPARTS = 4 / CG, KPT = BK / KPARTS;
    // waves per SIMD the registers must allow: four workgroups of the small tile per compute unit, two of the others
    static constexpr int MIN_WAVES = BM * BN <= 64 * 64 ? 4 : 2;
    static_assert(BM % 32 == 0 && (BN == 64 || BN == 128), "tile shapes");
    static_assert(LDS_BYTES * MIN_WAVES <= 160 * 1024, "LDS budget");
};

template <class Cfg>
__global__ __launch_bounds__(256, Cfg::MIN_WAVES) void igconv_f64m_kernel(const ConvKernelParams p) {
#if defined(__HIP_DEVICE_COMPILE__)
    constexpr int BM = Cfg::BM, BN = Cfg::BN, BK = Cfg::BK, LD = Cfg::LD;
    constexpr int MB = Cfg::MB, NB = Cfg::NB, KPT = Cfg::KPT;
    constexpr uint32_t ES = 8;
    constexpr bool VECA = Cfg::VECA;

    __shared__ __attribute__((aligned(16))) double lds[2 * (Cfg::A_ELEMS + Cfg::B_ELEMS)];
    double *const ldsA = lds;                         // [2][BM][LD]
    double *const ldsB = lds + 2 * Cfg::A_ELEMS;      // [2][BN][LD]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, lq = lane >> 4;

    // persistent workgroups, tiles numbered in contiguous ranges per XCD (see igconv_kernel.hpp)
    const int wg_xcd = (int)(blockIdx.x % 8u), wg_local = (int)(blockIdx.x / 8u);
    const int tiles_mn = p.tilesM * p.tilesN;
    const int tiles_total = tiles_mn * p.splits;
    auto tile_number = [&](int i) {
        const int local = wg_local + i * p.wgsPerXcd;
        const int t = wg_xcd * p.tilesPerXcd + local;
        return local < p.tilesPerXcd && t < tiles_total ? t : tiles_total;
    };
    if (tile_number(0) >= tiles_total) return;
    int m0 = 0, n0 = 0, split = 0, t_begin = 0;

    const __amdgpu_buffer_rsrc_t xbuf = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p.x), 0, p.x_bytes, kBufferWord3);
    const __amdgpu_buffer_rsrc_t wbuf = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p.w), 0, p.w_bytes, kBufferWord3);

    // ---- gather role: lane = column j -> (n,p,q); the wavefront's run of KPT reduction indices
    const int cg = wave % Cfg::CG;
    const int kpart = wave / Cfg::CG;
    const int jl = cg * 64 + lane;
    uint32_t colbase_b = 0;      // byte offset of x[n, 0, p*u - pad_h, q*v - pad_w] (mod 2^32)
    // bit tr*S + ts set when tap (tr, ts) of this column's window, counted in reading direction, lies outside the
    // image; all ones for a column beyond NPQ; bits from R*S on always set (bit 63 serves for "no such element")
    uint64_t inv_taps = ~0ull;
    uint64_t ms_row_bits = 0;    // bit r*S for every window row r
    for (int r = 0; r < p.R; ++r) ms_row_bits |= 1ull << (r * p.S);
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
        // window rows h0 .. h0+R-1: those with 0 <= h0 + t <= H-1 are valid (likewise columns); the valid columns
        // as a bit field of S bits, repeated for every valid row: the product with the rows' first bits
        const int rlo = h0 < 0 ? -h0 : 0, rhi = p.H - 1 - h0 < p.R - 1 ? p.H - 1 - h0 : p.R - 1;
        const int clo = w0 < 0 ? -w0 : 0, chi = p.W - 1 - w0 < p.S - 1 ? p.W - 1 - w0 : p.S - 1;
        auto bits64 = [](int lo, int hi) -> uint64_t {   // bits lo..hi, none when hi < lo (0 <= lo; hi <= 63)
            return hi >= lo ? ((~0ull >> (63 - (hi & 63))) & ~((1ull << (lo & 63)) - 1ull)) : 0ull;
        };
        const uint64_t cols = bits64(clo, chi);
        const uint64_t rows = rhi >= rlo ? (ms_row_bits & bits64(rlo * p.S, rhi * p.S)) : 0ull;
        inv_taps = cv ? ~(cols * rows) : ~0ull;
    };

    // ---- filter-tile role.  16-byte path: BM rows of 8 vectors, dealt to the threads in order.  Element path:
    // reduction index tid % 16 of the step, rows tid / 16 + 16 * pass.
    constexpr int A_PASSES = VECA ? BM * 8 / 256 : BM * BK / 256;
    const int a_kk = VECA ? (tid & 7) * 2 : (tid & 15);
    const int a_row0 = VECA ? tid >> 3 : tid >> 4;
    constexpr int A_ROWS_PER_PASS = VECA ? 32 : 16;
    uint32_t a_voff[A_PASSES];
    uint32_t a_jo = 0;   // element path: offset of this thread's reduction index in the filter
    auto setup_rows = [&]() {
#pragma unroll
        for (int ps = 0; ps < A_PASSES; ++ps) {
            const int row = m0 + a_row0 + ps * A_ROWS_PER_PASS;
            if constexpr (VECA)
                a_voff[ps] = row < p.K ? ((uint32_t)row * (uint32_t)p.CRS + (uint32_t)a_kk) * ES : kOutOfRange;
            else   // (rows beyond K are never stored: they may read row 0)
                a_voff[ps] = (uint32_t)(row < p.K ? row : 0) * (uint32_t)p.wsRow * ES;
        }
    };
    auto setup_tile = [&](int tile) {
        if (p.splits > 1) {
            split = tile / tiles_mn;
            tile -= split * tiles_mn;
            t_begin = split * p.stepsPerSplit;
        }
        m0 = (tile % p.tilesM) * BM;
        n0 = (tile / p.tilesM) * BN;
        setup_column();
        setup_rows();
    };

    // tiles in flight between memory and LDS: two register sets, step T uses set T & 1
    u32x4 a_vec[2][VECA ? A_PASSES : 1];
    u32x2 a_sca[2][VECA ? 1 : A_PASSES];
    u32x2 b_val[2][KPT];

    // the next element of this wavefront's run: columns left in its window row, rows left in its channel, byte
    // offset from the window origin, bit number, reduction indices left after it; and the three ways to step
    int sc_tau = 0;
    uint32_t ms_cs = 0, ms_cr = 0, ms_d = 0, ms_bit = 0, ms_left = 0;
    const uint32_t ms_dir = p.flip ? 0xFFFFFFFFu : 1u;
    const uint32_t ms_sm1 = (uint32_t)p.S - 1u, ms_rm1 = (uint32_t)p.R - 1u;
    const uint32_t ms_dd0 = ms_dir * (uint32_t)p.xsW * ES;
    const uint32_t ms_dd1 = ms_dir * ((uint32_t)p.xsH - ms_sm1 * (uint32_t)p.xsW) * ES;
    const uint32_t ms_dd2 = ((uint32_t)p.xsC - ms_dir * (ms_sm1 * (uint32_t)p.xsW + ms_rm1 * (uint32_t)p.xsH)) * ES;
    const uint32_t ms_db2 = 0u - ms_dir * ((uint32_t)p.RS - 1u);

    auto decode1 = [&](int tau) {
        // first index of this wavefront's run -> (c, r, s), all in scalar registers
        sc_tau = __builtin_amdgcn_readfirstlane(tau);
        const uint32_t i0 = (uint32_t)(sc_tau * BK + kpart * KPT);
        const uint32_t c = magic_div(i0, p.mRS);
        const uint32_t rs = i0 - c * (uint32_t)p.RS;
        const uint32_t r = magic_div(rs, p.mS);
        const uint32_t sx = rs - r * (uint32_t)p.S;
        const uint32_t tr = p.flip ? ms_rm1 - r : r, ts = p.flip ? ms_sm1 - sx : sx;
        ms_cs = ms_sm1 - sx;
        ms_cr = ms_rm1 - r;
        ms_d = (c * (uint32_t)p.xsC + tr * (uint32_t)p.xsH + ts * (uint32_t)p.xsW) * ES;
        ms_bit = tr * (uint32_t)p.S + ts;
        // (negative, as a signed number, from the first index past the end on; a step past the last one - a
        // backward-data phase that meets no tap runs zero steps - holds no element at all)
        ms_left = sc_tau < p.ksteps ? (uint32_t)p.CRS - 1u - i0 : 0xFFFFFFFFu;
    };
    auto decode2 = [&]() {
        if constexpr (!VECA) {
            const uint32_t ja = (uint32_t)(sc_tau * BK + a_kk);
            const uint32_t kc = magic_div(ja, p.mRS);
            const uint32_t rem = ja - kc * (uint32_t)p.RS;
            const uint32_t r = magic_div(rem, p.mS);
            const uint32_t sx = rem - r * (uint32_t)p.S;
            // (masks, not selects: the loop body stays one basic block)
            const uint32_t live = mask_lt(ja, (uint32_t)p.CRS) & mask_lt((uint32_t)sc_tau, (uint32_t)p.ksteps);
            const uint32_t off = (kc * (uint32_t)p.wsRed + (uint32_t)p.wTap0 + r * (uint32_t)p.wsTapR + sx * (uint32_t)p.wsTapS) * ES;
            a_jo = (off & live) | (kOutOfRange & ~live);
        } else {
            // the last step of a reduction that is not a multiple of 16 (an even number: a vector is inside or
            // outside): from there on the vectors past the end are requested out of range
            const uint32_t dead = (0u - (uint32_t)(sc_tau == p.tail_step)) & ~mask_lt((uint32_t)(sc_tau * BK + a_kk), (uint32_t)p.CRS);
#pragma unroll
            for (int ps = 0; ps < A_PASSES; ++ps) a_voff[ps] |= kOutOfRange & dead;
        }
    };
    auto load_a = [&](int set, int tau, int ps) {
        if constexpr (VECA) {
            const uint32_t k0 = (uint32_t)tau * BK;
            const uint32_t live = mask_lt(k0, (uint32_t)p.CRS) & mask_lt((uint32_t)tau, (uint32_t)p.ksteps);
            const uint32_t soff = ((k0 * ES) & live) | (p.w_bytes & ~live);
            a_vec[set][ps] = __builtin_amdgcn_raw_buffer_load_b128(wbuf, a_voff[ps], soff, 0);
        } else {
            a_sca[set][ps] = __builtin_amdgcn_raw_buffer_load_b64(wbuf, a_voff[ps] + a_jo, 0, 0);
        }
    };
    auto load_b = [&](int set, int e) __attribute__((always_inline)) {
        // bit 0 of the shifted mask: 1 when the tap lies outside the image (bit 63: the index is past the end);
        // shifted to bit 31 it puts the offset out of range (a valid offset lies below 2^31)
        const uint32_t bit = (int32_t)ms_left < 0 ? 63u : ms_bit;
        const uint32_t out = (uint32_t)(inv_taps >> bit);
        const uint32_t vo = (out << 31) | (colbase_b + ms_d);
        b_val[set][e] = __builtin_amdgcn_raw_buffer_load_b64(xbuf, vo, 0, 0);
    };
    // step the scalar state to the next element of the run (see igconv_kernel.hpp: ten scalar instructions chained
    // through the carry flag)
    auto advance_tap = [&]() __attribute__((always_inline)) {
        uint32_t t0, t1;
        asm volatile(
            "s_sub_u32 %0, %0, 1\n\t"
            "s_cselect_b32 %0, %7, %0\n\t"
            "s_cselect_b32 %5, %10, %9\n\t"
            "s_subb_u32 %1, %1, 0\n\t"
            "s_cselect_b32 %1, %8, %1\n\t"
            "s_cselect_b32 %5, %11, %5\n\t"
            "s_cselect_b32 %6, %13, %12\n\t"
            "s_add_u32 %2, %2, %5\n\t"
            "s_add_u32 %3, %3, %6\n\t"
            "s_sub_u32 %4, %4, 1"
            : "+s"(ms_cs), "+s"(ms_cr), "+s"(ms_d), "+s"(ms_bit), "+s"(ms_left), "=&s"(t0), "=&s"(t1)
            : "s"(ms_sm1), "s"(ms_rm1), "s"(ms_dd0), "s"(ms_dd1), "s"(ms_dd2), "s"(ms_dir), "s"(ms_db2)
            : "scc");
    };
    auto write_a = [&](int set, int buf, int ps) {
        double *const A = ldsA + buf * Cfg::A_ELEMS + (a_row0 + ps * A_ROWS_PER_PASS) * LD + a_kk;
        if constexpr (VECA) *reinterpret_cast<u32x4 *>(A) = a_vec[set][ps];
        else *reinterpret_cast<u32x2 *>(A) = a_sca[set][ps];
    };
    auto write_b = [&](int set, int buf, int q) {   // two consecutive reduction indices of this lane's column
        double *const dst = ldsB + buf * Cfg::B_ELEMS + jl * LD + kpart * KPT + 2 * q;
        const u32x4 o = {b_val[set][2 * q][0], b_val[set][2 * q][1], b_val[set][2 * q + 1][0], b_val[set][2 * q + 1][1]};
        *reinterpret_cast<u32x4 *>(dst) = o;
    };

    constexpr int NW_A = A_PASSES, NW_B = KPT / 2, NW = NW_A + NW_B;
    constexpr int NL = 2 + A_PASSES + 2 * KPT;
    auto load_item = [&](int i, int set, int tau) __attribute__((always_inline)) {
        if (i == 0) decode1(tau);
        else if (i == 1) decode2();
        else if (i < 2 + A_PASSES) load_a(set, tau, i - 2);
        else if ((i - 2 - A_PASSES) % 2 == 0) load_b(set, (i - 2 - A_PASSES) / 2);
        else advance_tap();
    };
    auto write_item = [&](int i, int set, int buf) {
        if (i < NW_A) write_a(set, buf, i);
        else write_b(set, buf, i - NW_A);
    };

    // ---- MFMA role
    const int wm = wave % Cfg::WM;
    const int wn = wave / Cfg::WM;
    f64x4m acc[MB][NB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) acc[mb][nb] = f64x4m{0.0, 0.0, 0.0, 0.0};

    constexpr int G = 2;                    // k-groups of 8 per step
    constexpr int MPG = 2 * MB * NB;        // MFMAs per group
    constexpr int NM = G * MPG, SB = NM - MPG;
    u32x4 fragA[2][MB], fragB[2][NB];
    const int fa_off = (wm * Cfg::TM + l16) * LD + lq * 2;
    const int fb_off = (wn * Cfg::TN + l16) * LD + lq * 2;
    auto read_frags = [&](int buf, int g, int fs) {
        const double *const A = ldsA + buf * Cfg::A_ELEMS + fa_off + g * 8;
        const double *const B = ldsB + buf * Cfg::B_ELEMS + fb_off + g * 8;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) fragA[fs][mb] = *reinterpret_cast<const u32x4 *>(A + mb * 16 * LD);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) fragB[fs][nb] = *reinterpret_cast<const u32x4 *>(B + nb * 16 * LD);
    };
    auto mfma = [&](int fs, int j) {
        const int e = j / (MB * NB), mb = (j / NB) % MB, nb = j % NB;
        const f64x2m va = __builtin_bit_cast(f64x2m, fragA[fs][mb]);
        const f64x2m vb = __builtin_bit_cast(f64x2m, fragB[fs][nb]);
        acc[mb][nb] = __builtin_amdgcn_mfma_f64_16x16x4f64(va[e], vb[e], acc[mb][nb], 0, 0, 0);
    };
    auto lds_barrier = [&]() {   // orders LDS traffic only: global loads stay in flight
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
    };

    // Step t multiplies LDS stage t & 1; meanwhile the loads of step t+2 are issued into register set t & 1, one
    // item per MFMA, and step t+1, requested a step earlier into the other set, is written to the other stage in the
    // slots just before the barrier, which sits before the last k-group; after it the first fragments of step t+1
    // are read.  Steps beyond the last read zeros, so no step is special.
    auto step = [&](auto parity, int k2) __attribute__((always_inline)) {
        constexpr int cur = decltype(parity)::value, nxt = cur ^ 1;
        static_for<NM>([&](auto mc) {
            constexpr int m = decltype(mc)::value;
            constexpr int g = m / MPG;
            constexpr int j = m - g * MPG;
            constexpr int fs = g & 1;
            if constexpr (j == 0 && g + 1 < G) read_frags(cur, g + 1, fs ^ 1);
            if constexpr (m == SB) {
                lds_barrier();
                read_frags(nxt, 0, fs ^ 1);
            }
            constexpr int l0 = (m * NL + NM - 1) / NM, l1 = ((m + 1) * NL + NM - 1) / NM;
            static_for<l1 - l0>([&](auto ic) { load_item(l0 + decltype(ic)::value, cur, k2); });
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

    const int nsteps = p.stepsPerSplit;   // (even; the host rounds an odd number of steps up)
    setup_tile(tile_number(0));
    static_for<NL>([&](auto ic) { load_item(decltype(ic)::value, 0, t_begin); });
    static_for<NL>([&](auto ic) { load_item(decltype(ic)::value, 1, t_begin + 1); });
    static_for<NW>([&](auto ic) { write_item(decltype(ic)::value, 0, 0); });
    lds_barrier();
    read_frags(0, 0, 0);
    // (enter the loop with no load outstanding: otherwise the compiler, merging this path with the loop's back
    // edge, waits for every load at the top of each step)
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
    __builtin_amdgcn_sched_barrier(0);
    const double alpha = p.alpha64, beta = p.beta64;
    for (int it = 1;; ++it) {
        for (int t = 2; t < nsteps; t += 2) {
            step(std::integral_constant<int, 0>{}, t_begin + t);
            step(std::integral_constant<int, 1>{}, t_begin + t + 1);
        }
        // the last two steps of this tile request the first two of the workgroup's next tile (of "no tile", whose
        // columns lie beyond the end, after the last one)
        const int out_m0 = m0, out_n0 = n0, out_split = split;
        const int next = tile_number(it);
        setup_tile(next);
        step(std::integral_constant<int, 0>{}, t_begin);
        step(std::integral_constant<int, 1>{}, t_begin + 1);
        // epilogue: value v of block (mb, nb) in lane (l16, lq) is row 4*v + lq, column l16 of the block
        const __amdgpu_buffer_rsrc_t ybuf = __builtin_amdgcn_make_buffer_rsrc(
            static_cast<char *>(p.y) + (size_t)out_split * p.ySplitBytes, 0, p.y_bytes, kBufferWord3);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            const int col = out_n0 + wn * Cfg::TN + nb * 16 + l16;
            const bool cv = col < p.NPQ;
            const uint32_t cc = cv ? (uint32_t)col : 0u;
            const uint32_t j0 = magic_div(cc, p.mPQ), rem = cc - j0 * (uint32_t)p.PQ;
            const uint32_t j1 = magic_div(rem, p.mQ), j2 = rem - j1 * (uint32_t)p.Q;
            const uint32_t ycol = j0 * (uint32_t)p.ysN + j1 * (uint32_t)p.ysP + j2 * (uint32_t)p.ysQ;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int row = out_m0 + wm * Cfg::TM + mb * 16 + 4 * v + lq;
                    const uint32_t off = cv && row < p.K ? (ycol + (uint32_t)row * (uint32_t)p.ysK) * ES : kOutOfRange;
                    double r = alpha * acc[mb][nb][v];
                    if (beta != 0.0) r += beta * __builtin_bit_cast(double, __builtin_amdgcn_raw_buffer_load_b64(ybuf, off, 0, 0));
                    __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2, r), ybuf, off, 0, 0);
                }
        }
        if (next >= tiles_total) break;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) acc[mb][nb] = f64x4m{0.0, 0.0, 0.0, 0.0};
    }
#endif
}

}  // namespace igc
#endif
