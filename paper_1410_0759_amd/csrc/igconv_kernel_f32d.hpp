// fp32 forward kernel for problems with few output elements and a long reduction (small
// mini-batches of the deeper layers): the tiles of the pipelined kernels, at least 64 x 64,
// leave most compute units without work there, and cutting the reduction across
// workgroups needs memory for the partial results.  Here a workgroup owns a 32 x 32 tile of
// O_m (paper, Section 3.1: O_m = F_m . D_m, D_m never stored) and cuts the reduction among
// its WAVES wavefronts inside the compute unit:
//  * a wavefront multiplies ITS range of the reduction for the whole tile with
//    v_mfma_f32_32x32x2_f32, whose operands are one element per lane - lane (l % 32, l / 32)
//    holds F_m[row l % 32][k] and D_m[k][column l % 32] for k = l / 32 of the instruction's
//    two - so both operands go from global memory straight into the registers the MFMA reads:
//    no LDS tiles, no barrier in the loop.  A step is 8 NV reduction indices: a lane loads NV
//    runs of four consecutive k of its filter row (16-byte loads when the filter allows) and
//    gathers the 4 NV elements of its column (pad 0: every tap of a valid column lies inside
//    the image; the offset of reduction index i relative to the window origin comes from a
//    table in LDS built once per workgroup), then feeds them to 4 NV MFMAs; requests run
//    DEPTH steps ahead in DEPTH register sets, each register refilled right after the MFMA
//    that read it.  (NV = 1 is built.  NV = 4, a whole 128-byte line of every filter row per
//    step, was measured 4 to 25 % slower: the loop is bound by the number of loads the
//    gathers need - two elements per lane and MFMA, a dozen cache lines per gather
//    instruction on small images - not by re-fetched filter lines.  Element-wise filter loads
//    cost a factor of three.)
//  * at the end the wavefronts leave their sums in LDS and every thread adds up one element
//    of the tile over the wavefronts in order (deterministic) and stores it through y's strides
//    with alpha, beta, bias and activation applied.
// Indices past the end of the reduction read zeros on both sides (out-of-range requests).
// With a zero border (MSK) every lane also keeps one bit per filter tap - whether that tap of its column's
// window lies inside the image - and a second table names the tap of every reduction index: a gather
// whose bit is clear is sent out of range and reads the border's zero (R*S <= 31; three more vector
// instructions per gathered element, which the loop, bound by the address unit, has room for).
#ifndef IGCONV_KERNEL_F32D_HPP_
#define IGCONV_KERNEL_F32D_HPP_

#include "igconv_kernel.hpp"

namespace igc {

template <int WAVES_, bool VECA_, int NV_, bool ALDS_ = false, bool MSK_ = false>
struct DirectConfig {
    static constexpr bool MSK = MSK_;     // zero border: window test from a tap mask per column
    // ALDS: the filter rows go through LDS.  Loaded as the MFMA wants them - lane = (row, half): 32 rows of 32 bytes - a
    // filter load touches 32 cache lines and costs the address unit as much as the step's four gathers together; taken
    // apart, the kernel without its filter loads or without its gathers runs at the MFMA rate, with both at half of
    // it: it is bound by the address unit, evenly by the two.  So the wavefront copies its rows in whole lines
    // instead (8 rows x 128 bytes per load, straight into its own piece of LDS: no registers, no LDS write
    // instructions; 32 reduction indices = four steps per copy, two copies in flight) and reads its MFMA operand back
    // with one 16-byte LDS read per step.  Rows sit 128 bytes apart in LDS; the 16-byte pieces of a row are stored
    // exchanged by (row / 2) % 8, so that 16 consecutive rows' reads of one piece fall on distinct banks.
    static constexpr bool ALDS = ALDS_;
    static constexpr int WAVES = WAVES_, THREADS = 64 * WAVES_;
    static constexpr bool VECA = VECA_;   // filter rows fetched with 16-byte loads (C*R*S a multiple of 4, aligned filter)
    static constexpr int NV = NV_;        // runs of four reduction indices per lane and step
    static constexpr int BM = 32, BN = 32, BK = 8 * NV_;
    static constexpr int DEPTH = direct_depth(BK, ALDS_);
    static constexpr int A_STAGE_BYTES = 32 * 128;   // ALDS: 32 rows x 32 reduction indices
    static constexpr int TAP_TABLE_BYTES = MSK_ ? kDirectTableEntries : 0;   // one byte per reduction index
    static constexpr int LDS_BYTES = kDirectTableEntries * 4 + TAP_TABLE_BYTES + (ALDS_ ? WAVES_ * 2 * A_STAGE_BYTES : 0);
    static_assert(!ALDS_ || (VECA_ && NV_ == 1 && LDS_BYTES <= 160 * 1024), "staged filter rows: 16-byte loads, steps of 8");
    static_assert(!MSK_ || NV_ == 1, "the tap mask is built for steps of 8");
    static_assert(WAVES_ * 16 * 64 <= kDirectTableEntries, "the exchange of the sums reuses the table's memory");
    static_assert(1024 % THREADS == 0, "whole elements per thread in the epilogue");
};

template <class Cfg>
__global__ __launch_bounds__(Cfg::THREADS) void igconv_f32d_kernel(const ConvKernelParams p) {
#if defined(__HIP_DEVICE_COMPILE__)
    constexpr int W = Cfg::WAVES, D = Cfg::DEPTH, THREADS = Cfg::THREADS, NV = Cfg::NV, BK = Cfg::BK;
    __shared__ __attribute__((aligned(1024))) uint32_t lds[Cfg::LDS_BYTES / 4];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, half = lane >> 5;

    // one tile per workgroup, tiles numbered in contiguous ranges per XCD (the M tiles of a column tile adjacent)
    const int tiles = p.tilesM * p.tilesN;
    const int item = (int)(blockIdx.x % 8u) * p.tilesPerXcd + (int)(blockIdx.x / 8u);
    if (item >= tiles) return;
    const int m0 = (item % p.tilesM) * 32, n0 = (item / p.tilesM) * 32;

    // offset of reduction index i = (c,r,s) relative to the window origin; out of range past the end.  The host
    // checked that every index a wavefront can request (its range and DEPTH + 1 steps beyond) has an entry.
    const int steps_w = p.stepsPerSplit;   // steps per wavefront, a multiple of DEPTH
    const uint32_t entries = (uint32_t)(W * steps_w + D + 1) * (uint32_t)BK;
    for (uint32_t i = (uint32_t)tid; i < entries; i += (uint32_t)THREADS) {
        const uint32_t c = magic_div(i, p.mRS);
        const uint32_t rs = i - c * (uint32_t)p.RS;
        const uint32_t r = magic_div(rs, p.mS);
        const uint32_t sx = rs - r * (uint32_t)p.S;
        const uint32_t tr = p.flip ? (uint32_t)p.R - 1u - r : r;
        const uint32_t ts = p.flip ? (uint32_t)p.S - 1u - sx : sx;
        const uint32_t so = (c * (uint32_t)p.xsC + tr * (uint32_t)p.xsH + ts * (uint32_t)p.xsW) * 4u;
        lds[i] = i < (uint32_t)p.CRS ? so : kOutOfRange;
        // (tap in filter order; 31, whose bit no mask has, past the end: adding the marker to the offset of a window
        // origin in the border - a negative number - could wrap back into range)
        if constexpr (Cfg::MSK) reinterpret_cast<uint8_t *>(lds + kDirectTableEntries)[i] = i < (uint32_t)p.CRS ? (uint8_t)rs : (uint8_t)31;
    }
    __syncthreads();

    const __amdgpu_buffer_rsrc_t xbuf = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p.x), 0, p.x_bytes, kBufferWord3);
    const __amdgpu_buffer_rsrc_t wbuf = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p.w), 0, p.w_bytes, kBufferWord3);

    // this lane's column j -> (n,p,q): byte offset of its window origin (a valid offset lies below 2^31, so adding
    // the marker of a dead index leaves it out of range; a column beyond NPQ reads anything: it is never stored)
    // (MSK: the origin may lie in the border, its offset negative - kept modulo 2^32: with the offset of a tap inside
    // the image added it is the element's true offset again)
    uint32_t colbase, tapmask = 0u;
    {
        const int j = n0 + l32;
        const uint32_t jj = j < p.NPQ ? (uint32_t)j : 0u;
        const uint32_t n = magic_div(jj, p.mPQ);
        const uint32_t rem = jj - n * (uint32_t)p.PQ;
        const uint32_t pp = magic_div(rem, p.mQ);
        const uint32_t qq = rem - pp * (uint32_t)p.Q;
        if constexpr (Cfg::MSK) {
            const int h0 = (int)pp * p.u - p.pad_h, w0 = (int)qq * p.v - p.pad_w;
            colbase = (n * (uint32_t)p.xsN + (uint32_t)h0 * (uint32_t)p.xsH + (uint32_t)w0 * (uint32_t)p.xsW) * 4u;
            for (int r = 0, bit = 0; r < p.R; ++r)
                for (int sx = 0; sx < p.S; ++sx, ++bit) {
                    const int hh = h0 + (p.flip ? p.R - 1 - r : r), ww = w0 + (p.flip ? p.S - 1 - sx : sx);
                    if ((unsigned)hh < (unsigned)p.H && (unsigned)ww < (unsigned)p.W) tapmask |= 1u << bit;
                }
        } else {
            colbase = (n * (uint32_t)p.xsN + pp * (uint32_t)p.u * (uint32_t)p.xsH + qq * (uint32_t)p.v * (uint32_t)p.xsW) * 4u;
        }
    }
    // this lane's filter row; within a step the lower half of the wavefront holds the first 4 NV reduction indices,
    // the upper half the others (both operands alike: which k meets which MFMA is free, the sum commutes), so that
    // a row's indices of a step are 32 NV contiguous bytes of the filter - a whole cache line for NV = 4
    const int row = m0 + l32;
    const uint32_t lane_k = 4u * NV * (uint32_t)half;
    const uint32_t a_base = row < p.K ? ((uint32_t)row * (uint32_t)p.CRS + lane_k) * 4u : kOutOfRange;

    u32x4 a_reg[D][NV];
    uint32_t b_reg[D][NV][4];
    u32x4 so4[NV];   // table entries of the step requested next
    uint32_t tap4[NV];   // MSK: their taps, a byte each
    auto read_table = [&](int t, int v) __attribute__((always_inline)) {
        so4[v] = *reinterpret_cast<const u32x4 *>(&lds[t * BK + (int)lane_k + 4 * v]);
        if constexpr (Cfg::MSK) tap4[v] = lds[kDirectTableEntries + ((t * BK + (int)lane_k + 4 * v) >> 2)];
    };
    // the request of step t in pieces, each short enough for the gap between two MFMAs
    auto request_a = [&](int set, int t, int v) __attribute__((always_inline)) {
        const uint32_t k0 = (uint32_t)t * (uint32_t)BK;
        const uint32_t kk = k0 + lane_k + 4u * (uint32_t)v;
        if constexpr (Cfg::VECA) {
            a_reg[set][v] = __builtin_amdgcn_raw_buffer_load_b128(wbuf, kk < (uint32_t)p.CRS ? a_base + 16u * (uint32_t)v : kOutOfRange,
                                                                  k0 * 4u, 0);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                a_reg[set][v][e] = __builtin_amdgcn_raw_buffer_load_b32(
                    wbuf, kk + (uint32_t)e < (uint32_t)p.CRS ? a_base + 16u * (uint32_t)v + 4u * (uint32_t)e : kOutOfRange, k0 * 4u, 0);
        }
    };
    auto request_b = [&](int set, int v, int e) __attribute__((always_inline)) {
        uint32_t off = colbase + so4[v][e];
        if constexpr (Cfg::MSK) off = ((tapmask >> ((tap4[v] >> (8 * e)) & 31u)) & 1u) ? off : kOutOfRange;
        b_reg[set][v][e] = __builtin_amdgcn_raw_buffer_load_b32(xbuf, off, 0, 0);
    };

    f32x16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;

    const int t0 = wave * steps_w;
    if constexpr (!Cfg::ALDS) {
        static_for<NV>([&](auto vc) { read_table(t0, decltype(vc)::value); });
        static_for<D>([&](auto dc) {
            constexpr int set = decltype(dc)::value;
            static_for<NV>([&](auto vc) {
                constexpr int v = decltype(vc)::value;
                request_a(set, t0 + set, v);
    #pragma unroll
                for (int e = 0; e < 4; ++e) request_b(set, v, e);
                read_table(t0 + set + 1, v);
            });
        });
        __builtin_amdgcn_sched_barrier(0);
        for (int s = 0; s < steps_w; s += D) {
            // (the order is pinned: one MFMA, then the request that refills the register it has just read - for step
            // t + DEPTH, which uses the same register set; after the four MFMAs of a run its filter vector and the table
            // entries of the step after)
            static_for<D>([&](auto dc) {
                constexpr int set = decltype(dc)::value;
                const int t = t0 + s + set + D;
                static_for<4 * NV>([&](auto ic) {
                    constexpr int v = decltype(ic)::value / 4, e = decltype(ic)::value % 4;
                    const f32x4 va = __builtin_bit_cast(f32x4, a_reg[set][v]);
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(va[e], __builtin_bit_cast(float, b_reg[set][v][e]), acc, 0, 0, 0);
                    request_b(set, v, e);
                    if constexpr (e == 3) {
                        request_a(set, t, v);
                        read_table(t + 1, v);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                });
            });
        }
    } else {
        // ---- filter rows staged in LDS (see DirectConfig) ----
        uint8_t *const a_lds = reinterpret_cast<uint8_t *>(lds + kDirectTableEntries) + Cfg::TAP_TABLE_BYTES + wave * (2 * Cfg::A_STAGE_BYTES);
        // copy j of a stage fills its 1 KB number j: lane -> 16-byte slot j*64 + lane = (row slot / 8, position slot % 8),
        // which holds the row's piece position ^ ((row / 2) % 8)
        uint32_t al_off[4], al_k[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int slot = j * 64 + lane, rowl = slot >> 3, piece = (slot & 7) ^ ((rowl >> 1) & 7);
            al_k[j] = 4u * (uint32_t)piece;
            al_off[j] = m0 + rowl < p.K ? ((uint32_t)(m0 + rowl) * (uint32_t)p.CRS + al_k[j]) * 4u : kOutOfRange;
        }
        auto request_rows = [&](int stage, int t) __attribute__((always_inline)) {   // the four steps from step t on
            const uint32_t k0 = (uint32_t)t * 8u;
#pragma unroll
            for (int j = 0; j < 4; ++j)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(
                    wbuf, (__attribute__((address_space(3))) void *)(a_lds + stage * Cfg::A_STAGE_BYTES + j * 1024), 16,
                    k0 + al_k[j] < (uint32_t)p.CRS ? al_off[j] : kOutOfRange, k0 * 4u, 0, 0);
        };
        // this lane's operand of step i (0..3) of a stage: piece 2 i + half of row lane % 32
        const int fr_base = l32 * 128, fr_x = (l32 >> 1) & 7;
        auto read_rows = [&](int stage, int i) __attribute__((always_inline)) -> u32x4 {
            return *reinterpret_cast<const u32x4 *>(a_lds + stage * Cfg::A_STAGE_BYTES + fr_base + (((2 * i + half) ^ fr_x) << 4));
        };
        static_assert(D == 4, "four register sets of gathered elements: one per step of a copy");
        request_rows(0, t0);
        request_rows(1, t0 + 4);
        read_table(t0, 0);
        static_for<D>([&](auto dc) {
            constexpr int set = decltype(dc)::value;
#pragma unroll
            for (int e = 0; e < 4; ++e) request_b(set, 0, e);
            read_table(t0 + set + 1, 0);
        });
        // (the first copy has arrived when at most the second and the 16 gathers requested after it are outstanding)
        asm volatile("s_waitcnt vmcnt(20)" ::: "memory");
        u32x4 frag = read_rows(0, 0);
        __builtin_amdgcn_sched_barrier(0);
        for (int s = 0; s < steps_w; s += 8) {
            static_for<8>([&](auto sc) {
                constexpr int st = decltype(sc)::value, stage = st / 4, i = st % 4, set = st % 4;
                const int t = t0 + s + st;
                u32x4 next;
                if constexpr (i < 3) {
                    next = read_rows(stage, i + 1);
                } else {
                    // the other stage's copy was requested a whole copy ago; since then: the gathers of three steps
                    asm volatile("s_waitcnt vmcnt(12)" ::: "memory");
                    next = read_rows(stage ^ 1, 0);
                }
                const f32x4 va = __builtin_bit_cast(f32x4, frag);
                static_for<4>([&](auto ec) {
                    constexpr int e = decltype(ec)::value;
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(va[e], __builtin_bit_cast(float, b_reg[set][0][e]), acc, 0, 0, 0);
                    request_b(set, 0, e);
                    if constexpr (e == 3) read_table(t + D + 1, 0);
                    __builtin_amdgcn_sched_barrier(0);
                });
                frag = next;
                if constexpr (i == 3) {
                    // this stage has been read to its end (its last operand is in registers): the copy after next
                    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                    request_rows(stage, t + 5);
                    __builtin_amdgcn_sched_barrier(0);
                }
            });
        }
    }

    // the wavefronts' sums meet in LDS (the table is no longer needed): [wavefront][register][lane]
    if constexpr (Cfg::ALDS) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // (no copy may still be on its way into LDS)
    __syncthreads();
    float *const xch = reinterpret_cast<float *>(lds);
#pragma unroll
    for (int v = 0; v < 16; ++v) xch[(wave * 16 + v) * 64 + lane] = acc[v];
    __syncthreads();
    const __amdgpu_buffer_rsrc_t ybuf = __builtin_amdgcn_make_buffer_rsrc(p.y, 0, p.y_bytes, kBufferWord3);
    const bool fused = p.bias != nullptr || p.act >= 0;
#pragma unroll
    for (int i = 0; i < 1024 / THREADS; ++i) {
        // register v of lane l holds row 8*(v/4) + 4*(l/32) + v%4, column l%32 of the tile
        const int val = tid + i * THREADS;
        const int v = val >> 6, l = val & 63;
        float sum = xch[v * 64 + l];
        for (int w = 1; w < W; ++w) sum += xch[(w * 16 + v) * 64 + l];
        const int orow = m0 + 8 * (v >> 2) + 4 * (l >> 5) + (v & 3);
        const int ocol = n0 + (l & 31);
        if (orow >= p.K || ocol >= p.NPQ) continue;
        const uint32_t n = magic_div((uint32_t)ocol, p.mPQ);
        const uint32_t rem = (uint32_t)ocol - n * (uint32_t)p.PQ;
        const uint32_t pp = magic_div(rem, p.mQ);
        const uint32_t qq = rem - pp * (uint32_t)p.Q;
        const uint32_t off = (n * (uint32_t)p.ysN + pp * (uint32_t)p.ysP + qq * (uint32_t)p.ysQ + (uint32_t)orow * (uint32_t)p.ysK) * 4u;
        float out = p.alpha * sum;
        if (p.beta != 0.f) out += p.beta * __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(ybuf, off, 0, 0));
        if (fused) {
            if (p.bias != nullptr) out += p.bias[orow];
            if (p.act == 0) out = 1.f / (1.f + __expf(-out));                   // sigmoid
            else if (p.act == 1) out = fmaxf(out, 0.f);                         // rectified linear
            else if (p.act == 2) out = 1.f - 2.f / (__expf(2.f * out) + 1.f);   // tanh
        }
        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, out), ybuf, off, 0, 0);
    }
#endif
}

}  // namespace igc
#endif
