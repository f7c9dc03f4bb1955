// Implicit-GEMM convolution forward kernel for gfx950 (CDNA4), generic over tensor
// strides.  Paper, Section 3.1: the convolution is the matrix product
//   O_m (K x NPQ) = F_m (K x CRS) . D_m (CRS x NPQ)
// where D_m, the lowered input, is never stored in off-chip memory: each workgroup
// forms BK x BN tiles of it in LDS straight from the input tensor, using the map
// column j -> (n,p,q), row i -> (c,r,s) and the accessing function of eq. 2, and
// feeds them with BM x BK tiles of F_m to an MFMA microkernel.  The next tiles are
// fetched from HBM while the current ones are multiplied (two LDS stages).  The
// epilogue applies alpha/beta and stores through y's strides (the "transposition
// to the user's layout").
//
// Work split inside a 256-thread workgroup (4 wavefronts of 64):
//  * gather of the D_m tile: lane = column j (coalesced along q for NCHW inputs),
//    each wavefront owns a run of KPT consecutive reduction indices, so the
//    (c,r,s) decode and the tap offset live in scalar registers;
//  * the F_m tile is a contiguous read of filter rows;
//  * MFMA: wave (wm, wn) owns a (BM/WM) x (BN/WN) block of the output tile, made of
//    32x32 MFMA blocks (v_mfma_f32_32x32x2_f32 or v_mfma_f32_32x32x16_bf16).
// LDS tiles are stored [row][k] with k contiguous and a row stride of BK plus 16
// bytes: a lane reads 16 bytes of k for its row, which is bank-conflict free because
// the stride is an odd multiple of 16 bytes.  Which k a lane feeds to which MFMA is
// a free choice as long as both operands agree (the sum over k commutes).
//
// Every global access goes through a buffer descriptor limited to the tensor's
// extent; an element that must read as zero (zero border of eq. 3, tile tails) is
// requested at an out-of-range offset, which the hardware returns as 0.
#ifndef IGCONV_KERNEL_HPP_
#define IGCONV_KERNEL_HPP_

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>
#include <utility>

#include "igconv_params.h"

namespace igc {

using f32x16 = float __attribute__((ext_vector_type(16)));
using f32x4 = float __attribute__((ext_vector_type(4)));
using u32x4 = uint32_t __attribute__((ext_vector_type(4)));
using bf16x8 = __bf16 __attribute__((ext_vector_type(8)));
using u16x2 = uint16_t __attribute__((ext_vector_type(2)));

constexpr uint32_t kBufferWord3 = 0x00020000u;  // raw buffer, 32-bit data format
constexpr uint32_t kOutOfRange = 0x80000000u;   // >= any extent this library accepts

// Compile-time loop: f(std::integral_constant<int, I>) for I = 0..N-1, so that every
// index below is a constant (register arrays stay in registers, schedule tests fold).
template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, I...>) {
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F &&f) {
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

__device__ __forceinline__ uint32_t magic_div(uint32_t n, Magic m) {
    return (__umulhi(n, m.mul) + n) >> m.shift;
}

// How the reduction index is ordered and how the gather of the D_m tile finds, for one
// element (column j, index i), the offset of x[n,c,h,w] and whether the tap lies inside
// the image.  What was measured on this chip and shapes these modes: fp32 MFMA and
// ordinary vector instructions do not overlap (every vector instruction in the loop is
// taken from the MFMA rate), a register move through the GPR index costs about 40
// cycles, while scalar instructions and buffer loads whose address is a fixed vector
// register plus a scalar offset cost nothing next to the MFMAs.
enum GatherMode {
    // i = (c,r,s) in filter order; window test per element on packed 16-bit coordinates
    // (about 7 vector instructions per element).  Any R, S, pad.
    GATHER_GENERIC = 0,
    // i = (channel chunk, tap, channel in chunk): a step covers ONE tap and BK
    // consecutive channels, so the per-column offset and window test are computed once
    // per step and each element is one load with a scalar channel offset.  Any R, S,
    // pad; steps = R*S*ceil(C/BK), so it wants C to fill a chunk.
    GATHER_TAPMAJOR = 1,
    // i = (c,r,s) in filter order, pad_h = pad_w = 0: every tap of a valid column is
    // inside the image, the whole tap offset is a scalar.  For small C.
    GATHER_NOPAD = 2
};

template <bool BF16_, int BM_, int BN_, int BK_, int WM_, int WN_, bool SWAP_, bool VECA_, int GMODE_ = GATHER_GENERIC>
struct KernelConfig {
    static constexpr int GMODE = GMODE_;
    static constexpr bool BF16 = BF16_;
    static constexpr int BM = BM_, BN = BN_, BK = BK_, WM = WM_, WN = WN_;
    static constexpr bool SWAP = SWAP_;  // lanes run along output channels in the epilogue
    static constexpr bool VECA = VECA_;  // filter rows fetched with 16-byte loads
    static constexpr int THREADS = 256;
    static constexpr int ESIZE = BF16 ? 2 : 4;
    static constexpr int VEC = 16 / ESIZE;           // elements per 16-byte LDS access
    static constexpr int KG = 2 * VEC;               // reduction elements per k-group
    static constexpr int LD = BK + VEC;              // LDS row stride in elements
    static constexpr int A_ELEMS = BM * LD, B_ELEMS = BN * LD;
    static constexpr int LDS_BYTES = 2 * (A_ELEMS + B_ELEMS) * ESIZE;
    static constexpr int TM = BM / WM, TN = BN / WN; // per-wave output block
    static constexpr int MB = TM / 32, NB = TN / 32; // 32x32 MFMA blocks per wave
    static constexpr int CG = BN / 64;               // column groups of 64 lanes
    static constexpr int KPARTS = 4 / CG;            // wavefronts sharing one column group
    static constexpr int KPT = BK / KPARTS;          // reduction indices gathered per thread
    static_assert(WM * WN == 4, "four wavefronts per workgroup");
    static_assert(BM % (32 * WM) == 0 && BN % (32 * WN) == 0, "wave blocks are 32x32 multiples");
    static_assert(BN == 64 || BN == 128 || BN == 256, "column tile is 1, 2 or 4 wavefronts wide");
    static_assert(BK % KG == 0 && KPT % VEC == 0, "k tile granularity");
    static_assert(VECA ? (BM * (BK / VEC)) % THREADS == 0 : (BM * BK) % THREADS == 0, "filter tile split");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget");
    static_assert(!(GMODE == GATHER_TAPMAJOR && VECA), "tap-major filter reads are strided, never 16-byte");
};

template <class Cfg>
__global__ __launch_bounds__(256) void igconv_fwd_kernel(const ConvKernelParams p) {
    constexpr int BM = Cfg::BM, BN = Cfg::BN, BK = Cfg::BK, LD = Cfg::LD;
    constexpr int VEC = Cfg::VEC, KG = Cfg::KG, ES = Cfg::ESIZE;
    constexpr int MB = Cfg::MB, NB = Cfg::NB, KPT = Cfg::KPT;
    using elem_t = typename std::conditional<Cfg::BF16, uint16_t, float>::type;

    __shared__ __attribute__((aligned(16))) elem_t lds[2 * (Cfg::A_ELEMS + Cfg::B_ELEMS)];
    elem_t *const ldsA = lds;                       // [2][BM][LD]
    elem_t *const ldsB = lds + 2 * Cfg::A_ELEMS;    // [2][BN][LD]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5;   // which half of the k-group this lane feeds
    const int l32 = lane & 31;

    // M tiles are adjacent in launch order so that workgroups sharing the same
    // columns of D_m run at the same time.
    const int tile_m = blockIdx.x % p.tilesM;
    const int tile_n = blockIdx.x / p.tilesM;
    const int m0 = tile_m * BM;
    const int n0 = tile_n * BN;

    const __amdgpu_buffer_rsrc_t xbuf = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p.x), 0, p.x_bytes, kBufferWord3);
    const __amdgpu_buffer_rsrc_t wbuf = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p.w), 0, p.w_bytes, kBufferWord3);
    const __amdgpu_buffer_rsrc_t ybuf = __builtin_amdgcn_make_buffer_rsrc(p.y, 0, p.y_bytes, kBufferWord3);

    // ---- gather role: this lane's column j -> (n,p,q) (loop invariant) ------------
    // hw0 packs (p*u - pad_h, q*v - pad_w) as two 16-bit fields (two's complement);
    // adding a packed tap (tr, ts) gives the input coordinates of that tap, and the
    // tap is inside the image iff both fields are <= (H-1, W-1) as unsigned 16-bit
    // numbers (the host limits H, W and pad to 2^14, so a coordinate left of / above
    // the image wraps to >= 0xC000 and nothing wraps back into range).
    const int cg = wave % Cfg::CG;
    const int kpart = wave / Cfg::CG;
    const int jl = cg * 64 + lane;
    u16x2 hw0;
    uint32_t colbase_b;  // byte offset of x[n, 0, p*u - pad_h, q*v - pad_w] (mod 2^32)
    {
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
            hw0[1] = 0x8000;           // no tap of a column beyond NPQ is ever in range
        }
    }
    u16x2 hw_max;
    hw_max[1] = (uint16_t)(p.H - 1);
    hw_max[0] = (uint16_t)(p.W - 1);
    // GATHER_NOPAD: the window origin of a valid column, else the out-of-range marker.
    const uint32_t vcol = hw0[1] == 0x8000 ? kOutOfRange : colbase_b;

    // ---- filter-tile role ----------------------------------------------------------
    constexpr int A_PASSES = Cfg::VECA ? (BM * (BK / VEC)) / 256 : (BM * BK) / 256;
    constexpr int A_ROWS_PER_PASS = Cfg::VECA ? 256 / (BK / VEC) : 256 / BK;
    const int a_row = Cfg::VECA ? tid / (BK / VEC) : tid / BK;
    const int a_kk = Cfg::VECA ? (tid % (BK / VEC)) * VEC : tid % BK;

    // Registers holding the tiles in flight between HBM and LDS: two sets, tile T uses
    // set T&1, so that the loads of tile t+2 can be issued while tile t+1 still waits
    // in the other set to be written to LDS.
    u32x4 a_vec[2][Cfg::VECA ? A_PASSES : 1];
    elem_t a_sca[2][Cfg::VECA ? 1 : A_PASSES];
    elem_t b_val[2][KPT];
    // GATHER_GENERIC: per-lane decode of reduction index (first index of this
    // wavefront's run) + lane: byte offset of the tap relative to the window origin, and
    // the packed tap (tr,ts).
    uint32_t dec_il = 0, dec_c = 0, dec_rs = 0, dec_delta = 0, dec_tap = 0;
    // GATHER_NOPAD: reduction index of the next element to gather; GATHER_TAPMAJOR:
    // first channel of the step's chunk, the step's tap, and whether the step exists.
    // All wavefront-uniform, kept (with everything derived from them) in scalar registers.
    uint32_t sc_i = 0, sc_c0 = 0, sc_tr = 0, sc_ts = 0, sc_asoff = 0;
    bool sc_live = false;
    int sc_tau = 0;
    // GATHER_TAPMAJOR: this column's offset for the step's tap, or the out-of-range
    // marker when the tap falls in the zero border.
    uint32_t vtap = kOutOfRange;

    // F_m tile: rows m0.., the step's reduction indices; zero beyond K and beyond the
    // reduction range.  The per-thread part of the offset is fixed, the step's part is a
    // scalar.  Natural order: index k0 + a_kk of row `row`.  Tap-major: channel
    // c0 + a_kk, tap of the step, i.e. a read with stride R*S elements.
    uint32_t a_voff[A_PASSES];
#pragma unroll
    for (int ps = 0; ps < A_PASSES; ++ps) {
        const int row = m0 + a_row + ps * A_ROWS_PER_PASS;
        const uint32_t col = Cfg::GMODE == GATHER_TAPMAJOR ? (uint32_t)a_kk * (uint32_t)p.RS : (uint32_t)a_kk;
        a_voff[ps] = row < p.K ? ((uint32_t)row * (uint32_t)p.CRS + col) * ES : kOutOfRange;
    }
    // Start of the load of tile number tau (reduction step tau).
    auto decode1 = [&](int tau) {
        if constexpr (Cfg::GMODE == GATHER_GENERIC) {
            // i -> (c,r,s): lane L decodes index i0+L once for everybody, in two halves
            // so that each fits between two MFMAs
            dec_il = (uint32_t)(tau * BK + kpart * KPT) + (uint32_t)lane;
            dec_c = magic_div(dec_il, p.mRS);
            dec_rs = dec_il - dec_c * (uint32_t)p.RS;
        } else if constexpr (Cfg::GMODE == GATHER_NOPAD) {
            // (readfirstlane states the wavefront-uniformity for the compiler)
            sc_i = __builtin_amdgcn_readfirstlane((uint32_t)(tau * BK + kpart * KPT));
        } else {
            const uint32_t ut = __builtin_amdgcn_readfirstlane((uint32_t)tau);
            sc_tau = (int)ut;
            const uint32_t cc = magic_div(ut, p.mRS);     // channel chunk
            const uint32_t tap = ut - cc * (uint32_t)p.RS;  // r*S+s
            const uint32_t r = magic_div(tap, p.mS);
            const uint32_t sx = tap - r * (uint32_t)p.S;
            sc_tr = p.flip ? (uint32_t)p.R - 1u - r : r;   // eq. 2 inverts the filter
            sc_ts = p.flip ? (uint32_t)p.S - 1u - sx : sx;
            sc_c0 = cc * BK;
            sc_live = tau < p.ksteps;
            sc_asoff = sc_live ? (sc_c0 * (uint32_t)p.RS + tap) * ES : 0u;
        }
    };
    auto decode2 = [&]() {
        if constexpr (Cfg::GMODE == GATHER_GENERIC) {
            const uint32_t r = magic_div(dec_rs, p.mS);
            const uint32_t sx = dec_rs - r * (uint32_t)p.S;
            const uint32_t tr = p.flip ? (uint32_t)p.R - 1u - r : r;
            const uint32_t ts = p.flip ? (uint32_t)p.S - 1u - sx : sx;
            dec_delta = (dec_c * (uint32_t)p.xsC + tr * (uint32_t)p.xsH + ts * (uint32_t)p.xsW) * ES;
            dec_tap = dec_il < (uint32_t)p.CRS ? ((tr << 16) | ts) : 0x80000000u;  // i >= CRS: never in range
        } else if constexpr (Cfg::GMODE == GATHER_TAPMAJOR) {
            const u16x2 tap = __builtin_bit_cast(u16x2, (sc_tr << 16) | sc_ts);
            const u16x2 hw = hw0 + tap;
            const u16x2 cl = __builtin_elementwise_min(hw, hw_max);
            const bool ok = __builtin_bit_cast(uint32_t, cl) == __builtin_bit_cast(uint32_t, hw);
            vtap = ok ? colbase_b + (sc_tr * (uint32_t)p.xsH + sc_ts * (uint32_t)p.xsW) * ES : kOutOfRange;
            // When C is not a multiple of BK the last channel chunk is ragged: on
            // entering it (once per tile; the chunks are the outer order) the filter
            // offsets of the channels beyond C are replaced by the out-of-range marker.
            if (sc_tau == p.tail_step) {
#pragma unroll
                for (int ps = 0; ps < A_PASSES; ++ps)
                    a_voff[ps] = sc_c0 + (uint32_t)a_kk < (uint32_t)p.C ? a_voff[ps] : kOutOfRange;
            }
        }
    };
    // A buffer descriptor that reads as zeros everywhere when `live` is false.  (The
    // scalar offset of a load takes part in the hardware range check as "limit - scalar",
    // so a dead load must also use scalar offset 0, and a live one never exceeds the
    // extent.)
    auto rsrc_if = [&](const void *ptr, uint32_t bytes, bool live) {
        return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(ptr), 0, live ? bytes : 0u, kBufferWord3);
    };
    auto load_a = [&](int set, int tau, int ps) {
        uint32_t voffa, soff;
        bool live = true;
        if constexpr (Cfg::GMODE == GATHER_TAPMAJOR) {
            voffa = a_voff[ps];  // (channels beyond C: masked in place by decode2)
            soff = sc_asoff;
            live = sc_live;
        } else {
            const int k0 = tau * BK;
            voffa = k0 + a_kk < p.CRS ? a_voff[ps] : kOutOfRange;
            soff = k0 < p.CRS ? (uint32_t)k0 * ES : 0u;
        }
        const __amdgpu_buffer_rsrc_t wb = Cfg::GMODE == GATHER_TAPMAJOR ? rsrc_if(p.w, p.w_bytes, live) : wbuf;
        if constexpr (Cfg::VECA) {
            a_vec[set][ps] = __builtin_amdgcn_raw_buffer_load_b128(wb, voffa, soff, 0);
        } else if constexpr (Cfg::BF16) {
            a_sca[set][ps] = __builtin_amdgcn_raw_buffer_load_b16(wb, voffa, soff, 0);
        } else {
            a_sca[set][ps] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(wb, voffa, soff, 0));
        }
    };
    // D_m tile, element e of this lane's column.
    auto load_b = [&](int set, int e) {
        uint32_t vo, so;
        bool live = true;
        if constexpr (Cfg::GMODE == GATHER_GENERIC) {
            // takes lane e's decode as scalars
            const uint32_t d = __builtin_amdgcn_readlane(dec_delta, e);
            const u16x2 tap = __builtin_bit_cast(u16x2, (uint32_t)__builtin_amdgcn_readlane(dec_tap, e));
            const u16x2 hw = hw0 + tap;
            const u16x2 cl = __builtin_elementwise_min(hw, hw_max);
            const bool ok = __builtin_bit_cast(uint32_t, cl) == __builtin_bit_cast(uint32_t, hw);
            vo = ok ? colbase_b + d : kOutOfRange;
            so = 0;
        } else if constexpr (Cfg::GMODE == GATHER_TAPMAJOR) {
            // fixed vector offset for the whole step, channel offset as a scalar
            const uint32_t c = sc_c0 + (uint32_t)(kpart * KPT + e);
            live = sc_live && (int)c < p.C;
            vo = vtap;
            so = live ? c * (uint32_t)p.xsC * ES : 0u;
        } else {
            // scalar decode of the running index: the whole tap offset is a scalar
            const uint32_t c = magic_div(sc_i, p.mRS);
            const uint32_t rs = sc_i - c * (uint32_t)p.RS;
            const uint32_t r = magic_div(rs, p.mS);
            const uint32_t sx = rs - r * (uint32_t)p.S;
            const uint32_t tr = p.flip ? (uint32_t)p.R - 1u - r : r;
            const uint32_t ts = p.flip ? (uint32_t)p.S - 1u - sx : sx;
            live = (int)c < p.C;
            ++sc_i;
            vo = vcol;
            so = live ? (c * (uint32_t)p.xsC + tr * (uint32_t)p.xsH + ts * (uint32_t)p.xsW) * ES : 0u;
        }
        const __amdgpu_buffer_rsrc_t xb = Cfg::GMODE == GATHER_GENERIC ? xbuf : rsrc_if(p.x, p.x_bytes, live);
        if constexpr (Cfg::BF16) {
            b_val[set][e] = __builtin_amdgcn_raw_buffer_load_b16(xb, vo, so, 0);
        } else {
            b_val[set][e] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(xb, vo, so, 0));
        }
    };
    auto write_a = [&](int set, int buf, int ps) {
        elem_t *const A = ldsA + buf * Cfg::A_ELEMS;
        const int row = a_row + ps * A_ROWS_PER_PASS;
        if constexpr (Cfg::VECA) {
            *reinterpret_cast<u32x4 *>(A + row * LD + a_kk) = a_vec[set][ps];
        } else {
            A[row * LD + a_kk] = a_sca[set][ps];
        }
    };
    // 16-byte chunk q of this lane's run of the D_m tile.
    auto write_b = [&](int set, int buf, int q) {
        elem_t *const dst = ldsB + buf * Cfg::B_ELEMS + jl * LD + kpart * KPT + q * VEC;
        u32x4 v;
        if constexpr (Cfg::BF16) {
#pragma unroll
            for (int d = 0; d < 4; ++d)
                v[d] = (uint32_t)b_val[set][q * VEC + 2 * d] | ((uint32_t)b_val[set][q * VEC + 2 * d + 1] << 16);
        } else {
#pragma unroll
            for (int d = 0; d < 4; ++d) v[d] = __builtin_bit_cast(uint32_t, b_val[set][q * VEC + d]);
        }
        *reinterpret_cast<u32x4 *>(dst) = v;
    };

    // Moving one tile is a list of small items: NL load items (decode halves, filter
    // loads, gathered elements) and NW LDS-write items.
    constexpr int NW_A = A_PASSES, NW_B = KPT / VEC, NW = NW_A + NW_B;
    constexpr int NL = 2 + A_PASSES + KPT;
    auto load_item = [&](int i, int set, int tau) {
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

    constexpr int G = BK / KG;                          // k-groups per step
    constexpr int EPG = Cfg::BF16 ? 1 : 4;              // MFMAs per (block, k-group)
    constexpr int MPG = EPG * MB * NB;                  // MFMAs per k-group
    constexpr int NM = G * MPG;                         // MFMAs per step
    static_assert(G % 2 == 0, "operand fragments alternate between two register sets");
    constexpr int SB = (G - 1) * MPG;                   // the step's barrier sits before MFMA number SB
    // Operand fragments: 16 bytes of k per lane and 32-row block, two sets (k-group
    // parity) so that the next group's fragments load while this group multiplies.
    u32x4 fragA[2][MB], fragB[2][NB];
    const int fa_off = (wm * Cfg::TM + l32) * LD + half * VEC;
    const int fb_off = (wn * Cfg::TN + l32) * LD + half * VEC;
    auto read_frags = [&](int buf, int g) {
        const elem_t *const A = ldsA + buf * Cfg::A_ELEMS + fa_off + g * KG;
        const elem_t *const B = ldsB + buf * Cfg::B_ELEMS + fb_off + g * KG;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) fragA[g & 1][mb] = *reinterpret_cast<const u32x4 *>(A + mb * 32 * LD);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) fragB[g & 1][nb] = *reinterpret_cast<const u32x4 *>(B + nb * 32 * LD);
    };
    // MFMA number j of k-group g.  Consecutive MFMAs go to different accumulators.
    auto mfma = [&](int g, int j) {
        const int e = j / (MB * NB), mb = (j / NB) % MB, nb = j % NB;
        if constexpr (Cfg::BF16) {
            const bf16x8 fa = __builtin_bit_cast(bf16x8, fragA[g & 1][mb]);
            const bf16x8 fb = __builtin_bit_cast(bf16x8, fragB[g & 1][nb]);
            if constexpr (Cfg::SWAP)
                acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb, fa, acc[mb][nb], 0, 0, 0);
            else
                acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, acc[mb][nb], 0, 0, 0);
        } else {
            // (whole-vector casts: a bit_cast applied to a single vector element reads
            // element 0 with this compiler)
            const f32x4 va = __builtin_bit_cast(f32x4, fragA[g & 1][mb]);
            const f32x4 vb = __builtin_bit_cast(f32x4, fragB[g & 1][nb]);
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

    // ---- main loop ----------------------------------------------------------------------
    // Software pipeline over the reduction steps t = 0..T-1 (Section 3.1: compute on the
    // current tiles while the next ones are fetched).  During step t, which multiplies
    // LDS stage t&1:
    //   * the loads of tile t+2 are issued into register set t&1, one item per MFMA;
    //   * tile t+1, requested a whole step earlier into the other set, is written to
    //     LDS stage (t+1)&1 in the slots just before the barrier;
    //   * before the last k-group the workgroup synchronises and the first fragments of
    //     step t+1 are read, so the MFMA pipe never waits for LDS.
    // The order is pinned with scheduling barriers: one short burst of side work, one
    // MFMA.  Tiles beyond the last step read as zeros (out-of-range requests), so no
    // step is special; the loop is unrolled by two because the register set and the LDS
    // stage alternate.
    auto step = [&](auto parity, int t) {
        constexpr int cur = decltype(parity)::value, nxt = cur ^ 1;
        const int k2 = t + 2;  // number of the tile requested during this step
        static_for<NM>([&](auto mc) {
            constexpr int m = decltype(mc)::value;
            constexpr int g = m / MPG, j = m % MPG;
            if constexpr (j == 0 && g + 1 < G) read_frags(cur, g + 1);
            if constexpr (m == SB) {
                lds_barrier();
                read_frags(nxt, 0);
            }
            // load items i with floor(i * NM / NL) == m: tile t+2 -> set cur
            constexpr int l0 = (m * NL + NM - 1) / NM, l1 = ((m + 1) * NL + NM - 1) / NM;
            static_for<l1 - l0>([&](auto ic) { load_item(l0 + decltype(ic)::value, cur, k2); });
            // write items, packed into the slots before the barrier: tile t+1, set nxt -> stage nxt
            constexpr int WS = NW < SB ? NW : SB;   // slots used for writes
            if constexpr (m >= SB - WS && m < SB) {
                constexpr int q = m - (SB - WS);
                constexpr int w0 = (q * NW + WS - 1) / WS, w1 = ((q + 1) * NW + WS - 1) / WS;
                static_for<w1 - w0>([&](auto ic) { write_item(w0 + decltype(ic)::value, nxt, nxt); });
            }
            mfma(g, j);
            __builtin_amdgcn_sched_barrier(0);
        });
    };

    const int ksteps = p.ksteps;
    static_for<NL>([&](auto ic) { load_item(decltype(ic)::value, 0, 0); });
    static_for<NW>([&](auto ic) { write_item(decltype(ic)::value, 0, 0); });
    static_for<NL>([&](auto ic) { load_item(decltype(ic)::value, 1, 1); });
    lds_barrier();
    read_frags(0, 0);
    // Enter the loop with no load outstanding: otherwise the compiler, merging this path
    // with the loop's back edge, waits for every load at the top of each step.
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
    __builtin_amdgcn_sched_barrier(0);
    // (always whole pairs of steps - an odd count runs one extra step on zero tiles - so
    // that the loop body stays a single basic block)
    for (int t = 0; t < ksteps; t += 2) {
        step(std::integral_constant<int, 0>{}, t);
        step(std::integral_constant<int, 1>{}, t + 1);
    }

    // ---- epilogue: alpha/beta, store through y's strides ---------------------------------
    // A 32x32 MFMA result block keeps, in lane l, register v, the element
    //   (row 8*(v/4) + 4*(l/32) + v%4, column l%32).
    // Without SWAP rows are output channels and columns are pixels; with SWAP the
    // operands were exchanged, so columns (lanes) are channels and rows are pixels.
    const bool use_beta = p.beta != 0.f;
    auto pixel_offset = [&](int j, bool &valid) -> uint32_t {
        valid = j < p.NPQ;
        const uint32_t jj = valid ? (uint32_t)j : 0u;
        const uint32_t n = magic_div(jj, p.mPQ);
        const uint32_t rem = jj - n * (uint32_t)p.PQ;
        const uint32_t pp = magic_div(rem, p.mQ);
        const uint32_t qq = rem - pp * (uint32_t)p.Q;
        return n * (uint32_t)p.ysN + pp * (uint32_t)p.ysP + qq * (uint32_t)p.ysQ;
    };
    auto emit = [&](float a, uint32_t off, bool valid) {
        const uint32_t voff = valid ? off * 4u : kOutOfRange;
        float out = p.alpha * a;
        if (use_beta) {
            const float old = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(ybuf, voff, 0, 0));
            out += p.beta * old;
        }
        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, out), ybuf, voff, 0, 0);
    };
    if constexpr (!Cfg::SWAP) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            bool pv;
            const uint32_t poff = pixel_offset(n0 + wn * Cfg::TN + nb * 32 + l32, pv);
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int k = m0 + wm * Cfg::TM + mb * 32 + 8 * (v / 4) + 4 * half + (v % 4);
                    emit(acc[mb][nb][v], poff + (uint32_t)k * (uint32_t)p.ysK, pv && k < p.K);
                }
            }
        }
    } else {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            const int k = m0 + wm * Cfg::TM + mb * 32 + l32;
            const bool kv = k < p.K;
            const uint32_t koff = (uint32_t)k * (uint32_t)p.ysK;
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    bool pv;
                    const uint32_t poff = pixel_offset(n0 + wn * Cfg::TN + nb * 32 + 8 * (v / 4) + 4 * half + (v % 4), pv);
                    emit(acc[mb][nb][v], poff + koff, pv && kv);
                }
            }
        }
    }
}

}  // namespace igc
#endif
