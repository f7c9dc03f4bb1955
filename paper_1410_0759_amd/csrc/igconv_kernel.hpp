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
// bytes, an odd multiple of 16: a lane reads 16 bytes of k for its row, and 16
// consecutive rows then start in 16 different groups of four banks, so the fragment
// reads and the D_m writes (lane = row) of 16 lanes meet no conflict.  The F_m writes
// do: they put 8 lanes (32 for element-wise loads) along one row, 128 contiguous
// bytes, and the next row starts 144 bytes on, i.e. four banks into the first row's
// wrap - a two-way conflict on those banks.  The counters agree that conflicts exist
// (SQ_LDS_BANK_CONFLICT / SQ_LDS_IDX_ACTIVE: 17 % on the first-layer workload, 25 %
// and 33 % on the two 3x3 ones), while LDS is active 14-28 % of the time: not what
// bounds these kernels.  Which k a lane feeds to which MFMA is a free choice as long
// as both operands agree (the sum over k commutes).
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
using u32x2 = uint32_t __attribute__((ext_vector_type(2)));

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

// All-ones when a < b, else 0, for 0 <= a, b < 2^31, with integer arithmetic only.
// Wavefront-uniform conditions of the loop are applied as such masks (x & mask) rather
// than as c ? x : 0: a select may become a branch around the computation of x, and a
// branch would split the loop body into blocks, while the pipelined schedule (and the
// compiler's tracking of outstanding loads) relies on it being a single one.
__device__ __forceinline__ uint32_t mask_lt(uint32_t a, uint32_t b) {
    return (uint32_t)((int32_t)(a - b) >> 31);
}

__device__ __forceinline__ uint32_t magic_div(uint32_t n, Magic m) {
    return (__umulhi(n, m.mul) + n) >> m.shift;
}

// Epilogue shared by the kernels: out = alpha*acc (+ beta*y), stored through y's strides
// (Section 3.1: the final transposition to the user's layout; Section 2.1.1: accumulate
// mode).  `acc` holds MB x NB MFMA result blocks of 32x32; a block keeps, in lane l,
// register v, the element (row 8*(v/4) + 4*(l/32) + v%4, column l%32).  Without SWAP rows
// are output channels and columns are pixels (lanes run along pixels: contiguous for
// NCHW); with SWAP the MFMA operands were exchanged, so lanes run along output channels
// (contiguous for NHWC) and rows are pixels.  krow0 / col0: first output channel / first
// column (n,p,q) of this wavefront's blocks.  Whatever does not depend on the lane goes
// into the store's scalar offset where that is possible; a wavefront whose blocks lie
// fully inside K x NPQ needs no per-element test.  LINEAR: column j sits at j*ysQ.
// The 32 bias values of each row block of a wavefront's tile, one per lane (zero when no bias
// is given or the row lies beyond K).  Loaded well before the epilogue that uses them, so
// that the epilogue does not have to wait behind the loads already in flight for the next tile.
template <int MB>
__device__ __forceinline__ void load_bias(const ConvKernelParams &p, int krow0, int l32, float (&bvec)[MB]) {
    const __amdgpu_buffer_rsrc_t bbuf = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float *>(p.bias), 0, p.bias != nullptr ? (uint32_t)p.K * 4u : 0u, kBufferWord3);
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
        bvec[mb] = p.bias != nullptr ? __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(
                                            bbuf, (uint32_t)(krow0 + mb * 32 + l32) * 4u, 0, 0))
                                     : 0.f;
}

template <bool SWAP, int MB, int NB, bool LINEAR = false>
__device__ __forceinline__ void store_tile(const ConvKernelParams &p, __amdgpu_buffer_rsrc_t ybuf,
                                           f32x16 (&acc)[MB][NB], const float (&bvec)[MB], int krow0, int col0, int half,
                                           int l32) {
    const bool use_beta = p.beta != 0.f;
    // Fused tail (Section 2.2's bias addition and activation, applied while the result is
    // still in registers): out = f(alpha*acc + beta*y + bias[k]).  bvec holds the 32 bias
    // values of each row block, one per lane; where rows are spread over registers, the value
    // of a register's row comes from the lane that holds it.
    const bool fused = p.bias != nullptr || p.act >= 0;   // wavefront-uniform
    auto row_bias = [&](int mb, int v) -> float {   // bias of the row register v of block row mb holds in this lane
        if (!fused) return 0.f;
        const int r0 = 8 * (v / 4) + (v % 4);
        const float b0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, bvec[mb]), r0));
        const float b1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, bvec[mb]), r0 + 4));
        return half ? b1 : b0;
    };
    auto pixel_offset = [&](uint32_t j) -> uint32_t {  // element offset of column j = (n,p,q) in y
        if constexpr (LINEAR) return j * (uint32_t)p.ysQ;   // columns a fixed distance apart
        const uint32_t n = magic_div(j, p.mPQ);
        const uint32_t rem = j - n * (uint32_t)p.PQ;
        const uint32_t pp = magic_div(rem, p.mQ);
        const uint32_t qq = rem - pp * (uint32_t)p.Q;
        return n * (uint32_t)p.ysN + pp * (uint32_t)p.ysP + qq * (uint32_t)p.ysQ;
    };
    auto emit = [&](float a, uint32_t voff, uint32_t soff, float b) {
        float out = p.alpha * a;
        if (use_beta) {
            const float old = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(ybuf, voff, soff, 0));
            out += p.beta * old;
        }
        if (fused) {
            out += b;
            if (p.act == 0) out = 1.f / (1.f + __expf(-out));                   // sigmoid
            else if (p.act == 1) out = fmaxf(out, 0.f);                         // rectified linear
            else if (p.act == 2) out = 1.f - 2.f / (__expf(2.f * out) + 1.f);   // tanh
        }
        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, out), ybuf, voff, soff, 0);
    };
    if constexpr (!SWAP) {
        const bool full = krow0 + MB * 32 <= p.K && col0 + NB * 32 <= p.NPQ;  // wavefront-uniform
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            const int j = col0 + nb * 32 + l32;
            const bool pv = j < p.NPQ;
            const uint32_t poff = pixel_offset(pv ? (uint32_t)j : 0u);
            if (full) {
                // lane part: pixel and the row half; scalar part: the register's row
                const uint32_t vo = (poff + (uint32_t)(4 * half) * (uint32_t)p.ysK) * 4u;
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        emit(acc[mb][nb][v], vo, (uint32_t)(krow0 + mb * 32 + 8 * (v / 4) + (v % 4)) * (uint32_t)p.ysK * 4u, row_bias(mb, v));
            } else {
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int k = krow0 + mb * 32 + 8 * (v / 4) + 4 * half + (v % 4);
                        emit(acc[mb][nb][v], pv && k < p.K ? (poff + (uint32_t)k * (uint32_t)p.ysK) * 4u : kOutOfRange, 0u, row_bias(mb, v));
                    }
            }
        }
    } else {
        // Rows of a block are pixels here: 32 per block, decoded once, one per lane (both
        // halves of the wavefront decode the same 32); register v of a lane then belongs
        // to pixel 8*(v/4) + v%4 (+4 in the upper half), whose offset is fetched from the
        // lane that decoded it.  A pixel past the end carries the out-of-range marker,
        // which survives the addition of the channel offset (both stay below 2^31).
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            const int jd = col0 + nb * 32 + l32;
            const uint32_t pd = jd < p.NPQ ? pixel_offset((uint32_t)jd) * 4u : kOutOfRange;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                const int k = krow0 + mb * 32 + l32;
                const bool kv = k < p.K;
                const uint32_t koff = (uint32_t)k * (uint32_t)p.ysK * 4u;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int r0 = 8 * (v / 4) + (v % 4);
                    const uint32_t d0 = __builtin_amdgcn_readlane(pd, r0), d1 = __builtin_amdgcn_readlane(pd, r0 + 4);
                    emit(acc[mb][nb][v], kv ? koff + (half ? d1 : d0) : kOutOfRange, 0u, bvec[mb]);
                }
            }
        }
    }
}

// How the reduction index is ordered and how the gather of the D_m tile finds, for one
// element (column j, index i), the offset of x[n,c,h,w] and whether the tap lies inside
// the image.  What was measured on this chip and shapes these modes: fp32 MFMA and
// ordinary vector instructions do not overlap (every vector instruction in the loop is
// taken from the MFMA rate); a register move through the GPR index costs about 40
// cycles; a wavefront issues in order, so whatever sits between two MFMAs - scalar
// instructions included - must fit in the 64 cycles one MFMA takes (about ten
// instructions), or the MFMA pipe idles; a buffer load whose address is a fixed vector
// register plus a scalar offset is one instruction.  So every fast mode gathers an
// element with a load from a loop-invariant (or per-step) vector offset plus a scalar
// offset, and zero-fills by making that sum fall outside the buffer.
enum GatherMode {
    // i = (c,r,s) in filter order; window test per element on packed 16-bit coordinates
    // (about 7 vector instructions per element).  Any R, S, pad, C.
    GATHER_GENERIC = 0,
    // i = (channel chunk, tap, channel in chunk): a step covers ONE tap and BK
    // consecutive channels; the per-column offset and window test are computed once per
    // step.  Any R, S, pad; steps = R*S*ceil(C/BK), so it wants C to fill a chunk, and
    // its filter reads are strided.
    GATHER_TAPMAJOR = 1,
    // i = (c,r,s) in filter order, pad_h = pad_w = 0: every tap of a valid column is
    // inside the image, the whole tap offset is a scalar.  Any R, S, C.
    GATHER_NOPAD = 2,
    // i = (c,r,s) in filter order with R*S = 9 and C a multiple of 4: a step is four
    // whole channels (BK = 36), so which tap an element has never changes; the nine
    // per-column tap offsets (window test folded in) are built once per tile and the
    // loop holds no vector instruction at all.  Any pad, stride, mode.
    GATHER_TAPS9 = 3,
    // GATHER_NOPAD for short reductions: the per-index tap offsets are computed once per
    // workgroup into an LDS table (kOffsetTableEntries entries: every step the kernel can
    // request, the two steps the pipeline asks for past the end included), so that a step
    // fetches its offsets with one LDS read instead of decoding them with vector
    // instructions, which would stall the fp32 MFMA.
    GATHER_NOPAD_TABLE = 7,
    // The same for problems whose last reduction step holds at most half a step of real
    // indices (C*R*S mod BK in 1..BK/2, an even number of steps): that step runs only half of
    // its k-groups, the others would multiply zeros.
    GATHER_NOPAD_TABLE_SHORT = 11,
    // GATHER_NOPAD_TABLE for an odd number of steps: the loop runs pairs of steps, and the second
    // step of a tile's last pair, which would multiply zeros, does its side work only (requests
    // and LDS writes for the workgroup's next tile) and no MFMA.
    GATHER_NOPAD_TABLE_ODD = 13,
    // i = (c,r,s) in filter order with a zero border and at most 63 taps: the tap of the next element is
    // tracked by the scalar unit (its position in the window, its offset from the window origin and its bit
    // number advance with every gathered element by one of three precomputed steps: scalar instructions
    // issue beside the MFMAs), and whether it lies inside the image is one bit of a 64-bit mask per column,
    // built once per tile.  A gathered element then costs three vector instructions (shift the mask, add
    // the offset, merge the bit as the out-of-range marker) instead of the generic gather's seven, and none
    // that moves data between lanes; the filter is read in its own order (contiguous rows), or, for backward
    // data, through the row / reduction / tap strides with one decode per thread and step.
    GATHER_MASKED = 14,
    // Backward-filter: the generic gather with the roles of the two index sets exchanged.
    // Columns are filter elements (c,r,s), the reduction runs over output pixels (n,p,q);
    // the first operand is dy, read through its strides with a per-step decode of (n,p,q);
    // the reduction may be cut into several ranges, one workgroup each.  (Modes 6, 8 and 9 are
    // the kernel of igconv_kernel_wgrad.hpp.)
    GATHER_WGRAD = 6,
    // Backward-filter with the columns ordered (tap, channel) and one tap per tile: lanes run
    // along the reduction index (n,p,q) - consecutive pixels, coalesced loads - and decode it
    // once per step, window test included, since the tile's tap is a scalar; the elements of
    // a thread are channels, reached through a scalar offset.  No vector instruction per
    // gathered element.  Any R, S, pad, stride; wants C to fill a column tile.
    GATHER_WGRAD_TAP = 8,
    // Backward-filter without padding (every tap of every output pixel lies inside the image)
    // for few channels: lanes along the reduction index as above, columns in filter order
    // (c,r,s); each thread keeps the offsets of its columns in registers for the whole tile
    // and a gathered element costs one vector addition.
    GATHER_WGRAD_NOPAD = 9
};

constexpr int kOffsetTableEntries = 2048;

// TEAMS > 1: a workgroup of TEAMS x 256 threads - TEAMS teams of four wavefronts, each running the
// whole pipeline in its own part of LDS over its own range of the reduction steps; before the
// epilogue the other teams' accumulators are added to the first team's through LDS, in team
// order.  For problems with few tiles and long reductions, one tile per workgroup: the compute
// units get several wavefronts per SIMD (which cover each other's waits) and the idle ones work.
template <bool BF16_, int BM_, int BN_, int BK_, int WM_, int WN_, bool SWAP_, bool VECA_, int GMODE_ = GATHER_GENERIC,
          int TEAMS_ = 1>
struct KernelConfig {
    static constexpr int GMODE = GMODE_;
    static constexpr int TEAMS = TEAMS_;
    static constexpr bool BF16 = BF16_;
    static constexpr int BM = BM_, BN = BN_, BK = BK_, WM = WM_, WN = WN_;
    static constexpr bool SWAP = SWAP_;  // lanes run along output channels in the epilogue
    static constexpr bool VECA = VECA_;  // filter rows fetched with 16-byte loads
    static constexpr int THREADS = 256 * TEAMS_;
    static constexpr int ESIZE = BF16 ? 2 : 4;
    static constexpr int VEC = 16 / ESIZE;           // elements per 16-byte LDS access
    static constexpr int KG = 2 * VEC;               // reduction elements per full k-group
    // LDS row stride: at least BK plus 16 bytes, and an odd number of 16-byte units, so
    // that 16-byte accesses of 16 consecutive rows fall on distinct banks
    static constexpr int LDV = (BK / VEC + 1) | 1;
    static constexpr int LD = LDV * VEC;
    static constexpr int A_ELEMS = BM * LD, B_ELEMS = BN * LD;
    static constexpr int TABLE_BYTES =
        GMODE_ == GATHER_NOPAD_TABLE || GMODE_ == GATHER_NOPAD_TABLE_SHORT || GMODE_ == GATHER_NOPAD_TABLE_ODD ? kOffsetTableEntries * 4 : 0;
    static constexpr int TEAM_LDS_BYTES = 2 * (A_ELEMS + B_ELEMS) * ESIZE;
    static constexpr int LDS_BYTES = TEAMS_ * TEAM_LDS_BYTES + TABLE_BYTES;
    // Waves per SIMD the registers must allow: steps of 16 leave room (LDS, registers) for three workgroups per
    // compute unit; where LDS lets two share it the registers must too - left alone, the kernels with the
    // largest tiles take more than half of a SIMD's 512 and run one wave per SIMD.
    static constexpr int MIN_WAVES = TEAMS_ > 1 ? TEAMS_ : (BK_ == 16 ? 3 : (LDS_BYTES <= 80 * 1024 ? 2 : 1));
    static constexpr int TM = BM / WM, TN = BN / WN; // per-wave output block
    static constexpr int MB = TM / 32, NB = TN / 32; // 32x32 MFMA blocks per wave
    static constexpr int CG = BN / 64;               // column groups of 64 lanes
    static constexpr int KPARTS = 4 / CG;            // wavefronts sharing one column group
    static constexpr int KPT = BK / KPARTS;          // reduction indices gathered per thread
    static constexpr int REM = BK % KG;              // elements of a last, partial k-group
    static_assert(WM * WN == 4, "four wavefronts per workgroup");
    static_assert(BM % (32 * WM) == 0 && BN % (32 * WN) == 0, "wave blocks are 32x32 multiples");
    static_assert(BN == 64 || BN == 128 || BN == 256, "column tile is 1, 2 or 4 wavefronts wide");
    static_assert(BK % VEC == 0 && BK % KPARTS == 0 && KPT % 2 == 0, "k tile granularity");
    static_assert(REM == 0 || (!BF16 && REM == 4), "a partial k-group is half a group, fp32 only");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget");
    static_assert(TEAMS_ == 1 || ((GMODE_ == GATHER_NOPAD || GMODE_ == GATHER_TAPS9) && !BF16_ && BM_ * BN_ * 4 <= TEAM_LDS_BYTES),
                  "teams: fp32 kernels whose steps stand alone; a team's results pass through its LDS");
    static_assert(!(GMODE == GATHER_TAPMAJOR && VECA), "tap-major filter reads are strided, never 16-byte");
    static_assert(GMODE != GATHER_WGRAD && GMODE != GATHER_WGRAD_TAP && GMODE != GATHER_WGRAD_NOPAD,
                  "the backward-filter gathers have their own kernel (igconv_kernel_wgrad.hpp)");
    static_assert(GMODE != GATHER_TAPS9 || (BK % 9 == 0 && KPT % 9 == 0), "whole channels of nine taps per thread");
};

template <class Cfg>
__global__ __launch_bounds__(Cfg::THREADS, Cfg::MIN_WAVES) void igconv_fwd_kernel(const ConvKernelParams p) {
    constexpr int BM = Cfg::BM, BN = Cfg::BN, BK = Cfg::BK, LD = Cfg::LD;
    constexpr int VEC = Cfg::VEC, KG = Cfg::KG, ES = Cfg::ESIZE;
    constexpr int MB = Cfg::MB, NB = Cfg::NB, KPT = Cfg::KPT;
    constexpr bool SHORT_LAST = Cfg::GMODE == GATHER_NOPAD_TABLE_SHORT;
    constexpr bool ODD_LAST = Cfg::GMODE == GATHER_NOPAD_TABLE_ODD;
    constexpr int GM = SHORT_LAST || ODD_LAST ? (int)GATHER_NOPAD_TABLE : Cfg::GMODE;
    constexpr bool GEN = GM == GATHER_GENERIC;  // per-element window test
    constexpr bool NOPADX = GM == GATHER_NOPAD || GM == GATHER_NOPAD_TABLE;
    constexpr bool MSK = GM == GATHER_MASKED;
    constexpr bool MSK_STRIDED = MSK && !Cfg::VECA;   // filter through strides, one reduction index per thread
    using elem_t = typename std::conditional<Cfg::BF16, uint16_t, float>::type;

    __shared__ __attribute__((aligned(16))) elem_t lds[Cfg::TEAMS * 2 * (Cfg::A_ELEMS + Cfg::B_ELEMS)];
    // (teams: `tid` and `wave` count within the thread's team, whose LDS follows the previous team's)
    const int team = Cfg::TEAMS > 1 ? __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 8) : 0;
    elem_t *const ldsA = lds + team * 2 * (Cfg::A_ELEMS + Cfg::B_ELEMS);   // [2][BM][LD]
    elem_t *const ldsB = ldsA + 2 * Cfg::A_ELEMS;                          // [2][BN][LD]
    __shared__ uint32_t so_table[GM == GATHER_NOPAD_TABLE ? kOffsetTableEntries : 1];

    const int tid = threadIdx.x & 255;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5;   // which half of the k-group this lane feeds
    const int l32 = lane & 31;

    // Workgroups are dealt round-robin to the 8 XCDs, each with its own L2.  The tiles
    // are numbered with the M tiles of one column tile adjacent (they gather the same
    // columns of D_m) and cut into 8 contiguous ranges, one per XCD, so that the
    // workgroups which share input rows and columns also share an L2.  A workgroup is
    // persistent: it takes every wgsPerXcd-th tile of its XCD's range, and its pipeline
    // runs on across tile boundaries (see the main loop).
    const int wg_xcd = (int)(blockIdx.x % 8u), wg_local = (int)(blockIdx.x / 8u);
    const int tiles_mn = p.tilesM * p.tilesN;
    const int tiles_total = tiles_mn * p.splits;   // (splits >= 1; above 1 the tile numbers repeat once per range of the reduction)
    // number of this workgroup's i-th tile; tiles_total when it has no i-th tile
    auto tile_number = [&](int i) {
        const int local = wg_local + i * p.wgsPerXcd;
        const int t = wg_xcd * p.tilesPerXcd + local;
        return local < p.tilesPerXcd && t < tiles_total ? t : tiles_total;
    };
    if (tile_number(0) >= tiles_total) return;
    // The tile whose loads are being issued ("tile state", set by setup_tile below).  A tile
    // number of tiles_total stands for "no tile": its columns lie beyond the end, so that all
    // it gathers is zeros.
    int m0 = 0, n0 = 0, split = 0, t_begin = 0;

    const __amdgpu_buffer_rsrc_t xbuf = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p.x), 0, p.x_bytes, kBufferWord3);
    const __amdgpu_buffer_rsrc_t wbuf = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p.w), 0, p.w_bytes, kBufferWord3);
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
    uint32_t colbase_b = 0;  // byte offset of x[n, 0, p*u - pad_h, q*v - pad_w] (mod 2^32)
    // GATHER_MASKED: bit tr*S + ts set when tap (tr, ts) of this column's window, counted in reading direction, lies
    // outside the image; all ones for a column beyond NPQ; the bits from R*S on are always set (bit 63 serves
    // for "no such element")
    uint64_t inv_taps = ~0ull;
    uint64_t ms_row_bits = 0;   // bit r*S for every window row r
    if constexpr (GM == GATHER_MASKED)
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
        hw0[1] = (uint16_t)h0;
        hw0[0] = (uint16_t)w0;
        if (!cv) {
            hw0[1] = 0x8000;           // no tap of a column beyond NPQ is ever in range
        }
        if constexpr (MSK) {
            // window rows h0 .. h0+R-1: those with 0 <= h0 + t <= H-1 are valid (likewise columns)
            const int rlo = h0 < 0 ? -h0 : 0, rhi = p.H - 1 - h0 < p.R - 1 ? p.H - 1 - h0 : p.R - 1;
            const int clo = w0 < 0 ? -w0 : 0, chi = p.W - 1 - w0 < p.S - 1 ? p.W - 1 - w0 : p.S - 1;
            // valid columns as a bit field of S bits, repeated for every valid row: the product with the rows'
            // first bits (no two partial products overlap)
            auto bits64 = [](int lo, int hi) -> uint64_t {   // bits lo..hi, none when hi < lo (0 <= lo; hi <= 63)
                return hi >= lo ? ((~0ull >> (63 - (hi & 63))) & ~((1ull << (lo & 63)) - 1ull)) : 0ull;
            };
            const uint64_t cols = bits64(clo, chi);
            const uint64_t rows = rhi >= rlo ? (ms_row_bits & bits64(rlo * p.S, rhi * p.S)) : 0ull;
            inv_taps = cv ? ~(cols * rows) : ~0ull;
        }
    };
    u16x2 hw_max;
    hw_max[1] = (uint16_t)(p.H - 1);
    hw_max[0] = (uint16_t)(p.W - 1);
    // Byte offset of tap (tr, ts) of this column in channel 0, or the out-of-range marker
    // when the tap falls in the zero border (or the column is beyond NPQ).
    auto tap_offset = [&](uint32_t tr, uint32_t ts) -> uint32_t {
        const u16x2 tap = __builtin_bit_cast(u16x2, (tr << 16) | ts);
        const u16x2 hw = hw0 + tap;
        const u16x2 cl = __builtin_elementwise_min(hw, hw_max);
        const bool ok = __builtin_bit_cast(uint32_t, cl) == __builtin_bit_cast(uint32_t, hw);
        return ok ? colbase_b + (tr * (uint32_t)p.xsH + ts * (uint32_t)p.xsW) * ES : kOutOfRange;
    };
    // GATHER_NOPAD: the window origin of a valid column, else the out-of-range marker.
    uint32_t vcol = kOutOfRange;
    // GATHER_TAPS9: the nine tap offsets of this column (tap t = r*3+s... in general
    // r*S+s with R*S = 9), eq. 2's inversion applied.
    uint32_t vtaps[GM == GATHER_TAPS9 ? 9 : 1];
    auto setup_taps = [&]() {
        vcol = hw0[1] == 0x8000 ? kOutOfRange : colbase_b;
        if constexpr (GM == GATHER_TAPS9) {
#pragma unroll
            for (int t = 0; t < 9; ++t) {
                const uint32_t r = magic_div((uint32_t)t, p.mS);
                const uint32_t sx = (uint32_t)t - r * (uint32_t)p.S;
                vtaps[t] = tap_offset(p.flip ? (uint32_t)p.R - 1u - r : r, p.flip ? (uint32_t)p.S - 1u - sx : sx);
            }
        }
    };

    // ---- filter-tile role ----------------------------------------------------------
    // 16-byte path: the tile is BM rows of BK/VEC vectors, dealt to the threads in order;
    // the last pass may be partial.  Scalar path: BM*BK elements, BK a power of two.
    constexpr int A_VPR = BK / VEC;  // vectors per row
    constexpr int A_TOTAL = Cfg::VECA ? BM * A_VPR : BM * BK;
    constexpr int A_PASSES = (A_TOTAL + 255) / 256;
    constexpr bool A_PARTIAL = A_TOTAL % 256 != 0;
    int a_row[A_PASSES], a_kk[A_PASSES];
#pragma unroll
    for (int ps = 0; ps < A_PASSES; ++ps) {
        const int idx = tid + ps * 256;
        a_row[ps] = Cfg::VECA ? idx / A_VPR : idx / BK;
        a_kk[ps] = Cfg::VECA ? (idx % A_VPR) * VEC : idx % BK;
    }

    // Registers holding the tiles in flight between HBM and LDS: two sets, tile T uses
    // set T&1, so that the loads of tile t+2 can be issued while tile t+1 still waits
    // in the other set to be written to LDS.
    u32x4 a_vec[2][Cfg::VECA ? A_PASSES : 1];
    elem_t a_sca[2][Cfg::VECA ? 1 : A_PASSES];
    elem_t b_val[2][KPT];
    // Per-lane decode, lane L standing for element L of this wavefront's run of the
    // step.  GATHER_GENERIC: byte offset of the tap relative to the window origin
    // (dec_so) and the packed tap (dec_tap).  GATHER_NOPAD / GATHER_TAPMAJOR: the
    // element's scalar offset, or the buffer size if the element does not exist (the
    // hardware compares the vector offset with "size - scalar offset": a scalar offset
    // equal to the size puts every lane out of range, a larger one would wrap).
    uint32_t dec_il = 0, dec_c = 0, dec_rs = 0, dec_so = 0, dec_tap = 0;
    // GATHER_TAPMAJOR: the step's tap; this column's offset for it; the filter's scalar
    // offset.  GATHER_TAPS9: the scalar offsets of the channels this thread gathers.
    uint32_t sc_tr = 0, sc_ts = 0, sc_c0 = 0, sc_asoff = 0;
    int sc_tau = 0;
    uint32_t vtap = kOutOfRange;
    uint32_t sc_cso[GM == GATHER_TAPS9 ? KPT / 9 : 1];
    // GATHER_MASKED: the next element of this wavefront's run - columns left in its window row and rows left in its
    // channel (the walk follows the filter's own order r, s), byte offset from the window origin, bit number,
    // reduction indices left after it - and the constants of the three ways to step to the one after: next
    // column of the window; first column of the next row; first tap of the next channel.  (dir: +1, or -1 when
    // eq. 2 inverts the filter: the window is then walked backwards.)
    uint32_t ms_cs = 0, ms_cr = 0, ms_d = 0, ms_bit = 0, ms_left = 0;
    const uint32_t ms_dir = p.flip ? 0xFFFFFFFFu : 1u;
    const uint32_t ms_sm1 = (uint32_t)p.S - 1u, ms_rm1 = (uint32_t)p.R - 1u;
    const uint32_t ms_dd0 = ms_dir * (uint32_t)p.xsW * ES;
    const uint32_t ms_dd1 = ms_dir * ((uint32_t)p.xsH - ms_sm1 * (uint32_t)p.xsW) * ES;
    const uint32_t ms_dd2 = ((uint32_t)p.xsC - ms_dir * (ms_sm1 * (uint32_t)p.xsW + ms_rm1 * (uint32_t)p.xsH)) * ES;
    const uint32_t ms_db2 = 0u - ms_dir * ((uint32_t)p.RS - 1u);
    uint32_t a_jo = 0;  // GATHER_MASKED through strides: offset of this thread's reduction index in the filter

    // F_m tile: rows m0.., the step's reduction indices; zero beyond K and beyond the
    // reduction range.  The per-thread part of the offset is fixed, the step's part is a
    // scalar.  Filter order: index k0 + a_kk of row `row`.  Tap-major: channel
    // c0 + a_kk, tap of the step, i.e. a strided read (stride R*S elements in the
    // forward pass); row, channel and tap strides come from the launch parameters.
    uint32_t a_voff[A_PASSES];
    auto setup_rows = [&]() {
#pragma unroll
      for (int ps = 0; ps < A_PASSES; ++ps) {
        const int row = m0 + a_row[ps];
        const bool ok = row < p.K && a_row[ps] < BM;
        if constexpr (GM == GATHER_TAPS9 && !Cfg::VECA) {
            // element-wise filter reads through the row / channel / tap strides (backward data,
            // or a filter that is not 16-byte aligned): channel a_kk/9 of the step, tap a_kk%9
            const uint32_t ch = (uint32_t)a_kk[ps] / 9u, t = (uint32_t)a_kk[ps] % 9u;
            const uint32_t r = magic_div(t, p.mS);
            const uint32_t sx = t - r * (uint32_t)p.S;
            const uint32_t off = (uint32_t)row * (uint32_t)p.wsRow + ch * (uint32_t)p.wsRed + (uint32_t)p.wTap0 +
                                 r * (uint32_t)p.wsTapR + sx * (uint32_t)p.wsTapS;
            a_voff[ps] = ok ? off * ES : kOutOfRange;
        } else if constexpr (MSK_STRIDED)
            // (rows beyond K are never stored: they may read row 0; the reduction index's part of
            // the offset, which also carries the out-of-range marker, is added per step)
            a_voff[ps] = (uint32_t)(row < p.K ? row : 0) * (uint32_t)p.wsRow * ES;
        else if constexpr (GM == GATHER_TAPMAJOR)
            a_voff[ps] = ok ? ((uint32_t)row * (uint32_t)p.wsRow + (uint32_t)a_kk[ps] * (uint32_t)p.wsRed) * ES : kOutOfRange;
        else
            a_voff[ps] = ok ? ((uint32_t)row * (uint32_t)p.CRS + (uint32_t)a_kk[ps]) * ES : kOutOfRange;
      }
    };
    // Everything the loads of a tile depend on.
    auto setup_tile = [&](int tile) {
        if (p.splits > 1) {
            split = tile / tiles_mn;
            tile -= split * tiles_mn;
            t_begin = split * p.stepsPerSplit;
        }
        if constexpr (Cfg::TEAMS > 1) t_begin = team * p.stepsPerSplit;   // (the host: one range, stepsPerSplit steps per team)
        m0 = (tile % p.tilesM) * BM;
        n0 = (tile / p.tilesM) * BN;
        setup_column();
        setup_taps();
        setup_rows();
    };

    // Start of the load of tile number tau (reduction step tau), in two halves so that
    // each fits between two MFMAs.
    auto decode1 = [&](int tau) {
        if constexpr (MSK) {
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
        } else if constexpr (GM == GATHER_NOPAD_TABLE) {
            sc_tau = __builtin_amdgcn_readfirstlane(tau);
            dec_so = so_table[sc_tau * BK + kpart * KPT + (lane < KPT ? lane : KPT - 1)];
        } else if constexpr (GEN || GM == GATHER_NOPAD) {
            // i -> (c, r*S+s) for i = first index of the run + lane
            sc_tau = __builtin_amdgcn_readfirstlane(tau);
            dec_il = (uint32_t)(tau * BK + kpart * KPT) + (uint32_t)lane;
            dec_c = magic_div(dec_il, p.mRS);
            dec_rs = dec_il - dec_c * (uint32_t)p.RS;
        } else if constexpr (GM == GATHER_TAPMAJOR) {
            // (readfirstlane states the wavefront-uniformity for the compiler)
            const uint32_t ut = __builtin_amdgcn_readfirstlane((uint32_t)tau);
            sc_tau = (int)ut;
            const uint32_t cc = magic_div(ut, p.mRS);       // channel chunk
            const uint32_t tap = ut - cc * (uint32_t)p.RS;  // r*S+s
            const uint32_t r = magic_div(tap, p.mS);
            const uint32_t sx = tap - r * (uint32_t)p.S;
            sc_tr = p.flip ? (uint32_t)p.R - 1u - r : r;    // eq. 2 inverts the filter
            sc_ts = p.flip ? (uint32_t)p.S - 1u - sx : sx;
            sc_c0 = cc * BK;
            const uint32_t live = mask_lt(ut, (uint32_t)p.ksteps);
            // (wrap-around arithmetic: a tap stride may be negative, the sum never is)
            const uint32_t woff = sc_c0 * (uint32_t)p.wsRed + (uint32_t)p.wTap0 + r * (uint32_t)p.wsTapR + sx * (uint32_t)p.wsTapS;
            sc_asoff = ((woff * ES) & live) | (p.w_bytes & ~live);
            const uint32_t c = sc_c0 + (uint32_t)(kpart * KPT) + (uint32_t)lane;
            dec_so = (c < (uint32_t)p.C && live) ? c * (uint32_t)p.xsC * ES : p.x_bytes;
        } else {
            const uint32_t ut = __builtin_amdgcn_readfirstlane((uint32_t)tau);
            const uint32_t live = mask_lt(ut, (uint32_t)p.ksteps);
            const uint32_t astep = Cfg::VECA ? (uint32_t)BK : (uint32_t)(BK / 9) * (uint32_t)p.wsRed;  // elements per step in a filter row
            sc_asoff = ((ut * astep * ES) & live) | (p.w_bytes & ~live);
            const uint32_t c = ut * (BK / 9) + (uint32_t)(kpart * (KPT / 9));
#pragma unroll
            for (int q = 0; q < KPT / 9; ++q)
                sc_cso[q] = (((c + q) * (uint32_t)p.xsC * ES) & live) | (p.x_bytes & ~live);
        }
    };
    auto decode2 = [&]() {
        if constexpr (MSK) {
            if constexpr (MSK_STRIDED) {
                // first operand: this thread's reduction index (the same in all its passes) through the
                // reduction and tap strides
                const uint32_t ja = (uint32_t)(sc_tau * BK + a_kk[0]);
                const uint32_t kc = magic_div(ja, p.mRS);
                const uint32_t rem = ja - kc * (uint32_t)p.RS;
                const uint32_t r = magic_div(rem, p.mS);
                const uint32_t sx = rem - r * (uint32_t)p.S;
                a_jo = ja < (uint32_t)p.CRS && sc_tau < p.ksteps
                           ? (kc * (uint32_t)p.wsRed + (uint32_t)p.wTap0 + r * (uint32_t)p.wsTapR + sx * (uint32_t)p.wsTapS) * ES
                           : kOutOfRange;
            } else if (sc_tau == p.tail_step) {   // (ragged last step: see below)
#pragma unroll
                for (int ps = 0; ps < A_PASSES; ++ps)
                    a_voff[ps] = (uint32_t)(sc_tau * BK + a_kk[ps]) < (uint32_t)p.CRS ? a_voff[ps] : kOutOfRange;
            }
        } else if constexpr (GM == GATHER_NOPAD_TABLE) {
            if (sc_tau == p.tail_step) {   // (see below)
#pragma unroll
                for (int ps = 0; ps < A_PASSES; ++ps)
                    a_voff[ps] = (uint32_t)(sc_tau * BK + a_kk[ps]) < (uint32_t)p.CRS ? a_voff[ps] : kOutOfRange;
            }
        } else if constexpr (GEN || GM == GATHER_NOPAD) {
            const uint32_t r = magic_div(dec_rs, p.mS);
            const uint32_t sx = dec_rs - r * (uint32_t)p.S;
            // window coordinates of the element: the tap, inverted for eq. 2
            const uint32_t tr = p.flip ? (uint32_t)p.R - 1u - r : r;
            const uint32_t ts = p.flip ? (uint32_t)p.S - 1u - sx : sx;
            const uint32_t so = (dec_c * (uint32_t)p.xsC + tr * (uint32_t)p.xsH + ts * (uint32_t)p.xsW) * ES;
            const bool live = dec_il < (uint32_t)p.CRS;
            if constexpr (GEN) {
                dec_so = so;
                dec_tap = live ? ((tr << 16) | ts) : 0x80000000u;  // i >= CRS: never in range
            } else {
                dec_so = live ? so : p.x_bytes;
            }
            // When C*R*S is not a multiple of BK the last step is ragged: on entering it
            // (once per tile) the filter offsets of the indices beyond the range are
            // replaced by the out-of-range marker.
            if (sc_tau == p.tail_step) {
#pragma unroll
                for (int ps = 0; ps < A_PASSES; ++ps)
                    a_voff[ps] = (uint32_t)(sc_tau * BK + a_kk[ps]) < (uint32_t)p.CRS ? a_voff[ps] : kOutOfRange;
            }
        } else if constexpr (GM == GATHER_TAPMAJOR) {
            vtap = tap_offset(sc_tr, sc_ts);
            // When C is not a multiple of BK the last channel chunk is ragged: in its steps
            // (the chunks are the outer order, so they are the last R*S steps; a range of a cut
            // reduction may begin in the middle of them) the filter offsets of the channels
            // beyond C are replaced by the out-of-range marker.  (tail_step = -1: never.)
            if ((uint32_t)sc_tau >= (uint32_t)p.tail_step) {
#pragma unroll
                for (int ps = 0; ps < A_PASSES; ++ps)
                    a_voff[ps] = sc_c0 + (uint32_t)a_kk[ps] < (uint32_t)p.C ? a_voff[ps] : kOutOfRange;
            }
        }
    };
    auto load_a = [&](int set, int tau, int ps) {
        uint32_t voffa = a_voff[ps], soff;
        if constexpr (MSK_STRIDED) {
            voffa += a_jo;
            soff = 0;
        } else if constexpr (GM == GATHER_TAPMAJOR || GM == GATHER_TAPS9) {
            soff = sc_asoff;  // (TAPS9: C % 4 == 0, so a row never ends inside a step)
        } else {
            // (a reduction range that ends inside the last step: masked in place by decode2)
            const uint32_t k0 = (uint32_t)tau * BK;
            uint32_t live = mask_lt(k0, (uint32_t)p.CRS);
            if constexpr (MSK) live &= mask_lt((uint32_t)tau, (uint32_t)p.ksteps);
            soff = ((k0 * ES) & live) | (p.w_bytes & ~live);
        }
        if constexpr (Cfg::VECA) {
            a_vec[set][ps] = __builtin_amdgcn_raw_buffer_load_b128(wbuf, voffa, soff, 0);
        } else if constexpr (Cfg::BF16) {
            a_sca[set][ps] = __builtin_amdgcn_raw_buffer_load_b16(wbuf, voffa, soff, 0);
        } else {
            a_sca[set][ps] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(wbuf, voffa, soff, 0));
        }
    };
    // D_m tile, element e of this lane's column.
    auto load_b = [&](int set, int e) __attribute__((always_inline)) {
        uint32_t vo, so;
        if constexpr (MSK) {
            // bit 0 of the shifted mask: 1 when the tap lies outside the image (bit 63: the index is past the end);
            // shifted to bit 31 it puts the offset out of range (a valid offset lies below 2^31)
            const uint32_t bit = (int32_t)ms_left < 0 ? 63u : ms_bit;
            const uint32_t out = (uint32_t)(inv_taps >> bit);
            vo = (out << 31) | (colbase_b + ms_d);
            so = 0;
        } else if constexpr (GEN) {
            // lane e's decode as scalars, then the window test
            const uint32_t d = __builtin_amdgcn_readlane(dec_so, e);
            const u16x2 tap = __builtin_bit_cast(u16x2, (uint32_t)__builtin_amdgcn_readlane(dec_tap, e));
            const u16x2 hw = hw0 + tap;
            const u16x2 cl = __builtin_elementwise_min(hw, hw_max);
            const bool ok = __builtin_bit_cast(uint32_t, cl) == __builtin_bit_cast(uint32_t, hw);
            vo = ok ? colbase_b + d : kOutOfRange;
            so = 0;
        } else if constexpr (GM == GATHER_TAPMAJOR) {
            vo = vtap;
            so = __builtin_amdgcn_readlane(dec_so, e);
        } else if constexpr (NOPADX) {
            vo = vcol;
            so = __builtin_amdgcn_readlane(dec_so, e);
        } else {
            vo = vtaps[e % 9];
            so = sc_cso[e / 9];
        }
        if constexpr (Cfg::BF16) {
            b_val[set][e] = __builtin_amdgcn_raw_buffer_load_b16(xbuf, vo, so, 0);
        } else {
            b_val[set][e] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(xbuf, vo, so, 0));
        }
    };
    // GATHER_MASKED: step the scalar state to the next element of the run (conditions as selects: no branch)
    // GATHER_MASKED: step the scalar state to the next element of the run.  Ten scalar instructions chained
    // through the carry flag (a column count that runs out borrows: the row count is decreased by that borrow,
    // and borrows itself at the end of a channel); written out because the compiler's version of the same
    // selects is three times as long, and what sits between two MFMAs has to fit in the time one takes.
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
        elem_t *const A = ldsA + buf * Cfg::A_ELEMS + a_row[ps] * LD + a_kk[ps];
        if (A_PARTIAL && ps == A_PASSES - 1 && a_row[ps] >= BM) return;  // threads beyond the tile
        if constexpr (Cfg::VECA) {
            *reinterpret_cast<u32x4 *>(A) = a_vec[set][ps];
        } else {
            *A = a_sca[set][ps];
        }
    };
    // Chunk q of this lane's run of the D_m tile: 16 bytes, or 8 where the run does not
    // start on a 16-byte boundary.
    constexpr bool B_W16 = (KPT * ES) % 16 == 0;
    constexpr int B_WE = B_W16 ? VEC : VEC / 2;  // elements per write
    auto write_b = [&](int set, int buf, int q) {
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

    // Moving one tile is a list of small items: NL load items (decode halves, filter
    // loads, gathered elements) and NW LDS-write items.
    constexpr int NB_ELEMS = KPT;   // gathered elements per thread and step
    constexpr int NW_A = A_PASSES, NW_B = KPT / B_WE, NW = NW_A + NW_B;
    // (GATHER_MASKED: an element is two items, its load and the step to the next one, so that neither is too long
    // for the gap between two MFMAs)
    constexpr int NL = 2 + A_PASSES + (MSK ? 2 : 1) * NB_ELEMS;
    auto load_item = [&](int i, int set, int tau) __attribute__((always_inline)) {
        if (i == 0) decode1(tau);
        else if (i == 1) decode2();
        else if (i < 2 + A_PASSES) load_a(set, tau, i - 2);
        else if constexpr (MSK) {
            if ((i - 2 - A_PASSES) % 2 == 0) load_b(set, (i - 2 - A_PASSES) / 2);
            else advance_tap();
        } else load_b(set, i - 2 - A_PASSES);
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
    // `groups`: the k-groups this step multiplies - all G of them, or (SHORT_LAST, last step of a
    // tile) only the first G/2, the rest of the step being zeros; both even, so that the fragment
    // sets keep alternating in step; or (ODD_LAST, last step of a tile) none.
    // (always_inline: the accumulators must stay in registers; left to its own judgement the inliner gives up on
    // bodies of this size and the captured arrays move to scratch memory)
    auto step_groups = [&](auto parity, auto groups, int k2) __attribute__((always_inline)) {   // k2: the step whose tiles are requested during this one
        constexpr int cur = decltype(parity)::value, nxt = cur ^ 1;
        constexpr int GS = decltype(groups)::value;
        constexpr int NMS = GS == G ? NM : GS * MPG_FULL;      // MFMAs of this step
        constexpr int SBS = GS == G ? SB : NMS - MPG_FULL;     // first MFMA of its last group
        constexpr int fs0 = (G & 1) ? cur : 0;  // fragment set of this step's group 0
        if constexpr (GS == 0) {
            // nothing to multiply: the step's side work only, then the first fragments of the next
            // step into the set that step starts with
            static_for<NL>([&](auto ic) { load_item(decltype(ic)::value, cur, k2); });
            static_for<NW>([&](auto ic) { write_item(decltype(ic)::value, nxt, nxt); });
            lds_barrier();
            read_frags(nxt, 0, (G & 1) ? nxt : 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        static_for<NMS>([&](auto mc) {
            constexpr int m = decltype(mc)::value;
            constexpr int g = m / MPG_FULL < GS - 1 ? m / MPG_FULL : GS - 1;
            constexpr int j = m - g * MPG_FULL;
            constexpr int fs = (fs0 + g) & 1;
            if constexpr (j == 0 && g + 1 < GS) read_frags(cur, g + 1, fs ^ 1);
            if constexpr (m == SBS) {
                lds_barrier();
                read_frags(nxt, 0, fs ^ 1);
            }
            // load items i with floor(i * NMS / NL) == m: tile t+2 -> set cur
            constexpr int l0 = (m * NL + NMS - 1) / NMS, l1 = ((m + 1) * NL + NMS - 1) / NMS;
            static_for<l1 - l0>([&](auto ic) { load_item(l0 + decltype(ic)::value, cur, k2); });
            // write items, packed into the slots before the barrier: tile t+1, set nxt -> stage nxt
            constexpr int WS = NW < SBS ? NW : SBS;   // slots used for writes
            if constexpr (m >= SBS - WS && m < SBS) {
                constexpr int q = m - (SBS - WS);
                constexpr int w0 = (q * NW + WS - 1) / WS, w1 = ((q + 1) * NW + WS - 1) / WS;
                static_for<w1 - w0>([&](auto ic) { write_item(w0 + decltype(ic)::value, nxt, nxt); });
            }
            mfma(fs, j);
            __builtin_amdgcn_sched_barrier(0);
        });
    };
    auto step = [&](auto parity, int k2) __attribute__((always_inline)) { step_groups(parity, std::integral_constant<int, G>{}, k2); };
    static_assert(!SHORT_LAST || (REM == 0 && G % 4 == 0), "half a step must be a whole, even number of full k-groups");

    // A tile takes `nsteps` steps, a whole number of pairs (an odd count runs one extra step
    // on zero tiles), so that the loop body stays a single basic block.  When the reduction is
    // cut into ranges (backward filter; forward on small problems with a workspace), a tile is
    // one range; a range that reaches past the last step reads zeros there.
    const int nsteps = p.stepsPerSplit;   // (even; the host rounds an odd number of steps up)
    if constexpr (GM == GATHER_NOPAD_TABLE) {
        // offset of reduction index i = (c,r,s) relative to the window origin, or the buffer size
        // for an index past the end (the host checked that (nsteps + 2) * BK entries fit)
        for (uint32_t i = (uint32_t)tid; i < (uint32_t)(nsteps + 2) * BK; i += 256u) {
            const uint32_t c = magic_div(i, p.mRS);
            const uint32_t rs = i - c * (uint32_t)p.RS;
            const uint32_t r = magic_div(rs, p.mS);
            const uint32_t sx = rs - r * (uint32_t)p.S;
            const uint32_t tr = p.flip ? (uint32_t)p.R - 1u - r : r;
            const uint32_t ts = p.flip ? (uint32_t)p.S - 1u - sx : sx;
            const uint32_t so = (c * (uint32_t)p.xsC + tr * (uint32_t)p.xsH + ts * (uint32_t)p.xsW) * ES;
            so_table[i] = i < (uint32_t)p.CRS ? so : p.x_bytes;
        }
        lds_barrier();
    }
    setup_tile(tile_number(0));
    float bias_cur[MB], bias_next[MB];
    load_bias<MB>(p, m0 + wm * Cfg::TM, l32, bias_cur);
    // Prologue: request the first two tiles back to back, then write the first to LDS stage
    // 0 as it arrives (the second stays in flight, it is written during the first step).
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
        // The last two steps of this tile request the first two steps of the workgroup's next
        // tile (of "no tile" after the last one): its operands arrive and its first fragments
        // are read while this tile is still being multiplied and stored.
        const int out_m0 = m0, out_n0 = n0, out_split = split;
        const int next = tile_number(it);
        setup_tile(next);
        load_bias<MB>(p, m0 + wm * Cfg::TM, l32, bias_next);
        step(std::integral_constant<int, 0>{}, t_begin);
        step_groups(std::integral_constant<int, 1>{}, std::integral_constant<int, SHORT_LAST ? G / 2 : (ODD_LAST ? 0 : G)>{}, t_begin + 1);
        // (each range of a cut reduction writes its own copy of the output, y_bytes long)
        const uint32_t ybase = (uint32_t)out_split * p.ySplitBytes;
        const __amdgpu_buffer_rsrc_t ybuf = __builtin_amdgcn_make_buffer_rsrc(
            static_cast<char *>(p.y) + ybase, 0, p.y_bytes, kBufferWord3);
        if constexpr (Cfg::TEAMS > 1) {
            // The host gives a workgroup of teams one tile, so nothing in LDS is needed any more: the
            // teams after the first leave their sums at the start of their LDS (16 bytes per lane and
            // piece: lane-contiguous), the first adds them in team order.
            __syncthreads();
            constexpr int TEAM_F4 = Cfg::TEAM_LDS_BYTES / 16;
            f32x4 *const xch = reinterpret_cast<f32x4 *>(lds) + (wave * MB * NB * 4) * 64 + lane;
            if (team > 0) {
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                        for (int c = 0; c < 4; ++c)
                            xch[team * TEAM_F4 + ((mb * NB + nb) * 4 + c) * 64] =
                                f32x4{acc[mb][nb][4 * c], acc[mb][nb][4 * c + 1], acc[mb][nb][4 * c + 2], acc[mb][nb][4 * c + 3]};
            }
            __syncthreads();
            if (team > 0) return;
            for (int tm = 1; tm < Cfg::TEAMS; ++tm)
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                        for (int c = 0; c < 4; ++c) {
                            const f32x4 o = xch[tm * TEAM_F4 + ((mb * NB + nb) * 4 + c) * 64];
#pragma unroll
                            for (int e = 0; e < 4; ++e) acc[mb][nb][4 * c + e] += o[e];
                        }
        }
        store_tile<Cfg::SWAP, MB, NB>(p, ybuf, acc, bias_cur, out_m0 + wm * Cfg::TM, out_n0 + wn * Cfg::TN, half, l32);
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
