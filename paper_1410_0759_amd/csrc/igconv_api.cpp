// Host part of the library: descriptors, validation, launch plan, C ABI.
// All validation runs before the first GPU call, so every error path works on a
// machine without a GPU.  See include/igconv.h for the contract of each entry point.
#include "../../include/igconv.h"

#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <algorithm>
#include <vector>
#include <new>

#include "igconv_kernel_table.h"
#include "igconv_params.h"

#include "igconv_desc.h"

namespace igc {

// The tile heuristic balances workgroups over the device's compute units, whose number the handle reads from the
// runtime when it is created (MI355X: 256; that figure also stands in on a machine without a GPU, where plans can
// still be queried).  The kernels deal workgroups to XCDs by blockIdx % 8: gfx950 parts have 8.
constexpr int kXcds = 8;
// gather mode 15: what loading an element costs, in multiply-add rows (see plan_cost)
constexpr double kDirectGatherCost = 20.0, kDirectGatherCostStaged = 9.0;
constexpr int kOffsetTableEntries = 2048;  // LDS offset table of the short-reduction unpadded kernels
constexpr long long kMaxBytes = 1ll << 31;  // byte offsets must stay below this

static const KernelGroup *const kGroups[] = {&kGroupF32Taps9, &kGroupF32TapMajor, &kGroupF32Nopad, &kGroupF32Generic, &kGroupF32Swap,
                                            &kGroupBF16, &kGroupBF16Channels, &kGroupWgrad, &kGroupF64, &kGroupWgradBF16Channels, &kGroupBF16Pointwise, &kGroupF32Teams,
                                            &kGroupF32Masked, &kGroupF64Masked, &kGroupF32Direct};

int kernel_count() {
    int n = 0;
    for (const KernelGroup *g : kGroups) n += g->count;
    return n;
}

const KernelInfo *kernel_info(int id) {
    if (id < 0) return nullptr;
    for (const KernelGroup *g : kGroups) {
        if (id < g->count) return &g->kernels[id];
        id -= g->count;
    }
    return nullptr;
}

// eq. 1: ceil((H - R + 1 + 2 pad) / u); <= 0 when there is no output.
static long long out_dim(long long H, long long R, long long u, long long pad) {
    const long long num = H - R + 1 + 2 * pad;
    if (num <= 0) return 0;
    return (num + u - 1) / u;
}

struct Problem {
    ConvKernelParams kp;
    bool bf16;
    bool f64 = false;  // double precision in and out
    int vec;  // elements per 16 bytes of input
    unsigned mode_mask = 0;   // non-zero: bit g set when gather mode g can run this problem
    bool zero_steps = false;  // nothing to accumulate: the kernel only scales the old output
    bool no_teams = false;    // leave the kernels that cut the reduction inside a workgroup (teams, gather mode 15) out of the
                              // choice: a workspace cuts it across compute units, which measured faster where both apply
};

// Everything igcConvolutionForward checks that does not need the data pointers.
static igcStatus validate(igcTensorDescriptor_t x, igcFilterDescriptor_t w,
                          igcConvolutionDescriptor_t cv, igcTensorDescriptor_t y, Problem *out) {
    if (!x || !w || !cv || !y) return IGC_STATUS_BAD_PARAM;
    if (!x->set || !w->set || !cv->set || !y->set) return IGC_STATUS_NOT_INITIALIZED;
    if (x->dim[1] != w->c) return IGC_STATUS_BAD_PARAM;
    const long long P = out_dim(x->dim[2], w->r, cv->u, cv->pad_h);
    const long long Q = out_dim(x->dim[3], w->s, cv->v, cv->pad_w);
    if (P < 1 || Q < 1) return IGC_STATUS_BAD_PARAM;
    if (y->dim[0] != x->dim[0] || y->dim[1] != w->k || y->dim[2] != P || y->dim[3] != Q)
        return IGC_STATUS_BAD_PARAM;
    if (!non_aliasing(y->dim, y->stride)) return IGC_STATUS_BAD_PARAM;

    const bool f32 = x->dtype == IGC_DATA_FLOAT && w->dtype == IGC_DATA_FLOAT;
    const bool b16 = x->dtype == IGC_DATA_BFLOAT16 && w->dtype == IGC_DATA_BFLOAT16;
    const bool f64 = x->dtype == IGC_DATA_DOUBLE && w->dtype == IGC_DATA_DOUBLE;
    if (!(f32 || b16 || f64) || y->dtype != (f64 ? IGC_DATA_DOUBLE : IGC_DATA_FLOAT)) return IGC_STATUS_NOT_SUPPORTED;

    const int es = elem_size(x->dtype);
    const long long xb = extent(x->dim, x->stride) * es;
    const long long yb = extent(y->dim, y->stride) * elem_size(y->dtype);
    const long long CRS = (long long)w->c * w->r * w->s;
    const long long wb = (long long)w->k * CRS * es;
    const long long NPQ = (long long)x->dim[0] * P * Q;
    if (xb >= kMaxBytes || yb >= kMaxBytes || wb >= kMaxBytes) return IGC_STATUS_NOT_SUPPORTED;
    // Index ranges the kernels decode with 32-bit magic division, and the reach of
    // the padded window in x measured in bytes (offsets of border taps are formed
    // before they are discarded).
    if (NPQ >= (1ll << 30) || CRS >= (1ll << 30)) return IGC_STATUS_NOT_SUPPORTED;
    // The kernels test "tap inside the image" on packed 16-bit coordinates.
    if (x->dim[2] > (1 << 14) || x->dim[3] > (1 << 14) || cv->pad_h >= (1 << 14) || cv->pad_w >= (1 << 14))
        return IGC_STATUS_NOT_SUPPORTED;

    if (out) {
        ConvKernelParams &k = out->kp;
        k = ConvKernelParams{};
        k.x_bytes = (uint32_t)xb;
        k.w_bytes = (uint32_t)wb;
        k.y_bytes = (uint32_t)yb;
        k.N = x->dim[0]; k.C = x->dim[1]; k.H = x->dim[2]; k.W = x->dim[3];
        k.K = w->k; k.R = w->r; k.S = w->s; k.P = (int)P; k.Q = (int)Q;
        k.pad_h = cv->pad_h; k.pad_w = cv->pad_w; k.u = cv->u; k.v = cv->v;
        k.flip = cv->mode == IGC_CONVOLUTION ? 1 : 0;
        k.CRS = (int)CRS; k.NPQ = (int)NPQ; k.PQ = (int)(P * Q); k.RS = w->r * w->s;
        k.Wp = k.W + 2 * k.pad_w;
        // (only the patch-staging kernels use HpWp; they are not offered when it is clamped here)
        k.HpWp = (int)std::min<long long>((long long)(k.H + 2 * k.pad_h) * k.Wp, 0x7fffffff);
        if (!magic_for((uint32_t)k.Wp, &k.mWp) || !magic_for((uint32_t)k.HpWp, &k.mHpWp)) return IGC_STATUS_NOT_SUPPORTED;
        if (!magic_for((uint32_t)k.PQ, &k.mPQ) || !magic_for((uint32_t)k.Q, &k.mQ) ||
            !magic_for((uint32_t)k.RS, &k.mRS) || !magic_for((uint32_t)k.S, &k.mS))
            return IGC_STATUS_NOT_SUPPORTED;
        k.wsRow = k.CRS; k.wsRed = k.RS; k.wTap0 = 0; k.wsTapR = k.S; k.wsTapS = 1;
        k.xsN = (int)x->stride[0]; k.xsC = (int)x->stride[1]; k.xsH = (int)x->stride[2]; k.xsW = (int)x->stride[3];
        k.ysN = (int)y->stride[0]; k.ysK = (int)y->stride[1]; k.ysP = (int)y->stride[2]; k.ysQ = (int)y->stride[3];
        out->bf16 = b16;
        out->f64 = f64;
        out->vec = 16 / es;
    }
    return IGC_STATUS_SUCCESS;
}

// Reduction steps a kernel needs: its order is either the filter's (c,r,s), cut into
// chunks of BK, or tap-major: per tap, the channels in chunks of BK.
static long long kernel_steps(const KernelInfo &ki, const ConvKernelParams &k) {
    if (ki.gmode == 1) return (long long)k.RS * ((k.C + ki.BK - 1) / ki.BK);
    if (ki.gmode == 3 || ki.gmode == 4 || ki.gmode == 5) return k.C / (ki.BK / 9);
    if (ki.gmode == 12) return (k.C + ki.BK - 1) / ki.BK;
    return (k.CRS + ki.BK - 1) / ki.BK;
}

static bool is_direct(int gmode) { return gmode == 15 || gmode == 16; }

// Gather modes 15 and 16 (igconv_kernel_f32d.hpp): steps of BK reduction indices per wavefront, the workgroup's wavefronts
// sharing the reduction evenly; a multiple of the request depth.
static long long direct_steps_per_wave(const KernelInfo &ki, const ConvKernelParams &k) {
    const long long waves = ki.threads / 64, steps = (k.CRS + ki.BK - 1) / ki.BK;
    const long long per = (steps + waves - 1) / waves;
    // (a multiple of the request depth; with the filter rows staged in LDS, of the eight steps of two row copies)
    const long long unit = ki.variant == 1 ? 8 : direct_depth(ki.BK);
    return (per + unit - 1) / unit * unit;
}

// Relative cost of running the problem with one kernel variant.  Tiles are padded to
// full size; a compute unit holds up to `occ` workgroups at a time (LDS), which share its
// MFMA pipes, so a full wave of 256*occ workgroups takes occ tile-times, and a last,
// partial wave as many tile-times as its fullest compute unit holds workgroups.
// Workgroups of a kernel a compute unit holds at a time: by LDS (160 KB), and by registers (as compiled:
// at most 512 / (VGPRs + AGPRs) waves per SIMD) two of the kernels with steps of 32 or more - four of the
// 64 x 64 x 32 ones (unpadded forward, backward filter by tap: 112 registers) -, three or (tiles up to 64 x 128) four of those with steps
// of 16.  More workgroups per compute unit cover more of each other's waits: Table-2 layer 3 gained 4 %.
static int workgroups_per_cu(const KernelInfo &ki) {
    const bool small_tile = (ki.gmode == 2 || (ki.gmode == 8 && !ki.bf16)) && ki.BM * ki.BN <= 64 * 64 && ki.BK == 32;
    if (is_direct(ki.gmode)) return ki.variant == 1 ? 1 : (160 * 1024) / ki.ldsBytes;   // (64 or 80 KB of LDS each, 64 more with the filter rows staged)
    // (double precision, pipelined: 105 registers for the 64 x 64 tile, 169 for 128 x 64)
    if (ki.f64) return ki.gmode == 14 ? (ki.BM * ki.BN <= 64 * 64 ? 4 : 2) : 4;
    const int by_regs = ki.BK == 16 ? (ki.BM * ki.BN <= 64 * 128 ? 4 : 3) : (small_tile ? 4 : 2);
    return std::max(1, std::min(by_regs, (160 * 1024) / ki.ldsBytes));
}

static double plan_cost(const igcContext *h, const KernelInfo &ki, const ConvKernelParams &k) {
    const long long cus = h->computeUnits;
    const long long tm = (k.K + ki.BM - 1) / ki.BM;
    const long long tn = (k.NPQ + ki.BN - 1) / ki.BN;
    const long long steps = kernel_steps(ki, k);
    const long long tiles = tm * tn;
    const long long occ = workgroups_per_cu(ki);
    const long long wave = cus * occ;
    const long long rem = tiles % wave;
    const double tile_times = (double)(tiles / wave) * occ + (double)((rem + cus - 1) / cus);
    // Per step a workgroup does BM*BN*BK multiply-adds and gathers BN*BK elements of
    // D_m; measured on the box, gathering one element costs about as much MFMA time as
    // `gather` multiply-add rows, depending on the mode.
    // The channel-vector bf16 kernels are bound by their loads, not by the MFMA pipe: measured,
    // a step costs about 2.75 units per filter row and 1 (1.5 when gathered tap by tap) per column,
    // plus a small MFMA term; the scale makes them comparable with the line below.
    // (1x1 filters over channel vectors: loads of both operands and a small MFMA term per step of 64 channels)
    if (ki.gmode == 12) return tile_times * steps * 1000.0 * (1.0 * ki.BM + 1.0 * ki.BN + ki.BM * ki.BN / 64.0);
    if (ki.gmode == 5 && ki.variant == 3) {
        // Moving and multiplying wavefronts apart (igconv_kernel_bf16s.hpp), one workgroup per compute unit.  Two
        // groups of multipliers (steps of 32 channels): for problems that leave compute units without a second
        // workgroup anyway, measured 0.82 of the two-team kernel's time on such a problem.  One group on a
        // 128 x 256 tile: measured 0.94 of the time of the 64 x 256 kernel at two workgroups per compute unit.
        const bool two_groups = ki.BK == 288;
        if (two_groups && tiles > cus) return 1e300;
        const double unit = 2.75 * ki.BM + 1.0 * ki.BN + ki.BM * ki.BN / 256.0;
        return tile_times * (double)steps * 1000.0 * unit * (two_groups ? 0.92 : 1.1);
    }
    if (ki.gmode == 4 || ki.gmode == 5) {
        // (two teams per workgroup, each on half of the steps, plus the exchange of the results: for problems
        // that leave compute units without a workgroup; with more tiles two workgroups per compute unit do the same)
        if (ki.variant == 2 && tiles > cus) return 1e300;
        const double st = ki.variant == 2 ? (double)((steps + 1) / 2 + 2) : (double)steps;
        return tile_times * st * 1000.0 *
               (2.75 * ki.BM + (ki.gmode == 5 ? 1.0 : 1.5) * ki.BN + ki.BM * ki.BN / 256.0);
    }
    const bool table = ki.gmode == 7 || ki.gmode == 11 || ki.gmode == 13;
    if (is_direct(ki.gmode)) {
        // 32 x 32 tiles, the wavefronts of a workgroup each on their share of the steps, operands straight from global
        // memory: a round of one step per wavefront is waves * 8 * 32 * 32 multiply-adds, bound by the loads (two
        // elements per lane and MFMA) rather than by the MFMA pipe; a fixed cost (offset table, exchange of the sums)
        // of about six steps.  Measured against the pipelined kernels on the deeper layers of Table 2: ahead up to
        // mini-batches of 32 (layer 3: 72 -> 97 TFLOP/s at 16; layer 4: 23 -> 53), level at 64, behind where tiles of
        // 64 x 64 and more fill the chip.  Element-wise filter loads (32 cache lines per instruction): three times slower.
        // With the filter rows staged in LDS (variant 1; one workgroup per compute unit) a filter load costs the address
        // unit a quarter: layer 4 at 16 / 32: 53 -> 67, 56 -> 72 TFLOP/s; with more than two tiles per compute unit the
        // two resident workgroups of the plain form do better (layer 3: 97 against 91), so it is offered up to there.
        const double waves = ki.threads / 64;
        if (ki.variant == 1 && tiles > 2 * cus) return 1e300;
        return tile_times * ((double)direct_steps_per_wave(ki, k) + 6.0) * waves * ki.BK * 32.0 *
               (32.0 + (ki.variant == 1 ? kDirectGatherCostStaged : kDirectGatherCost)) * (ki.veca ? 1.0 : 3.0) *
               (ki.gmode == 16 ? 1.03 : 1.0);   // (the window test: a little behind mode 15 where both can run)
    }
    if (ki.variant == 2) {
        // Teams: one tile per workgroup and one workgroup per compute unit at a time; each team multiplies its
        // share of the steps, the teams of a compute unit sharing its MFMA pipes - the work per compute unit is
        // that of the plain kernel, but its waits are covered (measured: about 0.8 of the time when the plain
        // kernel runs one workgroup per compute unit) and a fixed cost of about three steps is added.  Offered
        // only where the plain kernels leave compute units with a single workgroup or none.
        const int teams = ki.threads / 256;
        if (tiles > cus || steps < 8 * teams) return 1e300;
        const double gather2 = ki.gmode == 2 ? 29.0 : 6.0;
        return 0.8 * ((double)steps + 3.0 * teams) * (double)ki.BN * ki.BK * (ki.BM + gather2);
    }
    const double gather = ki.gmode == 0 ? 60.0 : (ki.gmode == 1 ? 30.0 : (ki.gmode == 2 ? 29.0 : (ki.gmode == 14 ? 18.0 : (table ? 14.0 : 6.0))));
    // (mode 11 multiplies only half of its last step; mode 13 skips the step that rounds an odd count up;
    // steps of 16 with three workgroups per compute unit: measured 2.7 % faster than steps of 32 with two)
    const double eff_steps = ki.gmode == 11 ? steps - 0.5 : (ki.gmode == 13 ? steps - 1.0 : (double)steps);
    return tile_times * eff_steps * (double)ki.BN * ki.BK * (ki.BM + gather) * (ki.BK == 16 ? 0.975 : 1.0);
}

// Largest number of pixels of the zero-extended images (flat index over all images) between
// the first pixel of a tile's first column window and the last pixel of its last column's,
// for tiles of bn consecutive columns: an upper bound.  Going from one column to the next
// advances the window start by v, by a row wrap or by an image wrap; within bn-1 such
// moves at most `rows` are wraps and at most `imgs` of those image wraps.
static long long patch_pixels_bound(const ConvKernelParams &k, int bn) {
    const long long d = bn - 1;
    const long long rows = (d + k.Q - 1) / k.Q, imgs = (d + k.PQ - 1) / k.PQ;
    const long long row_wrap = std::max<long long>((long long)k.u * k.Wp - (long long)(k.Q - 1) * k.v, k.v);
    const long long img_wrap =
        std::max<long long>((long long)k.HpWp - (long long)(k.P - 1) * k.u * k.Wp - (long long)(k.Q - 1) * k.v, row_wrap);
    return (d - rows) * k.v + (rows - imgs) * row_wrap + imgs * img_wrap + (long long)(k.R - 1) * k.Wp + k.S;
}

// Gather modes a kernel may use for this problem (see the kernel sources): the unpadded
// mode needs pad 0, the nine-tap table R*S = 9 and whole steps of four channels; the
// generic and the tap-major modes always work.  The channel-vector modes (bf16) read 8
// channels of one pixel with one 16-byte load: R*S = 9, whole steps of 16 channels, unit
// channel stride, every other stride a multiple of 8 elements and x itself 16-byte aligned;
// staging a patch of the zero-extended image needs every tile's pixel range to fit it.
// The masked filter-order mode keeps a bit per tap (up to 63 taps); the small-tile modes that
// cut the reduction inside a workgroup need an entry of their offset table for every index a
// wavefront can request, and pad 0 or - with a tap mask per column - at most 31 taps.
static bool gather_mode_ok(const KernelInfo &ki, const ConvKernelParams &k, bool x_aligned) {
    const int gmode = ki.gmode;
    if (gmode == 6 || gmode == 8 || gmode == 9 || gmode == 10) return false;  // backward-filter kernels are chosen by that pass itself
    if (gmode == 2) return k.pad_h == 0 && k.pad_w == 0;
    if (gmode == 14) return k.RS <= 63;   // (one bit of a 64-bit mask per tap, the last one spare)
    if (is_direct(gmode))   // unpadded or at most 31 taps, and every index a wavefront can request has an entry in the offset table
        return (gmode == 16 ? k.RS <= 31 : k.pad_h == 0 && k.pad_w == 0) &&
               ((long long)(ki.threads / 64) * direct_steps_per_wave(ki, k) + direct_depth(ki.BK, ki.variant == 1) + 1) * ki.BK <= kDirectTableEntries;
    if (gmode == 7 || gmode == 11 || gmode == 13) {   // unpadded, and every step the kernel can request has an entry in its offset table
        const long long steps = (k.CRS + ki.BK - 1) / ki.BK;
        if (!(k.pad_h == 0 && k.pad_w == 0 && (((steps + 1) & ~1ll) + 2) * ki.BK <= kOffsetTableEntries)) return false;
        // the short last step: an even number of steps, the last with at most half a step of real indices
        const long long last = k.CRS - (steps - 1) * ki.BK;
        if (gmode == 13) return steps % 2 == 1 && steps >= 3;   // the skipped step: the one that rounds an odd count up
        return gmode == 7 || (steps % 2 == 0 && last <= ki.BK / 2);
    }
    if (gmode == 3) return k.RS == 9 && k.C % (ki.BK / 9) == 0;  // whole steps of BK/9 channels (16-byte filter loads: checked apart)
    if (gmode == 12)   // 1x1 filters, whole 16-byte channel vectors in x and in the filter rows
        return x_aligned && k.RS == 1 && k.C % 8 == 0 && k.xsC == 1 && k.xsN % 8 == 0 && k.xsH % 8 == 0 && k.xsW % 8 == 0;
    if (gmode == 4 || gmode == 5) {
        if (!(x_aligned && k.RS == 9 && k.C % 16 == 0 && k.xsC == 1 && k.xsN % 8 == 0 && k.xsH % 8 == 0 &&
              k.xsW % 8 == 0))
            return false;
        if (k.C % (ki.BK / 9) != 0) return false;   // (whole reduction steps)
        if (gmode == 5)
            return (long long)k.N * (k.H + 2 * k.pad_h) * k.Wp < (1ll << 31) && patch_pixels_bound(k, ki.BN) <= ki.patchPixels;
    }
    return true;
}

static igcStatus choose(const igcContext *h, const Problem &pr, bool w_aligned, bool x_aligned, int *id_out) {
    const ConvKernelParams &k = pr.kp;
    const bool can_vec = w_aligned && (k.CRS % pr.vec == 0);
    // Lanes should run along y's unit-stride dimension in the epilogue.
    const bool want_swap = k.ysK == 1 && k.K > 1 && !(k.ysQ == 1 && k.Q > 1);
    if (h->kernelOverride >= 0 && pr.mode_mask == 0) {   // (the override is for the forward pass)
        const KernelInfo *ki = kernel_info(h->kernelOverride);
        if (!ki || ki->bf16 != pr.bf16 || ki->f64 != pr.f64 || (ki->veca && !can_vec) || !gather_mode_ok(*ki, k, x_aligned))
            return IGC_STATUS_NOT_SUPPORTED;
        *id_out = h->kernelOverride;
        return IGC_STATUS_SUCCESS;
    }
    int best = -1;
    double best_cost = 0;
    for (int id = 0; id < kernel_count(); ++id) {
        const KernelInfo &ki = *kernel_info(id);
        if (ki.bf16 != pr.bf16 || ki.f64 != pr.f64 || (ki.veca && !can_vec) || !gather_mode_ok(ki, k, x_aligned)) continue;
        if (pr.mode_mask != 0 && !((pr.mode_mask >> ki.gmode) & 1u)) continue;
        if (pr.no_teams && ((ki.variant == 2 && ki.gmode < 4) || is_direct(ki.gmode))) continue;
        double c = plan_cost(h, ki, k);
        if (ki.swap != want_swap) c *= 1.5;
        if (!ki.veca && can_vec && ki.gmode != 1) c *= 1.05;
        if (best < 0 || c < best_cost) {
            best = id;
            best_cost = c;
        }
    }
    if (best < 0) return IGC_STATUS_NOT_SUPPORTED;
    *id_out = best;
    return IGC_STATUS_SUCCESS;
}

// Workgroups launched per XCD.  The kernels of igconv_kernel.hpp are persistent: as many
// workgroups as the chip holds at once (32 compute units per XCD, one or two workgroups
// each depending on their LDS), each walking through several tiles; the channel-vector
// bf16 kernels take one tile per workgroup.
static int workgroups_per_xcd(const igcContext *h, const KernelInfo &ki, int tiles_per_xcd) {
    if (ki.gmode == 4 || ki.gmode == 5 || ki.gmode == 10 || (ki.f64 && ki.gmode != 14) || ki.variant == 2 || is_direct(ki.gmode)) return tiles_per_xcd;
    return std::min(tiles_per_xcd, std::max(1, h->computeUnits / kXcds) * workgroups_per_cu(ki));
}

// A float problem with a zero border and at most four channels (a first layer), which would run with the masked or the
// generic gather: over a copy of x with the border written out the same layer has no border and runs with its tap
// offsets tabulated.  Bytes of that copy, 0 when this does not apply.
static long long padded_copy_bytes(const KernelInfo &ki, const Problem &pr, igcTensorDescriptor_t xDesc) {
    const ConvKernelParams &k = pr.kp;
    if ((ki.gmode != 0 && ki.gmode != 14) || k.C > 4 || pr.bf16 || pr.f64 || (k.pad_h == 0 && k.pad_w == 0)) return 0;
    const long long bytes = (long long)k.N * k.C * (k.H + 2 * k.pad_h) * (k.W + 2 * k.pad_w) * 4;
    if (bytes >= kMaxBytes) return 0;
    for (int d = 0; d < 4; ++d)
        if (xDesc->stride[d] < 0 || xDesc->stride[d] >= (1ll << 32)) return 0;
    return bytes;
}

// Forward pass on a problem with few tiles: with a workspace the reduction can be cut into
// ranges as in the backward-filter pass (partial results summed in order afterwards), which
// puts idle compute units to work.  Returns the number of ranges (1: do not cut) and the
// steps per range.  Only for kernels whose steps stand alone (modes 0-3 and 14), outputs packed
// without gaps, and no fused epilogue; no range shorter than 8 steps.  The number of ranges
// minimises a small model of the run time in units of one reduction step: the busiest
// compute unit holds ceil(tiles*s/256) workgroups, which share its MFMA pipes, each taking
// its range plus a fixed start-up/epilogue share (about 6 steps); cutting adds the summing
// pass (about 12).  Cutting must win by a tenth, or it is not done.
static int forward_split(const igcContext *h, const KernelInfo &ki, const ConvKernelParams &k, bool packed_y, long long max_parts,
                         int *per_out) {
    const long long cus = h->computeUnits;
    *per_out = (k.ksteps + 1) & ~1;
    if ((ki.gmode > 3 && ki.gmode != 14) || ki.variant == 2 || !packed_y) return 1;
    const long long tiles = (long long)k.tilesM * k.tilesN;
    const long long smax = std::min<long long>(std::min<long long>(64, k.ksteps / 8), max_parts);
    const double kFixed = 6.0, kSumPass = 12.0;
    auto cost = [&](long long s) {
        const long long per = (k.ksteps + s - 1) / s;
        return (double)((tiles * s + cus - 1) / cus) * ((double)per + kFixed) + (s > 1 ? kSumPass : 0.0);
    };
    long long best = 1;
    for (long long s = 2; s <= smax; ++s)
        if (cost(s) < cost(best)) best = s;
    if (best == 1 || cost(best) > 0.9 * cost(1)) return 1;
    long long per = (k.ksteps + best - 1) / best;
    per += per & 1;
    *per_out = (int)per;
    return (int)((k.ksteps + per - 1) / per);
}

static igcStatus fill_plan(const igcContext *h, int id, Problem *pr, igcConvolutionForwardPlan *plan) {
    const KernelInfo &ki = *kernel_info(id);
    ConvKernelParams &k = pr->kp;
    k.tilesM = (k.K + ki.BM - 1) / ki.BM;
    k.tilesN = (k.NPQ + ki.BN - 1) / ki.BN;
    k.tilesPerXcd = (int)(((long long)k.tilesM * k.tilesN + kXcds - 1) / kXcds);
    const long long steps = pr->zero_steps ? 0 : kernel_steps(ki, k);
    if (steps >= (1ll << 30)) return IGC_STATUS_NOT_SUPPORTED;
    k.ksteps = (int)steps;
    // first step of a ragged end of the reduction range (see the kernel): tap-major order,
    // the last channel chunk; filter order, the last step; none when everything divides
    k.tail_step = -1;
    if (ki.gmode == 1 && k.C % ki.BK != 0) k.tail_step = (int)((long long)(k.C / ki.BK) * k.RS);
    if ((ki.gmode == 0 || ki.gmode == 2 || ki.gmode == 7 || ki.gmode == 11 || ki.gmode == 13 || ki.gmode == 14) && k.CRS % ki.BK != 0)
        k.tail_step = k.ksteps - 1;
    // one workgroup per tile; the runtime limits a launch to fewer than 2^32 threads
    if ((long long)k.tilesM * k.tilesN >= (1ll << 24)) return IGC_STATUS_NOT_SUPPORTED;
    k.wgsPerXcd = workgroups_per_xcd(h, ki, k.tilesPerXcd);
    k.splits = 1;
    k.stepsPerSplit = (k.ksteps + 1) & ~1;
    if (is_direct(ki.gmode)) k.stepsPerSplit = (int)direct_steps_per_wave(ki, k);
    if (ki.variant == 2 && ki.gmode < 4) {   // (fp32 team kernels: an even number of steps per team)
        const int teams = ki.threads / 256;
        k.stepsPerSplit = ((k.ksteps + teams - 1) / teams + 1) & ~1;
    }
    if (plan) {
        plan->kernelId = id;
        plan->tileM = ki.BM;
        plan->tileN = ki.BN;
        plan->tileK = ki.BK;
        plan->gridX = kXcds * k.wgsPerXcd;
        plan->kSteps = k.ksteps;
        plan->threads = ki.threads;
        plan->ldsBytes = ki.ldsBytes;
        plan->swapOperands = ki.swap ? 1 : 0;
        plan->vecFilterLoads = ki.veca ? 1 : 0;
        plan->gatherMode = ki.gmode;
    }
    return IGC_STATUS_SUCCESS;
}


// ---- backward data ------------------------------------------------------------------
// dx[n,c,h,w] = sum over (k,p,q,r,s) whose forward read lands on (h,w) of w[k,c,r,s] * dy[n,k,p,q].
// Per axis, with e the tap counted in reading direction (e = r for cross-correlation,
// R-1-r for eq. 2), the forward pass reads row p*u + e - pad.  The rows h = ph (mod u) of dx
// therefore only meet the taps e = a (mod u), a = (ph + pad) mod u: writing h = ph + u*i and
// e = a + u*t gives p = i + b - t with b = (ph + pad - a)/u.  That is a stride-1 gather over
// dy with R' = ceil((R - a)/u) taps: with tap index g = R'-1-t it reads row i + g - (R'-1-b),
// i.e. the forward kernel's own addressing with pad R'-1-b, taps walked backwards through
// the filter, and the roles of k and c exchanged.  One launch per phase (ph, pw), each
// writing its own rows and columns of dx through strides multiplied by (u, v); for u = v = 1
// there is a single phase.  A phase that meets no tap still runs, with zero reduction
// steps, so that its part of dx becomes beta * dx.
struct PhaseAxis {
    int count;   // outputs of this phase along the axis
    int taps;    // R' (0: none)
    int pad;     // pad of the equivalent stride-1 gather (may be negative)
    int tap0;    // filter index of gather tap g = 0
    int tap_step;  // filter index step per gather tap
};

static PhaseAxis phase_axis(int H, int R, int pad, int u, bool flip, int ph) {
    PhaseAxis a{};
    a.count = ph < H ? (H - ph + u - 1) / u : 0;
    const int r0 = (ph + pad) % u, b = (ph + pad) / u;
    a.taps = r0 < R ? (R - r0 + u - 1) / u : 0;
    a.pad = a.taps - 1 - b;
    const int e0 = r0 + u * (a.taps - 1);   // reading-direction tap of g = 0; g steps it by -u
    a.tap0 = flip ? R - 1 - e0 : e0;
    a.tap_step = flip ? u : -u;
    return a;
}

struct BackwardDataProblem {
    // validated sizes, forward naming
    int N, C, H, W, K, R, S, P, Q, pad_h, pad_w, u, v;
    bool flip, bf16, f64;
    long long dys[4], dxs[4];
    long long dy_bytes, w_bytes, dx_bytes;
};

static igcStatus validate_backward_data(igcFilterDescriptor_t w, igcTensorDescriptor_t dy, igcConvolutionDescriptor_t cv,
                                        igcTensorDescriptor_t dx, BackwardDataProblem *out) {
    if (!w || !dy || !cv || !dx) return IGC_STATUS_BAD_PARAM;
    if (!w->set || !dy->set || !cv->set || !dx->set) return IGC_STATUS_NOT_INITIALIZED;
    if (dx->dim[1] != w->c || dy->dim[1] != w->k || dy->dim[0] != dx->dim[0]) return IGC_STATUS_BAD_PARAM;
    const long long P = out_dim(dx->dim[2], w->r, cv->u, cv->pad_h);
    const long long Q = out_dim(dx->dim[3], w->s, cv->v, cv->pad_w);
    if (P < 1 || Q < 1 || dy->dim[2] != P || dy->dim[3] != Q) return IGC_STATUS_BAD_PARAM;
    if (!non_aliasing(dx->dim, dx->stride)) return IGC_STATUS_BAD_PARAM;
    const bool f32 = dy->dtype == IGC_DATA_FLOAT && w->dtype == IGC_DATA_FLOAT;
    const bool b16 = dy->dtype == IGC_DATA_BFLOAT16 && w->dtype == IGC_DATA_BFLOAT16;
    const bool f64 = dy->dtype == IGC_DATA_DOUBLE && w->dtype == IGC_DATA_DOUBLE;
    if (!(f32 || b16 || f64) || dx->dtype != (f64 ? IGC_DATA_DOUBLE : IGC_DATA_FLOAT)) return IGC_STATUS_NOT_SUPPORTED;
    const int es = elem_size(dy->dtype);
    BackwardDataProblem b{};
    b.f64 = f64;
    b.dy_bytes = extent(dy->dim, dy->stride) * es;
    b.dx_bytes = extent(dx->dim, dx->stride) * elem_size(dx->dtype);
    b.w_bytes = (long long)w->k * w->c * w->r * w->s * es;
    if (b.dy_bytes >= kMaxBytes || b.dx_bytes >= kMaxBytes || b.w_bytes >= kMaxBytes) return IGC_STATUS_NOT_SUPPORTED;
    if ((long long)dx->dim[0] * dx->dim[2] * dx->dim[3] >= (1ll << 30) || (long long)w->k * w->r * w->s >= (1ll << 30))
        return IGC_STATUS_NOT_SUPPORTED;
    // packed 16-bit window coordinates: sizes, pads and tap counts stay below 2^14
    if (dx->dim[2] > (1 << 14) || dx->dim[3] > (1 << 14) || cv->pad_h >= (1 << 14) || cv->pad_w >= (1 << 14) ||
        w->r > (1 << 14) || w->s > (1 << 14) || P > (1 << 14) || Q > (1 << 14))
        return IGC_STATUS_NOT_SUPPORTED;
    b.N = dx->dim[0]; b.C = dx->dim[1]; b.H = dx->dim[2]; b.W = dx->dim[3];
    b.K = w->k; b.R = w->r; b.S = w->s; b.P = (int)P; b.Q = (int)Q;
    b.pad_h = cv->pad_h; b.pad_w = cv->pad_w; b.u = cv->u; b.v = cv->v;
    b.flip = cv->mode == IGC_CONVOLUTION;
    b.bf16 = b16;
    for (int i = 0; i < 4; ++i) { b.dys[i] = dy->stride[i]; b.dxs[i] = dx->stride[i]; }
    if (out) *out = b;
    return IGC_STATUS_SUCCESS;
}

// The launch parameters of phase (ph, pw); false when the phase has no output element.
static bool backward_data_phase(const BackwardDataProblem &b, int ph, int pw, Problem *pr, long long *dx_offset) {
    const PhaseAxis ah = phase_axis(b.H, b.R, b.pad_h, b.u, b.flip, ph);
    const PhaseAxis aw = phase_axis(b.W, b.S, b.pad_w, b.v, b.flip, pw);
    if (ah.count <= 0 || aw.count <= 0) return false;
    *pr = Problem{};
    pr->bf16 = b.bf16;
    pr->f64 = b.f64;
    pr->vec = b.bf16 ? 8 : (b.f64 ? 2 : 4);
    // tap-major, the nine-tap table when the phase has nine taps, or filter order under a tap mask; double precision:
    // the tap mask, or the generic gather
    pr->mode_mask = b.f64 ? (1u << 0) | (1u << 14) : (1u << 1) | (1u << 3) | (1u << 14);
    pr->zero_steps = ah.taps == 0 || aw.taps == 0;
    ConvKernelParams &k = pr->kp;
    const int es = b.bf16 ? 2 : 4;
    const int out_es = b.f64 ? 8 : 4;
    const int Rp = std::max(ah.taps, 1), Sp = std::max(aw.taps, 1);
    *dx_offset = (long long)ph * b.dxs[2] + (long long)pw * b.dxs[3];
    k.x_bytes = (uint32_t)b.dy_bytes;
    k.w_bytes = (uint32_t)b.w_bytes;
    k.y_bytes = (uint32_t)(b.dx_bytes - *dx_offset * out_es);
    // the gather runs over dy: its channels are the reduction, its rows and columns the image
    k.N = b.N; k.C = b.K; k.H = b.P; k.W = b.Q;
    k.K = b.C; k.R = Rp; k.S = Sp; k.P = ah.count; k.Q = aw.count;
    k.pad_h = ah.pad; k.pad_w = aw.pad; k.u = 1; k.v = 1; k.flip = 0;
    k.RS = Rp * Sp; k.CRS = b.K * k.RS; k.PQ = ah.count * aw.count; k.NPQ = b.N * k.PQ;
    k.Wp = 1; k.HpWp = 1;   // (patch staging is never used here)
    magic_for(1, &k.mWp); magic_for(1, &k.mHpWp);
    magic_for((uint32_t)k.PQ, &k.mPQ); magic_for((uint32_t)k.Q, &k.mQ);
    magic_for((uint32_t)k.RS, &k.mRS); magic_for((uint32_t)k.S, &k.mS);
    k.wsRow = b.R * b.S; k.wsRed = b.C * b.R * b.S;
    k.wTap0 = ah.tap0 * b.S + aw.tap0; k.wsTapR = ah.tap_step * b.S; k.wsTapS = aw.tap_step;
    k.xsN = (int)b.dys[0]; k.xsC = (int)b.dys[1]; k.xsH = (int)b.dys[2]; k.xsW = (int)b.dys[3];
    k.ysN = (int)b.dxs[0]; k.ysK = (int)b.dxs[1]; k.ysP = (int)(b.dxs[2] * b.u); k.ysQ = (int)(b.dxs[3] * b.v);
    (void)es;
    return true;
}


// bf16 with unit stride, nine taps or one and dy's channels contiguous: backward data IS a
// forward pass over dy with the filter's k and c exchanged and its taps read in the other
// direction (tap g of the gather is filter tap R-1-g resp. g for eq. 2), pad R-1-pad.  With
// the exchanged filter written to a workspace (K*C*R*S elements) the channel-vector kernels
// of the forward pass apply.  False when the problem does not have that shape.
static bool backward_data_as_forward(const BackwardDataProblem &b, Problem *pr) {
    const int taps = b.R * b.S;
    if (!b.bf16 || b.u != 1 || b.v != 1 || (taps != 9 && taps != 1) || b.K % (taps == 9 ? 16 : 8) != 0 || b.dys[1] != 1) return false;
    if (b.pad_h > b.R - 1 || b.pad_w > b.S - 1) return false;
    *pr = Problem{};
    pr->bf16 = true;
    pr->vec = 8;
    pr->mode_mask = taps == 9 ? (1u << 4) | (1u << 5) : 1u << 12;
    ConvKernelParams &k = pr->kp;
    k.x_bytes = (uint32_t)b.dy_bytes;
    k.w_bytes = (uint32_t)b.w_bytes;
    k.y_bytes = (uint32_t)b.dx_bytes;
    k.N = b.N; k.C = b.K; k.H = b.P; k.W = b.Q;
    k.K = b.C; k.R = b.R; k.S = b.S; k.P = b.H; k.Q = b.W;
    k.pad_h = b.R - 1 - b.pad_h; k.pad_w = b.S - 1 - b.pad_w; k.u = 1; k.v = 1;
    k.flip = b.flip ? 0 : 1;
    k.RS = taps; k.CRS = b.K * taps; k.PQ = b.H * b.W; k.NPQ = b.N * k.PQ;
    k.Wp = k.W + 2 * k.pad_w;
    k.HpWp = (int)std::min<long long>((long long)(k.H + 2 * k.pad_h) * k.Wp, 0x7fffffff);
    if (!magic_for((uint32_t)k.Wp, &k.mWp) || !magic_for((uint32_t)k.HpWp, &k.mHpWp)) return false;
    if (!magic_for((uint32_t)k.PQ, &k.mPQ) || !magic_for((uint32_t)k.Q, &k.mQ) ||
        !magic_for((uint32_t)k.RS, &k.mRS) || !magic_for((uint32_t)k.S, &k.mS))
        return false;
    k.wsRow = k.CRS; k.wsRed = k.RS; k.wTap0 = 0; k.wsTapR = k.S; k.wsTapS = 1;
    k.xsN = (int)b.dys[0]; k.xsC = 1; k.xsH = (int)b.dys[2]; k.xsW = (int)b.dys[3];
    k.ysN = (int)b.dxs[0]; k.ysK = (int)b.dxs[1]; k.ysP = (int)b.dxs[2]; k.ysQ = (int)b.dxs[3];
    return true;
}

// ---- backward filter ------------------------------------------------------------------
// dw[k,c,r,s] = sum_{n,p,q} dy[n,k,p,q] * x0[n,c,row(p,r),col(q,s)]: an implicit GEMM with rows
// k, columns i = (c,r,s) and the reduction over j = (n,p,q).  The gathered operand is x
// again, with the two index sets exchanged: a column fixes (c, tap) and therefore the
// window origin tap - pad (tap counted in reading direction), a reduction index adds
// (p*u, q*v).  The kernel's generic gather does exactly that once its divisors, strides
// and multipliers are renamed; the first operand is dy, read through its strides.  The
// output is small (K x CRS) and the reduction long (NPQ), so the reduction is cut into
// ranges that run as separate workgroups, each writing a partial result into the
// workspace; a second kernel adds the parts in order (deterministic) and applies alpha
// and beta.  Without workspace the whole reduction runs in one range, straight into dw.
struct BackwardFilterProblem {
    Problem pr;        // launch parameters with splits = 1, writing dw directly
    int kernel_id;
    long long ksteps;  // reduction steps in all
    long long tiles;   // output tiles
    long long tiles_n; // of which along the columns
    uint32_t out_elems;  // K*C*R*S
    // channel-vector kernels (gather mode 10): a part of the workspace holds [tap][row position][column position],
    // rows and columns padded to whole tiles; 0 for the other kernels, whose parts are copies of dw
    long long pos_rows = 0, pos_cols = 0;
    long long part_elems() const { return pos_rows ? pos_rows * pos_cols * (out_elems / (pr.kp.K * (long long)pr.kp.NPQ)) : out_elems; }
};

static igcStatus validate_backward_filter(igcTensorDescriptor_t x, igcTensorDescriptor_t dy,
                                          igcConvolutionDescriptor_t cv, igcFilterDescriptor_t dw,
                                          BackwardFilterProblem *out, bool aligned16 = true) {
    if (!x || !dy || !cv || !dw) return IGC_STATUS_BAD_PARAM;
    if (!x->set || !dy->set || !cv->set || !dw->set) return IGC_STATUS_NOT_INITIALIZED;
    if (x->dim[1] != dw->c || dy->dim[1] != dw->k || dy->dim[0] != x->dim[0]) return IGC_STATUS_BAD_PARAM;
    const long long P = out_dim(x->dim[2], dw->r, cv->u, cv->pad_h);
    const long long Q = out_dim(x->dim[3], dw->s, cv->v, cv->pad_w);
    if (P < 1 || Q < 1 || dy->dim[2] != P || dy->dim[3] != Q) return IGC_STATUS_BAD_PARAM;
    const bool f32 = x->dtype == IGC_DATA_FLOAT && dy->dtype == IGC_DATA_FLOAT;
    const bool b16 = x->dtype == IGC_DATA_BFLOAT16 && dy->dtype == IGC_DATA_BFLOAT16;
    const bool f64 = x->dtype == IGC_DATA_DOUBLE && dy->dtype == IGC_DATA_DOUBLE;
    if (!(f32 || b16 || f64) || dw->dtype != (f64 ? IGC_DATA_DOUBLE : IGC_DATA_FLOAT)) return IGC_STATUS_NOT_SUPPORTED;
    const int es = elem_size(x->dtype);
    const long long xb = extent(x->dim, x->stride) * es, dyb = extent(dy->dim, dy->stride) * es;
    const long long CRS = (long long)dw->c * dw->r * dw->s, NPQ = (long long)x->dim[0] * P * Q;
    const long long dwb = (long long)dw->k * CRS * elem_size(dw->dtype);
    if (xb >= kMaxBytes || dyb >= kMaxBytes || dwb >= kMaxBytes) return IGC_STATUS_NOT_SUPPORTED;
    if (NPQ >= (1ll << 30) || CRS >= (1ll << 30)) return IGC_STATUS_NOT_SUPPORTED;
    // packed 16-bit window coordinates: here the reduction index contributes up to
    // (P-1)*u <= H + 2 pad - R, which must stay below 2^14 like the image size itself
    if (x->dim[2] + 2ll * cv->pad_h > (1 << 14) || x->dim[3] + 2ll * cv->pad_w > (1 << 14)) return IGC_STATUS_NOT_SUPPORTED;
    if (!out) return IGC_STATUS_SUCCESS;

    *out = BackwardFilterProblem{};
    Problem &pr = out->pr;
    pr.bf16 = b16;
    pr.f64 = f64;
    pr.vec = 16 / es;
    pr.mode_mask = 1u << 6;
    ConvKernelParams &k = pr.kp;
    const bool flip = cv->mode == IGC_CONVOLUTION;
    k.x_bytes = (uint32_t)xb;
    k.w_bytes = (uint32_t)dyb;
    k.y_bytes = (uint32_t)dwb;
    k.N = x->dim[0]; k.C = x->dim[1]; k.H = x->dim[2]; k.W = x->dim[3];
    k.K = dw->k; k.R = dw->r; k.S = dw->s; k.P = (int)P; k.Q = dw->s;
    // columns (c,r,s): window origin (tap - pad) with the tap in reading direction
    k.PQ = dw->r * dw->s; k.NPQ = (int)CRS;
    k.u = flip ? -1 : 1; k.v = flip ? -1 : 1;
    k.pad_h = flip ? cv->pad_h - (dw->r - 1) : cv->pad_h;
    k.pad_w = flip ? cv->pad_w - (dw->s - 1) : cv->pad_w;
    // reduction (n,p,q): adds (p*u, q*v)
    k.RS = (int)(P * Q); k.CRS = (int)NPQ;
    const int red_inner = (int)Q;
    k.flip = 0; k.redMulH = cv->u; k.redMulW = cv->v;
    k.Wp = 1; k.HpWp = 1;
    magic_for(1, &k.mWp); magic_for(1, &k.mHpWp);
    magic_for((uint32_t)k.PQ, &k.mPQ); magic_for((uint32_t)k.Q, &k.mQ);
    magic_for((uint32_t)k.RS, &k.mRS); magic_for((uint32_t)red_inner, &k.mS);
    k.S = red_inner;   // (from here on S is the reduction's inner divisor, Q of the forward pass)
    k.xsN = (int)x->stride[1]; k.xsC = (int)x->stride[0]; k.xsH = (int)x->stride[2]; k.xsW = (int)x->stride[3];
    k.ysN = dw->r * dw->s; k.ysK = (int)CRS; k.ysP = dw->s; k.ysQ = 1;
    k.wsRow = (int)dy->stride[1]; k.wsRed = (int)dy->stride[0]; k.wsTapR = (int)dy->stride[2]; k.wsTapS = (int)dy->stride[3];
    k.splits = 1;
    out->out_elems = (uint32_t)(dw->k * CRS);
    // Two ways to run it.  Enough channels to fill a column tile: columns ordered (tap, channel),
    // one tap per tile (gather mode 8; any filter size).  Otherwise the generic gather over
    // columns (c,r,s) set up above (mode 6).  Row tile: the smaller one when it covers K.
    const bool by_tap = dw->c >= 24 && !f64;   // (double precision has the generic gather only)
    // bf16 with unit channel strides, whole 16-byte channel vectors everywhere: columns (tap, channel) as for
    // mode 8, operands loaded as channel vectors and transposed on the way into LDS (mode 10)
    bool vectors = b16 && by_tap && aligned16 && x->stride[1] == 1 && dy->stride[1] == 1 && dw->c % 8 == 0 && dw->k % 8 == 0;
    for (int d : {0, 2, 3})
        if (x->stride[d] % 8 != 0 || dy->stride[d] % 8 != 0) vectors = false;
    const bool unpadded = !by_tap && !f64 && cv->pad_h == 0 && cv->pad_w == 0;   // few channels, no padding: mode 9
    const int want_mode = vectors ? 10 : (by_tap ? 8 : (unpadded ? 9 : 6));
    if (f64) {
        for (int i = 0; i < kernel_count(); ++i)
            if (kernel_info(i)->f64 && kernel_info(i)->gmode == 6) out->kernel_id = i;
        const KernelInfo &kf = *kernel_info(out->kernel_id);
        out->ksteps = (NPQ + kf.BK - 1) / kf.BK;
        out->tiles_n = (CRS + kf.BN - 1) / kf.BN;
        out->tiles = (long long)((dw->k + kf.BM - 1) / kf.BM) * out->tiles_n;
        return IGC_STATUS_SUCCESS;
    }
    // row tile: least padding of K among 64, 96 (fp32 only), 128; the larger one on a tie
    int want_bm = 64;
    for (int bm : {96, 128}) {
        if (bm == 96 && b16) continue;
        if (vectors && dw->k <= 64) continue;   // (the vector kernels run one tile per workgroup: no gain from padding K)
        const long long pad_new = (long long)((dw->k + bm - 1) / bm) * bm, pad_old = (long long)((dw->k + want_bm - 1) / want_bm) * want_bm;
        if (pad_new <= pad_old) want_bm = bm;
    }
    const int want_bn = !by_tap ? 128 : ((dw->c - 1) % 128 < 64 ? 64 : 128);   // (least padding of C)
    int id = -1;
    for (int attempt = 0; attempt < 2 && id < 0; ++attempt) {
        for (int i = 0; i < kernel_count(); ++i) {
            const KernelInfo &ki = *kernel_info(i);
            if (ki.gmode == want_mode && ki.bf16 == b16 && ki.BM == want_bm && ki.BN == want_bn) id = i;
        }
        if (id < 0) want_bm = 128;   // (not every tile shape exists with 96 rows)
    }
    if (id < 0) return IGC_STATUS_NOT_SUPPORTED;
    out->kernel_id = id;
    const KernelInfo &ki = *kernel_info(id);
    out->ksteps = (NPQ + ki.BK - 1) / ki.BK;
    pr.mode_mask = 1u << ki.gmode;
    if (by_tap) {
        // columns: channels c < C at distance R*S in dw, the tap chosen per tile; PQ = channel
        // blocks per tap, Q = S and R = R decode the tile's tap; the window test uses the
        // forward pads and mode directly
        const int cblocks = (dw->c + ki.BN - 1) / ki.BN;
        k.NPQ = dw->c; k.PQ = cblocks; k.Q = dw->s; k.R = dw->r;
        k.flip = flip ? 1 : 0; k.pad_h = cv->pad_h; k.pad_w = cv->pad_w; k.u = 1; k.v = 1;
        magic_for((uint32_t)k.PQ, &k.mPQ); magic_for((uint32_t)k.Q, &k.mQ);
        k.ysQ = dw->r * dw->s; k.ysN = 0; k.ysP = 0;
        out->tiles_n = (long long)dw->r * dw->s * cblocks;
        if (ki.gmode == 10) {
            out->pos_rows = (long long)((dw->k + ki.BM - 1) / ki.BM) * ki.BM;
            out->pos_cols = (long long)cblocks * ki.BN;
            if (out->pos_rows * out->pos_cols * dw->r * dw->s * 4 >= kMaxBytes) return IGC_STATUS_NOT_SUPPORTED;
        }
    } else if (unpadded) {
        // columns (c,r,s) in filter order at distance 1 in dw; PQ = R*S, Q = S and R decode a column
        k.NPQ = (int)CRS; k.PQ = dw->r * dw->s; k.Q = dw->s; k.R = dw->r;
        k.flip = flip ? 1 : 0; k.pad_h = 0; k.pad_w = 0; k.u = 1; k.v = 1;
        magic_for((uint32_t)k.PQ, &k.mPQ); magic_for((uint32_t)k.Q, &k.mQ);
        k.ysQ = 1; k.ysN = 0; k.ysP = 0;
        out->tiles_n = (CRS + ki.BN - 1) / ki.BN;
    } else {
        out->tiles_n = (CRS + ki.BN - 1) / ki.BN;
    }
    out->tiles = (long long)((dw->k + ki.BM - 1) / ki.BM) * out->tiles_n;
    return IGC_STATUS_SUCCESS;
}

// The general route of backward data: one launch per phase, each planned like a forward problem.
struct PhaseLaunch {
    Problem pr;
    int id, grid;
    long long dx_offset;   // elements of dx before the phase's first one
};

static igcStatus plan_backward_data_phases(const igcContext *handle, const BackwardDataProblem &b, std::vector<PhaseLaunch> *out) {
    for (int ph = 0; ph < b.u; ++ph)
        for (int pw = 0; pw < b.v; ++pw) {
            PhaseLaunch l;
            l.dx_offset = 0;
            if (!backward_data_phase(b, ph, pw, &l.pr, &l.dx_offset)) continue;
            igcStatus st = choose(handle, l.pr, /*w_aligned=*/false, /*x_aligned=*/false, &l.id);
            if (st != IGC_STATUS_SUCCESS) return st;
            igcConvolutionForwardPlan plan;
            st = fill_plan(handle, l.id, &l.pr, &plan);
            if (st != IGC_STATUS_SUCCESS) return st;
            l.grid = plan.gridX;
            out->push_back(l);
        }
    return IGC_STATUS_SUCCESS;
}

// Float or bfloat16 phases that all run in tap-major order (and have something to reduce): their filter reads, elements
// C*R*S apart, become contiguous with the filter rewritten as wt[c][t][k] in a workspace of the filter's size.
static bool phases_want_filter_workspace(const BackwardDataProblem &b, const std::vector<PhaseLaunch> &launches) {
    if (b.f64 || launches.empty() || b.K < 2) return false;
    for (const PhaseLaunch &l : launches)
        if (kernel_info(l.id)->gmode != 1) return false;
    return true;
}

// Backward data of a strided layer with few channels as one forward pass over dy with u*v*C output maps (see
// igconv_kernels_wgrad.hip): float only, a stride above 1, at most 128 such maps (beyond that the per-phase
// launches fill their tiles anyway).  The workspace holds the filter of that pass, then its result.
struct PackedPhases {
    int Rp, Sp, I, J, maps;
    long long filter_bytes, bytes;   // (filter_bytes: rounded up to a multiple of 256)
};

static bool packed_phases(const BackwardDataProblem &b, PackedPhases *out) {
    if (b.bf16 || b.f64 || b.u * b.v <= 1) return false;
    const long long maps = (long long)b.u * b.v * b.C;
    if (maps > 128) return false;
    PackedPhases p{};
    p.maps = (int)maps;
    p.Rp = (b.R + b.u - 1) / b.u;
    p.Sp = (b.S + b.v - 1) / b.v;
    p.I = b.P + p.Rp - 1;
    p.J = b.Q + p.Sp - 1;
    const long long fb = maps * b.K * p.Rp * p.Sp * 4, yb = (long long)b.N * maps * p.I * p.J * 4;
    p.filter_bytes = (fb + 255) / 256 * 256;
    p.bytes = p.filter_bytes + yb;
    if (yb >= kMaxBytes || fb >= kMaxBytes || (long long)b.N * b.C * b.H * b.W >= (1ll << 32)) return false;
    for (int d = 0; d < 4; ++d)
        if (b.dxs[d] >= (1ll << 32)) return false;
    *out = p;
    return true;
}

// How to cut the reduction: as many ranges as keep all (tile, range) workgroups resident at
// once (two per compute unit, four of the small fp32 tiles and of the double-precision kernel) - one more would leave
// a second, nearly empty round -, ranges of an even number of steps and not shorter than 8; at most max_parts ranges.
// (Double precision: possibly finer, see below.)
static void backward_filter_split(const igcContext *h, const BackwardFilterProblem &b, long long max_parts, int *splits,
                                  int *steps_per_split) {
    const long long cus = h->computeUnits;
    const KernelInfo *ki = kernel_info(b.kernel_id);
    const long long per_cu = ki && ki->f64 ? 4 : (ki && ki->gmode != 10 ? workgroups_per_cu(*ki) : 2);
    long long want = std::max<long long>(1, (per_cu * cus) / b.tiles);
    want = std::min(want, std::max<long long>(1, b.ksteps / 8));
    want = std::min(want, std::max<long long>(1, max_parts));
    if (ki && (ki->f64 || ki->gmode == 10)) {
        // These kernels run one workgroup per (tile, range), handed to the compute units as they come free.  With few
        // ranges per tile the rounding above leaves compute units short of a workgroup (double precision, 216 tiles:
        // 4 ranges, 864 workgroups, three or four per compute unit - the ones with four set the time).  Finer ranges
        // even that out: the busiest compute unit does ceil(tiles * ranges / compute units) workgroups of
        // steps / ranges + 3 steps (start-up), and every range adds its pass of the ordered sum (in steps: a part's
        // bytes by 1.5 MB in double precision, by 1.9 MB for the bf16 channel-vector kernels).  Measured, double precision
        // on those 216 tiles: 4 ranges 412 us, 7 ranges 358, 13 ranges 355, 28 ranges 372; bf16, 144 tiles, mini-batch
        // 256: 3 ranges 271 us, 5 264, 7 256, 10 273 (mini-batch 32: 3 ranges 48 us, more are slower - as the model says).
        // The workspace stays within the scratch array of the allocation-free entry point.
        const double part_bytes = (double)b.part_elems() * (ki->f64 ? 8.0 : 4.0);
        const long long by_bytes = (long long)((double)IGC_NOALLOC_SCRATCH_BYTES / part_bytes);
        const long long hi = std::min({std::max(want, std::min(4 * want, by_bytes)), std::max<long long>(1, b.ksteps / 8),
                                       std::max<long long>(1, max_parts)});
        const double sum_steps = part_bytes / (ki->f64 ? 1.5e6 : 1.9e6);
        double base = 0.0, best = 0.0;
        long long pick = want;
        for (long long s = want; s <= hi; ++s) {
            const double cost = (double)((b.tiles * s + cus - 1) / cus) * ((double)b.ksteps / (double)s + 3.0) + (double)s * sum_steps;
            if (s == want) base = best = cost;
            if (cost < best && cost < base * 0.98) {   // (a finer cut must pay: it also takes more workspace)
                best = cost;
                pick = s;
            }
        }
        want = pick;
    }
    long long per = (b.ksteps + want - 1) / want;
    per += per & 1;
    *steps_per_split = (int)per;
    *splits = (int)((b.ksteps + per - 1) / per);
}

}  // namespace igc

using namespace igc;

extern "C" {

const char *igcGetErrorString(igcStatus status) {
    switch (status) {
        case IGC_STATUS_SUCCESS: return "IGC_STATUS_SUCCESS";
        case IGC_STATUS_BAD_PARAM: return "IGC_STATUS_BAD_PARAM";
        case IGC_STATUS_NOT_SUPPORTED: return "IGC_STATUS_NOT_SUPPORTED";
        case IGC_STATUS_NOT_INITIALIZED: return "IGC_STATUS_NOT_INITIALIZED";
        case IGC_STATUS_ALLOC_FAILED: return "IGC_STATUS_ALLOC_FAILED";
        case IGC_STATUS_EXECUTION_FAILED: return "IGC_STATUS_EXECUTION_FAILED";
    }
    return "IGC_STATUS_UNKNOWN";
}

igcStatus igcCreate(igcHandle_t *handle) {
    if (!handle) return IGC_STATUS_BAD_PARAM;
    igcContext *c = new (std::nothrow) igcContext;
    if (!c) return IGC_STATUS_ALLOC_FAILED;
    const int cus = igc::query_compute_units();   // (0: no device to ask)
    if (cus >= igc::kXcds) c->computeUnits = cus;
    *handle = c;
    return IGC_STATUS_SUCCESS;
}

igcStatus igcDestroy(igcHandle_t handle) {
    if (!handle) return IGC_STATUS_BAD_PARAM;
    delete handle;
    return IGC_STATUS_SUCCESS;
}

igcStatus igcSetStream(igcHandle_t handle, void *hipStream) {
    if (!handle) return IGC_STATUS_BAD_PARAM;
    handle->stream = hipStream;
    return IGC_STATUS_SUCCESS;
}

igcStatus igcGetStream(igcHandle_t handle, void **hipStream) {
    if (!handle || !hipStream) return IGC_STATUS_BAD_PARAM;
    *hipStream = handle->stream;
    return IGC_STATUS_SUCCESS;
}

igcStatus igcCreateTensorDescriptor(igcTensorDescriptor_t *desc) {
    if (!desc) return IGC_STATUS_BAD_PARAM;
    igcTensorStruct *d = new (std::nothrow) igcTensorStruct;
    if (!d) return IGC_STATUS_ALLOC_FAILED;
    *desc = d;
    return IGC_STATUS_SUCCESS;
}

igcStatus igcDestroyTensorDescriptor(igcTensorDescriptor_t desc) {
    if (!desc) return IGC_STATUS_BAD_PARAM;
    delete desc;
    return IGC_STATUS_SUCCESS;
}

igcStatus igcSetTensor4dDescriptor(igcTensorDescriptor_t desc, igcDataType dataType, int n, int c, int h,
                                   int w, long long nStride, long long cStride, long long hStride,
                                   long long wStride) {
    if (!desc) return IGC_STATUS_BAD_PARAM;
    if (dataType != IGC_DATA_FLOAT && dataType != IGC_DATA_BFLOAT16 && dataType != IGC_DATA_DOUBLE) return IGC_STATUS_BAD_PARAM;
    if (n < 1 || c < 1 || h < 1 || w < 1) return IGC_STATUS_BAD_PARAM;
    if (nStride < 0 || cStride < 0 || hStride < 0 || wStride < 0) return IGC_STATUS_BAD_PARAM;
    const int dim[4] = {n, c, h, w};
    const long long stride[4] = {nStride, cStride, hStride, wStride};
    // keep the extent computable without overflow
    for (int i = 0; i < 4; ++i)
        if (stride[i] >= kMaxBytes) return IGC_STATUS_NOT_SUPPORTED;
    desc->dtype = dataType;
    for (int i = 0; i < 4; ++i) {
        desc->dim[i] = dim[i];
        desc->stride[i] = stride[i];
    }
    desc->set = true;
    return IGC_STATUS_SUCCESS;
}

igcStatus igcGetTensor4dDescriptor(igcTensorDescriptor_t desc, igcDataType *dataType, int *n, int *c, int *h,
                                   int *w, long long *nStride, long long *cStride, long long *hStride,
                                   long long *wStride) {
    if (!desc || !dataType || !n || !c || !h || !w || !nStride || !cStride || !hStride || !wStride)
        return IGC_STATUS_BAD_PARAM;
    if (!desc->set) return IGC_STATUS_NOT_INITIALIZED;
    *dataType = desc->dtype;
    *n = desc->dim[0]; *c = desc->dim[1]; *h = desc->dim[2]; *w = desc->dim[3];
    *nStride = desc->stride[0]; *cStride = desc->stride[1]; *hStride = desc->stride[2]; *wStride = desc->stride[3];
    return IGC_STATUS_SUCCESS;
}

igcStatus igcCreateFilterDescriptor(igcFilterDescriptor_t *desc) {
    if (!desc) return IGC_STATUS_BAD_PARAM;
    igcFilterStruct *d = new (std::nothrow) igcFilterStruct;
    if (!d) return IGC_STATUS_ALLOC_FAILED;
    *desc = d;
    return IGC_STATUS_SUCCESS;
}

igcStatus igcDestroyFilterDescriptor(igcFilterDescriptor_t desc) {
    if (!desc) return IGC_STATUS_BAD_PARAM;
    delete desc;
    return IGC_STATUS_SUCCESS;
}

igcStatus igcSetFilter4dDescriptor(igcFilterDescriptor_t desc, igcDataType dataType, int k, int c, int r, int s) {
    if (!desc) return IGC_STATUS_BAD_PARAM;
    if (dataType != IGC_DATA_FLOAT && dataType != IGC_DATA_BFLOAT16 && dataType != IGC_DATA_DOUBLE) return IGC_STATUS_BAD_PARAM;
    if (k < 1 || c < 1 || r < 1 || s < 1) return IGC_STATUS_BAD_PARAM;
    desc->dtype = dataType;
    desc->k = k; desc->c = c; desc->r = r; desc->s = s;
    desc->set = true;
    return IGC_STATUS_SUCCESS;
}

igcStatus igcGetFilter4dDescriptor(igcFilterDescriptor_t desc, igcDataType *dataType, int *k, int *c, int *r, int *s) {
    if (!desc || !dataType || !k || !c || !r || !s) return IGC_STATUS_BAD_PARAM;
    if (!desc->set) return IGC_STATUS_NOT_INITIALIZED;
    *dataType = desc->dtype;
    *k = desc->k; *c = desc->c; *r = desc->r; *s = desc->s;
    return IGC_STATUS_SUCCESS;
}

igcStatus igcCreateConvolutionDescriptor(igcConvolutionDescriptor_t *desc) {
    if (!desc) return IGC_STATUS_BAD_PARAM;
    igcConvolutionStruct *d = new (std::nothrow) igcConvolutionStruct;
    if (!d) return IGC_STATUS_ALLOC_FAILED;
    *desc = d;
    return IGC_STATUS_SUCCESS;
}

igcStatus igcDestroyConvolutionDescriptor(igcConvolutionDescriptor_t desc) {
    if (!desc) return IGC_STATUS_BAD_PARAM;
    delete desc;
    return IGC_STATUS_SUCCESS;
}

igcStatus igcSetConvolution2dDescriptor(igcConvolutionDescriptor_t desc, int pad_h, int pad_w, int u, int v,
                                        igcConvolutionMode mode) {
    if (!desc) return IGC_STATUS_BAD_PARAM;
    if (pad_h < 0 || pad_w < 0 || u < 1 || v < 1) return IGC_STATUS_BAD_PARAM;
    if (mode != IGC_CONVOLUTION && mode != IGC_CROSS_CORRELATION) return IGC_STATUS_BAD_PARAM;
    desc->pad_h = pad_h; desc->pad_w = pad_w; desc->u = u; desc->v = v;
    desc->mode = mode;
    desc->set = true;
    return IGC_STATUS_SUCCESS;
}

igcStatus igcGetConvolution2dDescriptor(igcConvolutionDescriptor_t desc, int *pad_h, int *pad_w, int *u, int *v,
                                        igcConvolutionMode *mode) {
    if (!desc || !pad_h || !pad_w || !u || !v || !mode) return IGC_STATUS_BAD_PARAM;
    if (!desc->set) return IGC_STATUS_NOT_INITIALIZED;
    *pad_h = desc->pad_h; *pad_w = desc->pad_w; *u = desc->u; *v = desc->v;
    *mode = desc->mode;
    return IGC_STATUS_SUCCESS;
}

igcStatus igcGetConvolution2dForwardOutputDim(igcConvolutionDescriptor_t convDesc, igcTensorDescriptor_t xDesc,
                                              igcFilterDescriptor_t wDesc, int *n, int *k, int *p, int *q) {
    if (!convDesc || !xDesc || !wDesc || !n || !k || !p || !q) return IGC_STATUS_BAD_PARAM;
    if (!convDesc->set || !xDesc->set || !wDesc->set) return IGC_STATUS_NOT_INITIALIZED;
    if (xDesc->dim[1] != wDesc->c) return IGC_STATUS_BAD_PARAM;
    const long long P = out_dim(xDesc->dim[2], wDesc->r, convDesc->u, convDesc->pad_h);
    const long long Q = out_dim(xDesc->dim[3], wDesc->s, convDesc->v, convDesc->pad_w);
    if (P < 1 || Q < 1 || P > 0x7fffffff || Q > 0x7fffffff) return IGC_STATUS_BAD_PARAM;
    *n = xDesc->dim[0];
    *k = wDesc->k;
    *p = (int)P;
    *q = (int)Q;
    return IGC_STATUS_SUCCESS;
}

igcStatus igcGetConvolutionForwardWorkspaceSize(igcHandle_t handle, igcTensorDescriptor_t xDesc,
                                                igcFilterDescriptor_t wDesc, igcConvolutionDescriptor_t convDesc,
                                                igcTensorDescriptor_t yDesc, size_t *sizeInBytes) {
    if (!handle || !sizeInBytes) return IGC_STATUS_BAD_PARAM;
    const igcStatus st = validate(xDesc, wDesc, convDesc, yDesc, nullptr);
    if (st != IGC_STATUS_SUCCESS) return st;
    *sizeInBytes = 0;  // the lowered matrix only ever exists in LDS
    return IGC_STATUS_SUCCESS;
}

igcStatus igcGetConvolutionForwardOptionalWorkspaceSize(igcHandle_t handle, igcTensorDescriptor_t xDesc,
                                                        igcFilterDescriptor_t wDesc, igcConvolutionDescriptor_t convDesc,
                                                        igcTensorDescriptor_t yDesc, size_t *sizeInBytes) {
    if (!handle || !sizeInBytes) return IGC_STATUS_BAD_PARAM;
    Problem pr;
    igcStatus st = validate(xDesc, wDesc, convDesc, yDesc, &pr);
    if (st != IGC_STATUS_SUCCESS) return st;
    int id = -1;
    pr.no_teams = true;   // (as the forward call does when it is lent a workspace)
    st = choose(handle, pr, /*w_aligned=*/true, /*x_aligned=*/true, &id);
    if (st != IGC_STATUS_SUCCESS) return st;
    st = fill_plan(handle, id, &pr, nullptr);
    if (st != IGC_STATUS_SUCCESS) return st;
    const bool packed = extent(yDesc->dim, yDesc->stride) == (long long)pr.kp.K * pr.kp.NPQ;
    int per;
    const int splits = pr.f64 ? 1 : forward_split(handle, *kernel_info(id), pr.kp, packed, 1 << 20, &per);
    *sizeInBytes = splits > 1 ? (size_t)splits * pr.kp.y_bytes : 0;
    // a float problem that runs in tap-major order: room for the filter with the channel index innermost
    if (splits <= 1 && kernel_info(id)->gmode == 1 && !pr.f64 && pr.kp.RS > 1) *sizeInBytes = (size_t)pr.kp.w_bytes;
    // few channels and a zero border: room for x with the border written out
    if (splits <= 1 && padded_copy_bytes(*kernel_info(id), pr, xDesc) > 0) *sizeInBytes = (size_t)padded_copy_bytes(*kernel_info(id), pr, xDesc);
    return IGC_STATUS_SUCCESS;
}

// One past the largest byte offset the kernels form for an existing element of each argument, in 64 bits from the
// launch parameters: the gathered tensor at the last image, last reduction channel and the last row and column any
// window reaches inside the image; the filter at the last row, last reduction channel and the tap of largest offset
// (tap strides may be negative); the output at the last column and row of O_m.
static void address_reach(const ConvKernelParams &k, int es_in, int es_out, long long reach[3]) {
    auto last_inside = [](int outputs, int stride, int pad, int taps, int size) {
        return std::min<long long>((long long)(outputs - 1) * stride - pad + (taps - 1), size - 1);
    };
    const long long hmax = last_inside(k.P, k.u, k.pad_h, k.R, k.H), wmax = last_inside(k.Q, k.v, k.pad_w, k.S, k.W);
    reach[0] = hmax < 0 || wmax < 0
                   ? 0
                   : ((long long)(k.N - 1) * k.xsN + (long long)(k.C - 1) * k.xsC + hmax * k.xsH + wmax * k.xsW + 1) * es_in;
    const long long tap_max = (long long)k.wTap0 + std::max<long long>(0, (long long)(k.R - 1) * k.wsTapR) +
                              std::max<long long>(0, (long long)(k.S - 1) * k.wsTapS);
    reach[1] = ((long long)(k.K - 1) * k.wsRow + (long long)(k.C - 1) * k.wsRed + tap_max + 1) * es_in;
    reach[2] = ((long long)(k.N - 1) * k.ysN + (long long)(k.K - 1) * k.ysK + (long long)(k.P - 1) * k.ysP +
                (long long)(k.Q - 1) * k.ysQ + 1) * es_out;
}

igcStatus igcSetComputeUnits(igcHandle_t handle, int computeUnits) {
    if (!handle || computeUnits < kXcds || computeUnits > 4096) return IGC_STATUS_BAD_PARAM;
    handle->computeUnits = computeUnits;
    return IGC_STATUS_SUCCESS;
}

igcStatus igcGetComputeUnits(igcHandle_t handle, int *computeUnits) {
    if (!handle || !computeUnits) return IGC_STATUS_BAD_PARAM;
    *computeUnits = handle->computeUnits;
    return IGC_STATUS_SUCCESS;
}

igcStatus igcGetConvolutionForwardAddressReach(igcHandle_t handle, igcTensorDescriptor_t xDesc, igcFilterDescriptor_t wDesc,
                                               igcConvolutionDescriptor_t convDesc, igcTensorDescriptor_t yDesc,
                                               long long reachBytes[3], long long extentBytes[3]) {
    if (!handle || !reachBytes || !extentBytes) return IGC_STATUS_BAD_PARAM;
    Problem pr;
    igcStatus st = validate(xDesc, wDesc, convDesc, yDesc, &pr);
    if (st != IGC_STATUS_SUCCESS) return st;
    int id = -1;
    st = choose(handle, pr, /*w_aligned=*/true, /*x_aligned=*/true, &id);
    if (st != IGC_STATUS_SUCCESS) return st;
    st = fill_plan(handle, id, &pr, nullptr);
    if (st != IGC_STATUS_SUCCESS) return st;
    address_reach(pr.kp, pr.bf16 ? 2 : (pr.f64 ? 8 : 4), pr.f64 ? 8 : 4, reachBytes);
    extentBytes[0] = pr.kp.x_bytes; extentBytes[1] = pr.kp.w_bytes; extentBytes[2] = pr.kp.y_bytes;
    return IGC_STATUS_SUCCESS;
}

igcStatus igcGetConvolutionBackwardDataAddressReach(igcHandle_t handle, igcFilterDescriptor_t wDesc, igcTensorDescriptor_t dyDesc,
                                                    igcConvolutionDescriptor_t convDesc, igcTensorDescriptor_t dxDesc,
                                                    long long reachBytes[3], long long extentBytes[3]) {
    if (!handle || !reachBytes || !extentBytes) return IGC_STATUS_BAD_PARAM;
    BackwardDataProblem b;
    igcStatus st = validate_backward_data(wDesc, dyDesc, convDesc, dxDesc, &b);
    if (st != IGC_STATUS_SUCCESS) return st;
    std::vector<PhaseLaunch> launches;
    st = plan_backward_data_phases(handle, b, &launches);
    if (st != IGC_STATUS_SUCCESS) return st;
    const int es = b.bf16 ? 2 : (b.f64 ? 8 : 4), out_es = b.f64 ? 8 : 4;
    for (int i = 0; i < 3; ++i) reachBytes[i] = 0;
    for (const PhaseLaunch &l : launches) {
        long long r[3];
        address_reach(l.pr.kp, es, out_es, r);
        // (a phase that meets no tap reads nothing; every phase's output offsets count from its own first element)
        if (!l.pr.zero_steps) {
            reachBytes[0] = std::max(reachBytes[0], r[0]);
            reachBytes[1] = std::max(reachBytes[1], r[1]);
        }
        reachBytes[2] = std::max(reachBytes[2], l.dx_offset * out_es + r[2]);
        if (l.dx_offset * out_es + (long long)l.pr.kp.y_bytes != b.dx_bytes) return IGC_STATUS_EXECUTION_FAILED;
    }
    extentBytes[0] = b.dy_bytes; extentBytes[1] = b.w_bytes; extentBytes[2] = b.dx_bytes;
    return IGC_STATUS_SUCCESS;
}

igcStatus igcGetConvolutionForwardPlan(igcHandle_t handle, igcTensorDescriptor_t xDesc, igcFilterDescriptor_t wDesc,
                                       igcConvolutionDescriptor_t convDesc, igcTensorDescriptor_t yDesc,
                                       igcConvolutionForwardPlan *plan) {
    if (!handle || !plan) return IGC_STATUS_BAD_PARAM;
    Problem pr;
    igcStatus st = validate(xDesc, wDesc, convDesc, yDesc, &pr);
    if (st != IGC_STATUS_SUCCESS) return st;
    int id = -1;
    st = choose(handle, pr, /*w_aligned=*/true, /*x_aligned=*/true, &id);
    if (st != IGC_STATUS_SUCCESS) return st;
    igcConvolutionForwardPlan tmp;
    st = fill_plan(handle, id, &pr, &tmp);
    if (st != IGC_STATUS_SUCCESS) return st;
    *plan = tmp;
    return IGC_STATUS_SUCCESS;
}

int igcGetKernelCount(void) { return kernel_count(); }

const char *igcGetKernelName(int kernelId) {
    const KernelInfo *ki = kernel_info(kernelId);
    return ki ? ki->name : nullptr;
}

igcStatus igcSetKernelOverride(igcHandle_t handle, int kernelId) {
    if (!handle) return IGC_STATUS_BAD_PARAM;
    if (kernelId < -1 || kernelId >= kernel_count()) return IGC_STATUS_BAD_PARAM;
    handle->kernelOverride = kernelId;
    return IGC_STATUS_SUCCESS;
}

igcStatus igcMagicDivisor(unsigned int d, unsigned int *mul, unsigned int *shift) {
    if (!mul || !shift) return IGC_STATUS_BAD_PARAM;
    Magic m;
    if (!magic_for(d, &m)) return IGC_STATUS_BAD_PARAM;
    *mul = m.mul;
    *shift = m.shift;
    return IGC_STATUS_SUCCESS;
}

unsigned int igcMagicDivide(unsigned int n, unsigned int mul, unsigned int shift) {
    const uint32_t hi = (uint32_t)(((uint64_t)n * (uint64_t)mul) >> 32);
    return (hi + n) >> shift;
}

igcStatus igcConvolutionForward(igcHandle_t handle, const void *alpha, igcTensorDescriptor_t xDesc, const void *x,
                                igcFilterDescriptor_t wDesc, const void *w, igcConvolutionDescriptor_t convDesc,
                                void *workSpace, size_t workSpaceSizeInBytes, const void *beta,
                                igcTensorDescriptor_t yDesc, void *y) {
    return igcConvolutionBiasActivationForward(handle, alpha, xDesc, x, wDesc, w, convDesc, workSpace, workSpaceSizeInBytes,
                                               beta, nullptr, IGC_ACTIVATION_IDENTITY, yDesc, y);
}

igcStatus igcConvolutionBiasActivationForward(igcHandle_t handle, const void *alpha, igcTensorDescriptor_t xDesc, const void *x,
                                              igcFilterDescriptor_t wDesc, const void *w, igcConvolutionDescriptor_t convDesc,
                                              void *workSpace, size_t workSpaceSizeInBytes, const void *beta,
                                              const void *bias, int activation, igcTensorDescriptor_t yDesc, void *y) {
    if (!handle || !alpha || !beta || !x || !w || !y) return IGC_STATUS_BAD_PARAM;
    if (activation < IGC_ACTIVATION_IDENTITY || activation > IGC_ACTIVATION_TANH || (uintptr_t)bias % 4) return IGC_STATUS_BAD_PARAM;
    Problem pr;
    igcStatus st = validate(xDesc, wDesc, convDesc, yDesc, &pr);
    if (st != IGC_STATUS_SUCCESS) return st;
    const int es = pr.bf16 ? 2 : (pr.f64 ? 8 : 4);
    if ((uintptr_t)x % es || (uintptr_t)w % es || (uintptr_t)y % (pr.f64 ? 8 : 4)) return IGC_STATUS_BAD_PARAM;
    if (pr.f64 && (bias || activation != IGC_ACTIVATION_IDENTITY)) return IGC_STATUS_NOT_SUPPORTED;
    int id = -1;
    igcConvolutionForwardPlan plan;
    // With a workspace the reduction of a small problem is cut into ranges (below), finer than the team kernels
    // cut it: those are left out of the choice then, unless the cut does not pay for the kernel chosen instead.
    const bool can_cut = workSpace && (uintptr_t)workSpace % 4 == 0 && !bias && activation == IGC_ACTIVATION_IDENTITY && !pr.f64;
    bool cut_found = false;
    if (can_cut) {
        Problem trial = pr;
        trial.no_teams = true;
        int tid_ = -1, per_ = 0;
        if (choose(handle, trial, ((uintptr_t)w % 16) == 0, ((uintptr_t)x % 16) == 0, &tid_) == IGC_STATUS_SUCCESS &&
            fill_plan(handle, tid_, &trial, &plan) == IGC_STATUS_SUCCESS) {
            const bool packed = extent(yDesc->dim, yDesc->stride) == (long long)trial.kp.K * trial.kp.NPQ;
            if (forward_split(handle, *kernel_info(tid_), trial.kp, packed, (long long)(workSpaceSizeInBytes / trial.kp.y_bytes), &per_) > 1) {
                pr = trial;
                id = tid_;
                cut_found = true;
            }
        }
    }
    if (!cut_found) {
        st = choose(handle, pr, /*w_aligned=*/((uintptr_t)w % 16) == 0, /*x_aligned=*/((uintptr_t)x % 16) == 0, &id);
        if (st != IGC_STATUS_SUCCESS) return st;
        st = fill_plan(handle, id, &pr, &plan);
        if (st != IGC_STATUS_SUCCESS) return st;
    }
    pr.kp.x = x;
    pr.kp.w = w;
    pr.kp.y = y;
    if (pr.f64) {
        pr.kp.alpha64 = *static_cast<const double *>(alpha);
        pr.kp.beta64 = *static_cast<const double *>(beta);
    } else {
        pr.kp.alpha = *static_cast<const float *>(alpha);
        pr.kp.beta = *static_cast<const float *>(beta);
    }
    pr.kp.bias = static_cast<const float *>(bias);
    pr.kp.act = activation;
    // A small problem with a workspace: cut the reduction into ranges (see forward_split).
    int grid = plan.gridX;
    int splits = 1;
    if (can_cut) {
        ConvKernelParams &k = pr.kp;
        const bool packed = extent(yDesc->dim, yDesc->stride) == (long long)k.K * k.NPQ;
        int per;
        splits = forward_split(handle, *kernel_info(id), k, packed, (long long)(workSpaceSizeInBytes / k.y_bytes), &per);
        if (splits > 1) {
            k.splits = splits;
            k.stepsPerSplit = per;
            k.ySplitBytes = k.y_bytes;
            k.tilesPerXcd = (int)(((long long)k.tilesM * k.tilesN * splits + kXcds - 1) / kXcds);
            k.wgsPerXcd = workgroups_per_xcd(handle, *kernel_info(id), k.tilesPerXcd);
            grid = kXcds * k.wgsPerXcd;
            k.y = workSpace;
            k.alpha = 1.f;
            k.beta = 0.f;
        }
    }
    // Few channels, a zero border and room for x with the border written out: the copy is made and the pass runs
    // over it as a problem without a border (alpha, beta, bias and activation unchanged).
    {
        const long long pb = splits <= 1 ? padded_copy_bytes(*kernel_info(id), pr, xDesc) : 0;
        if (pb > 0 && handle->kernelOverride < 0 && workSpace && (uintptr_t)workSpace % 16 == 0 && workSpaceSizeInBytes >= (size_t)pb) {
            const ConvKernelParams &k = pr.kp;
            igcTensorStruct xd;
            igcConvolutionStruct cd;
            xd.set = true; xd.dtype = IGC_DATA_FLOAT;
            xd.dim[0] = k.N; xd.dim[1] = k.C; xd.dim[2] = k.H + 2 * k.pad_h; xd.dim[3] = k.W + 2 * k.pad_w;
            xd.stride[3] = 1; xd.stride[2] = xd.dim[3]; xd.stride[1] = (long long)xd.dim[2] * xd.dim[3]; xd.stride[0] = xd.stride[1] * k.C;
            cd.set = true; cd.pad_h = 0; cd.pad_w = 0; cd.u = k.u; cd.v = k.v; cd.mode = convDesc->mode;
            Magic mWp, mHp, mC;
            if (magic_for((uint32_t)xd.dim[3], &mWp) && magic_for((uint32_t)xd.dim[2], &mHp) && magic_for((uint32_t)k.C, &mC)) {
                if (launch_pad_image(static_cast<const float *>(x), static_cast<float *>(workSpace), k.N, k.C, k.H, k.W, k.pad_h, k.pad_w,
                                     xDesc->stride, mWp, mHp, mC, handle->stream) != 0)
                    return IGC_STATUS_EXECUTION_FAILED;
                igcContext inner = *handle;   // (same stream and device; the caller's handle is not touched)
                inner.kernelOverride = -1;
                st = igcConvolutionBiasActivationForward(&inner, alpha, &xd, workSpace, wDesc, w, &cd, nullptr, 0, beta, bias, activation,
                                                         yDesc, y);
                // (a refusal comes from the checks before any launch on y: the pass below still runs as planned)
                if (st != IGC_STATUS_NOT_SUPPORTED) return st;
            }
        }
    }
    // Tap-major order with a lent workspace of the filter's size: the filter is first rewritten with the channel
    // index innermost (wt[k][t][c]) and read through those strides - a step's filter elements are then contiguous
    // instead of R*S apart (a 5x5 layer with 96 channels: 74 -> 129 TFLOP/s).  Same sums in the same order.
    if (splits <= 1 && kernel_info(id)->gmode == 1 && !pr.f64 && pr.kp.RS > 1 && workSpace &&
        (uintptr_t)workSpace % 16 == 0 && workSpaceSizeInBytes >= (size_t)pr.kp.w_bytes) {
        ConvKernelParams &k = pr.kp;
        Magic mC, mRS;
        if (magic_for((uint32_t)k.C, &mC) && magic_for((uint32_t)k.RS, &mRS)) {
            if (launch_filter_taps_outer(w, workSpace, pr.bf16 ? 2 : 4, k.K, k.C, k.RS, false, mC, mRS, handle->stream) != 0)
                return IGC_STATUS_EXECUTION_FAILED;
            k.w = workSpace;
            k.wsRow = k.CRS; k.wsRed = 1; k.wTap0 = 0; k.wsTapR = k.S * k.C; k.wsTapS = k.C;
        }
    }
    if (kernel_info(id)->launch(pr.kp, grid, handle->stream) != 0) return IGC_STATUS_EXECUTION_FAILED;
    if (splits > 1 && launch_sum_parts(static_cast<const float *>(workSpace), static_cast<float *>(y), pr.kp.y_bytes / 4, splits,
                                       pr.kp.y_bytes / 4, *static_cast<const float *>(alpha),
                                       *static_cast<const float *>(beta), handle->stream) != 0)
        return IGC_STATUS_EXECUTION_FAILED;
    return IGC_STATUS_SUCCESS;
}

igcStatus igcGetConvolutionBackwardDataWorkspaceSize(igcHandle_t handle, igcFilterDescriptor_t wDesc,
                                                     igcTensorDescriptor_t dyDesc, igcConvolutionDescriptor_t convDesc,
                                                     igcTensorDescriptor_t dxDesc, size_t *sizeInBytes) {
    if (!handle || !sizeInBytes) return IGC_STATUS_BAD_PARAM;
    BackwardDataProblem b;
    const igcStatus st = validate_backward_data(wDesc, dyDesc, convDesc, dxDesc, &b);
    if (st != IGC_STATUS_SUCCESS) return st;
    Problem pr;
    PackedPhases pp;
    *sizeInBytes = backward_data_as_forward(b, &pr) ? (size_t)b.w_bytes : (packed_phases(b, &pp) ? (size_t)pp.bytes : 0);
    if (*sizeInBytes == 0) {
        std::vector<PhaseLaunch> launches;
        if (plan_backward_data_phases(handle, b, &launches) == IGC_STATUS_SUCCESS && phases_want_filter_workspace(b, launches))
            *sizeInBytes = (size_t)b.w_bytes;
    }
    return IGC_STATUS_SUCCESS;
}

igcStatus igcConvolutionBackwardData(igcHandle_t handle, const void *alpha, igcFilterDescriptor_t wDesc, const void *w,
                                     igcTensorDescriptor_t dyDesc, const void *dy, igcConvolutionDescriptor_t convDesc,
                                     void *workSpace, size_t workSpaceSizeInBytes, const void *beta,
                                     igcTensorDescriptor_t dxDesc, void *dx) {
    if (!handle || !alpha || !beta || !w || !dy || !dx) return IGC_STATUS_BAD_PARAM;
    BackwardDataProblem b;
    igcStatus st = validate_backward_data(wDesc, dyDesc, convDesc, dxDesc, &b);
    if (st != IGC_STATUS_SUCCESS) return st;
    const int es = b.bf16 ? 2 : (b.f64 ? 8 : 4);
    if ((uintptr_t)dy % es || (uintptr_t)w % es || (uintptr_t)dx % (b.f64 ? 8 : 4)) return IGC_STATUS_BAD_PARAM;
    // The forward pass over dy with the exchanged filter, when the shape allows and the caller
    // lends room for that filter; else the general route below.
    {
        Problem pr;
        int id = -1;
        if (workSpace && (uintptr_t)workSpace % 16 == 0 && backward_data_as_forward(b, &pr) &&
            workSpaceSizeInBytes >= (size_t)b.w_bytes &&
            choose(handle, pr, /*w_aligned=*/true, /*x_aligned=*/((uintptr_t)dy % 16) == 0, &id) == IGC_STATUS_SUCCESS) {
            igcConvolutionForwardPlan plan;
            st = fill_plan(handle, id, &pr, &plan);
            if (st != IGC_STATUS_SUCCESS) return st;
            pr.kp.x = dy;
            pr.kp.w = workSpace;
            pr.kp.y = dx;
            pr.kp.alpha = *static_cast<const float *>(alpha);
            pr.kp.beta = *static_cast<const float *>(beta);
            if (getenv("IGCONV_DEBUG")) fprintf(stderr, "igconv: backward data as a forward pass, kernel %s\n", kernel_info(id)->name);
            if (launch_filter_exchange(w, workSpace, b.K, b.C, b.R * b.S, handle->stream) != 0) return IGC_STATUS_EXECUTION_FAILED;
            if (kernel_info(id)->launch(pr.kp, plan.gridX, handle->stream) != 0) return IGC_STATUS_EXECUTION_FAILED;
            return IGC_STATUS_SUCCESS;
        }
    }
    // A strided layer with few channels and room for the packed filter and result: one forward pass over dy
    // for all phases together, then the move of its result to dx.
    PackedPhases pp;
    if (workSpace && (uintptr_t)workSpace % 16 == 0 && packed_phases(b, &pp) && workSpaceSizeInBytes >= (size_t)pp.bytes) {
        float *const fpack = static_cast<float *>(workSpace);
        float *const ypack = reinterpret_cast<float *>(static_cast<char *>(workSpace) + pp.filter_bytes);
        igcTensorStruct xd, yd;
        igcFilterStruct fd;
        igcConvolutionStruct cd;
        xd.set = true; xd.dtype = IGC_DATA_FLOAT;
        for (int d = 0; d < 4; ++d) { xd.dim[d] = dyDesc->dim[d]; xd.stride[d] = dyDesc->stride[d]; }
        fd.set = true; fd.dtype = IGC_DATA_FLOAT; fd.k = pp.maps; fd.c = b.K; fd.r = pp.Rp; fd.s = pp.Sp;
        cd.set = true; cd.pad_h = pp.Rp - 1; cd.pad_w = pp.Sp - 1; cd.u = 1; cd.v = 1; cd.mode = IGC_CROSS_CORRELATION;
        yd.set = true; yd.dtype = IGC_DATA_FLOAT;
        yd.dim[0] = b.N; yd.dim[1] = pp.maps; yd.dim[2] = pp.I; yd.dim[3] = pp.J;
        yd.stride[3] = 1; yd.stride[2] = pp.J; yd.stride[1] = (long long)pp.I * pp.J; yd.stride[0] = yd.stride[1] * pp.maps;
        Magic mSp, mRp, mK, mC, mv, mu, mW, mH;
        if (!magic_for((uint32_t)pp.Sp, &mSp) || !magic_for((uint32_t)pp.Rp, &mRp) || !magic_for((uint32_t)b.K, &mK) ||
            !magic_for((uint32_t)b.C, &mC) || !magic_for((uint32_t)b.v, &mv) || !magic_for((uint32_t)b.u, &mu) ||
            !magic_for((uint32_t)b.W, &mW) || !magic_for((uint32_t)b.H, &mH))
            goto per_phase;
        if (getenv("IGCONV_DEBUG"))
            fprintf(stderr, "igconv: backward data of %d phases as one forward pass with %d maps, %dx%d taps\n", b.u * b.v, pp.maps, pp.Rp, pp.Sp);
        if (launch_pack_phase_filter(static_cast<const float *>(w), fpack, b.K, b.C, b.R, b.S, b.u, b.v, pp.Rp, pp.Sp, b.flip, mSp, mRp,
                                     mK, mC, mv, handle->stream) != 0)
            return IGC_STATUS_EXECUTION_FAILED;
        const float one = 1.f, zero = 0.f;
        igcContext inner = *handle;   // (same stream and device; an override names a kernel for the caller's problem, not for this one)
        inner.kernelOverride = -1;
        st = igcConvolutionBiasActivationForward(&inner, &one, &xd, dy, &fd, fpack, &cd, nullptr, 0, &zero, nullptr,
                                                 IGC_ACTIVATION_IDENTITY, &yd, ypack);
        // (a refusal comes from the checks before any launch: nothing of dx is written yet, the phases run one by one)
        if (st == IGC_STATUS_NOT_SUPPORTED) goto per_phase;
        if (st != IGC_STATUS_SUCCESS) return st;
        if (launch_phase_scatter(ypack, static_cast<float *>(dx), b.N, b.C, b.H, b.W, pp.I, pp.J, b.u, b.v, b.pad_h, b.pad_w, b.dxs,
                                 mW, mH, mC, mu, mv, *static_cast<const float *>(alpha), *static_cast<const float *>(beta),
                                 handle->stream) != 0)
            return IGC_STATUS_EXECUTION_FAILED;
        return IGC_STATUS_SUCCESS;
    }
per_phase:
    // plan every phase before the first launch, so that a rejected problem launches nothing
    std::vector<PhaseLaunch> launches;
    st = plan_backward_data_phases(handle, b, &launches);
    if (st != IGC_STATUS_SUCCESS) return st;
    for (PhaseLaunch &l : launches) {
        l.pr.kp.x = dy;
        l.pr.kp.w = w;
        if (b.f64) {
            l.pr.kp.y = static_cast<double *>(dx) + l.dx_offset;
            l.pr.kp.alpha64 = *static_cast<const double *>(alpha);
            l.pr.kp.beta64 = *static_cast<const double *>(beta);
        } else {
            l.pr.kp.y = static_cast<float *>(dx) + l.dx_offset;
            l.pr.kp.alpha = *static_cast<const float *>(alpha);
            l.pr.kp.beta = *static_cast<const float *>(beta);
        }
    }
    // Float phases that all run in tap-major order, and room for the filter: it is first rewritten as wt[c][t][k]
    // (reduction index innermost) and read through those strides - a step's filter elements are then contiguous
    // instead of C*R*S apart.  Same sums in the same order as without.
    if (phases_want_filter_workspace(b, launches) && workSpace && (uintptr_t)workSpace % 16 == 0 && workSpaceSizeInBytes >= (size_t)b.w_bytes) {
        Magic mK, mRS;
        if (magic_for((uint32_t)b.K, &mK) && magic_for((uint32_t)(b.R * b.S), &mRS)) {
            if (launch_filter_taps_outer(w, workSpace, b.bf16 ? 2 : 4, b.K, b.C, b.R * b.S, true, mK, mRS, handle->stream) != 0)
                return IGC_STATUS_EXECUTION_FAILED;
            for (PhaseLaunch &l : launches) {
                ConvKernelParams &k = l.pr.kp;
                k.w = workSpace;
                k.wsRow = b.R * b.S * b.K;
                k.wsRed = 1;
                k.wTap0 *= b.K; k.wsTapR *= b.K; k.wsTapS *= b.K;
            }
        }
    }
    for (const PhaseLaunch &l : launches)
        if (kernel_info(l.id)->launch(l.pr.kp, l.grid, handle->stream) != 0) return IGC_STATUS_EXECUTION_FAILED;
    return IGC_STATUS_SUCCESS;
}

igcStatus igcGetConvolutionBackwardFilterWorkspaceSize(igcHandle_t handle, igcTensorDescriptor_t xDesc,
                                                       igcTensorDescriptor_t dyDesc, igcConvolutionDescriptor_t convDesc,
                                                       igcFilterDescriptor_t dwDesc, size_t *sizeInBytes) {
    if (!handle || !sizeInBytes) return IGC_STATUS_BAD_PARAM;
    BackwardFilterProblem b;
    const igcStatus st = validate_backward_filter(xDesc, dyDesc, convDesc, dwDesc, &b);
    if (st != IGC_STATUS_SUCCESS) return st;
    int splits, per;
    backward_filter_split(handle, b, 1 << 20, &splits, &per);
    // (the channel-vector kernels want their workspace even for a single range: see the entry point)
    *sizeInBytes = splits > 1 || b.pos_rows ? (size_t)splits * b.part_elems() * (b.pr.f64 ? 8 : 4) : 0;
    return IGC_STATUS_SUCCESS;
}

igcStatus igcConvolutionBackwardFilter(igcHandle_t handle, const void *alpha, igcTensorDescriptor_t xDesc, const void *x,
                                       igcTensorDescriptor_t dyDesc, const void *dy, igcConvolutionDescriptor_t convDesc,
                                       void *workSpace, size_t workSpaceSizeInBytes, const void *beta,
                                       igcFilterDescriptor_t dwDesc, void *dw) {
    if (!handle || !alpha || !beta || !x || !dy || !dw) return IGC_STATUS_BAD_PARAM;
    BackwardFilterProblem b;
    igcStatus st = validate_backward_filter(xDesc, dyDesc, convDesc, dwDesc, &b, (uintptr_t)x % 16 == 0 && (uintptr_t)dy % 16 == 0);
    if (st != IGC_STATUS_SUCCESS) return st;
    const bool f64 = b.pr.f64;
    const int es = b.pr.bf16 ? 2 : (f64 ? 8 : 4), out_es = f64 ? 8 : 4;
    if ((uintptr_t)x % es || (uintptr_t)dy % es || (uintptr_t)dw % out_es || (uintptr_t)workSpace % out_es) return IGC_STATUS_BAD_PARAM;
    const size_t part_bytes = (size_t)b.part_elems() * out_es;
    int splits, per;
    const long long room = workSpace ? (long long)(workSpaceSizeInBytes / part_bytes) : 0;
    backward_filter_split(handle, b, room, &splits, &per);
    // Channel-vector kernels: with room for at least one part the results go to the workspace in accumulator
    // order (coalesced) and the summing kernel moves them to dw; writing dw's layout from the tile is slow.
    const bool positions = b.pos_rows != 0 && room >= 1;
    ConvKernelParams &k = b.pr.kp;
    igcConvolutionForwardPlan plan;
    st = fill_plan(handle, b.kernel_id, &b.pr, &plan);
    if (st != IGC_STATUS_SUCCESS) return st;
    k.tilesN = (int)b.tiles_n;
    const float a = f64 ? 0.f : *static_cast<const float *>(alpha), bt = f64 ? 0.f : *static_cast<const float *>(beta);
    const double a64 = f64 ? *static_cast<const double *>(alpha) : 0.0, bt64 = f64 ? *static_cast<const double *>(beta) : 0.0;
    k.x = x;
    k.w = dy;
    k.splits = splits;
    k.stepsPerSplit = splits > 1 ? per : (int)(b.ksteps + (b.ksteps & 1));
    k.ySplitBytes = (uint32_t)part_bytes;
    k.tilesPerXcd = (int)((b.tiles * splits + kXcds - 1) / kXcds);
    if ((long long)k.tilesPerXcd * kXcds >= (1ll << 24)) return IGC_STATUS_NOT_SUPPORTED;
    k.wgsPerXcd = workgroups_per_xcd(handle, *kernel_info(b.kernel_id), k.tilesPerXcd);
    if (splits > 1 || positions) {
        k.y = workSpace;
        k.alpha = 1.f; k.alpha64 = 1.0;
        k.beta = 0.f; k.beta64 = 0.0;
        if (positions) {
            k.ysN = 1; k.ysP = (int)b.pos_rows; k.ysK = (int)b.pos_cols;
            k.y_bytes = (uint32_t)part_bytes;
        }
    } else {
        k.y = dw;
        k.alpha = a; k.alpha64 = a64;
        k.beta = bt; k.beta64 = bt64;
    }
    if (getenv("IGCONV_DEBUG"))
        fprintf(stderr, "igconv: backward filter with '%s', %lld tiles x %d ranges of %d steps\n", kernel_info(b.kernel_id)->name,
                b.tiles, splits, k.stepsPerSplit);
    if (kernel_info(b.kernel_id)->launch(k, kXcds * k.wgsPerXcd, handle->stream) != 0) return IGC_STATUS_EXECUTION_FAILED;
    if (splits > 1 && f64 &&
        launch_sum_parts_f64(static_cast<const double *>(workSpace), static_cast<double *>(dw), b.out_elems, splits, b.out_elems,
                             a64, bt64, handle->stream) != 0)
        return IGC_STATUS_EXECUTION_FAILED;
    if (positions) {
        const KernelInfo &ki = *kernel_info(b.kernel_id);
        const int RS = (int)(b.out_elems / ((long long)k.K * k.NPQ));
        if (launch_sum_positions(static_cast<const float *>(workSpace), static_cast<float *>(dw), b.out_elems, splits,
                                 (uint32_t)b.part_elems(), a, bt, k.NPQ, RS, ki.BM, ki.BN, (int)b.pos_rows, (int)b.pos_cols,
                                 handle->stream) != 0)
            return IGC_STATUS_EXECUTION_FAILED;
        return IGC_STATUS_SUCCESS;
    }
    if (splits > 1 && !f64 && launch_sum_parts(static_cast<const float *>(workSpace), static_cast<float *>(dw), b.out_elems, splits,
                                               b.out_elems, a, bt, handle->stream) != 0)
        return IGC_STATUS_EXECUTION_FAILED;
    return IGC_STATUS_SUCCESS;
}

}  // extern "C"
