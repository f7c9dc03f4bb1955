// Driver for a build of the library's host tier (igconv_api.cpp: descriptors, validation, kernel choice, launch
// plans, workspace sizes, the address-reach check) under AddressSanitizer and UndefinedBehaviorSanitizer.  Runs
// without a GPU: it calls only entry points that end before the first launch - queries over a few thousand random
// layers in all three data types and both layouts, and every pass with null data pointers or contradictory
// descriptors, which must be refused.  A sanitizer report aborts the run; a wrong status code or a reach beyond an
// extent fails it.  Prints "host check ok".
#include <cstdio>
#include <cstdlib>
#include <initializer_list>

#include "../../include/igconv.h"

static unsigned long long state = 14100759ull;
static int draw(int lo, int hi) {   // uniform in lo..hi
    state = state * 6364136223846793005ull + 1442695040888963407ull;
    return (int)(lo + (long long)((state >> 33) % (unsigned long long)((long long)hi - lo + 1)));
}

#define REQUIRE(cond)                                                                  \
    do {                                                                               \
        if (!(cond)) {                                                                 \
            std::fprintf(stderr, "host check failed at line %d: %s (case %d)\n", __LINE__, #cond, it); \
            return 1;                                                                  \
        }                                                                              \
    } while (0)

int main() {
    igcHandle_t h = nullptr;
    int it = -1;
    REQUIRE(igcCreate(&h) == IGC_STATUS_SUCCESS);
    igcTensorDescriptor_t x, y, dx;
    igcFilterDescriptor_t w;
    igcConvolutionDescriptor_t c;
    REQUIRE(igcCreateTensorDescriptor(&x) == IGC_STATUS_SUCCESS && igcCreateTensorDescriptor(&y) == IGC_STATUS_SUCCESS &&
            igcCreateTensorDescriptor(&dx) == IGC_STATUS_SUCCESS && igcCreateFilterDescriptor(&w) == IGC_STATUS_SUCCESS &&
            igcCreateConvolutionDescriptor(&c) == IGC_STATUS_SUCCESS);
    const igcDataType types[3] = {IGC_DATA_FLOAT, IGC_DATA_BFLOAT16, IGC_DATA_DOUBLE};
    long long plans = 0;
    for (it = 0; it < 3000; ++it) {
        const bool big = it % 50 == 0;   // now and then a layer of realistic size
        const int N = big ? draw(16, 256) : draw(1, 5), C = big ? draw(3, 512) : draw(1, 70), K = big ? draw(16, 512) : draw(1, 200);
        const int R = draw(1, 11), S = draw(1, 11);
        const int pad_h = draw(0, R - 1), pad_w = draw(0, S - 1), u = draw(1, 4), v = draw(1, 4);
        const int H = draw(R > 2 * pad_h ? R - 2 * pad_h : 1, big ? 230 : 40), W = draw(S > 2 * pad_w ? S - 2 * pad_w : 1, big ? 230 : 40);
        const igcDataType dt = types[it % 3], odt = dt == IGC_DATA_DOUBLE ? IGC_DATA_DOUBLE : IGC_DATA_FLOAT;
        const bool nhwc = (it / 3) % 2 == 1;
        if (it % 97 == 0) REQUIRE(igcSetComputeUnits(h, draw(8, 400)) == IGC_STATUS_SUCCESS);
        REQUIRE(igcSetTensor4dDescriptor(x, dt, N, C, H, W, nhwc ? (long long)H * W * C : (long long)C * H * W, nhwc ? 1 : (long long)H * W,
                                         nhwc ? (long long)W * C : W, nhwc ? C : 1) == IGC_STATUS_SUCCESS);
        REQUIRE(igcSetTensor4dDescriptor(dx, odt, N, C, H, W, nhwc ? (long long)H * W * C : (long long)C * H * W, nhwc ? 1 : (long long)H * W,
                                         nhwc ? (long long)W * C : W, nhwc ? C : 1) == IGC_STATUS_SUCCESS);
        REQUIRE(igcSetFilter4dDescriptor(w, dt, K, C, R, S) == IGC_STATUS_SUCCESS);
        REQUIRE(igcSetConvolution2dDescriptor(c, pad_h, pad_w, u, v, it % 2 ? IGC_CONVOLUTION : IGC_CROSS_CORRELATION) == IGC_STATUS_SUCCESS);
        int n, k, p, q;
        REQUIRE(igcGetConvolution2dForwardOutputDim(c, x, w, &n, &k, &p, &q) == IGC_STATUS_SUCCESS);
        REQUIRE(n == N && k == K && p >= 1 && q >= 1);
        REQUIRE(igcSetTensor4dDescriptor(y, odt, n, k, p, q, nhwc ? (long long)p * q * k : (long long)k * p * q, nhwc ? 1 : (long long)p * q,
                                         nhwc ? (long long)q * k : q, nhwc ? k : 1) == IGC_STATUS_SUCCESS);
        igcConvolutionForwardPlan plan;
        const igcStatus st = igcGetConvolutionForwardPlan(h, x, w, c, y, &plan);
        REQUIRE(st == IGC_STATUS_SUCCESS || st == IGC_STATUS_NOT_SUPPORTED);
        if (st != IGC_STATUS_SUCCESS) continue;   // (extents of 2 GiB and more)
        ++plans;
        REQUIRE(plan.kernelId >= 0 && plan.kernelId < igcGetKernelCount() && igcGetKernelName(plan.kernelId) != nullptr);
        REQUIRE(plan.gridX >= 8 && plan.gridX % 8 == 0 && plan.threads % 64 == 0 && plan.ldsBytes <= 160 * 1024);
        size_t ws = 1, opt = 0;
        REQUIRE(igcGetConvolutionForwardWorkspaceSize(h, x, w, c, y, &ws) == IGC_STATUS_SUCCESS && ws == 0);
        REQUIRE(igcGetConvolutionForwardOptionalWorkspaceSize(h, x, w, c, y, &opt) == IGC_STATUS_SUCCESS);
        long long reach[3], extent[3];
        REQUIRE(igcGetConvolutionForwardAddressReach(h, x, w, c, y, reach, extent) == IGC_STATUS_SUCCESS);
        for (int i = 0; i < 3; ++i) REQUIRE(reach[i] > 0 && reach[i] <= extent[i] && extent[i] < (1ll << 31));
        // backward data and backward filter of the same layer (dy takes the inputs' type, dx / dw the output rule)
        igcTensorDescriptor_t dy = y;
        if (dt == IGC_DATA_BFLOAT16) {
            REQUIRE(igcCreateTensorDescriptor(&dy) == IGC_STATUS_SUCCESS);
            REQUIRE(igcSetTensor4dDescriptor(dy, dt, n, k, p, q, nhwc ? (long long)p * q * k : (long long)k * p * q, nhwc ? 1 : (long long)p * q,
                                             nhwc ? (long long)q * k : q, nhwc ? k : 1) == IGC_STATUS_SUCCESS);
        }
        size_t bd = 0, bf = 0;
        // (a float dx for bfloat16 inputs is twice the size of x: it may pass 2 GiB where x did not)
        const igcStatus sbd = igcGetConvolutionBackwardDataWorkspaceSize(h, w, dy, c, dx, &bd);
        REQUIRE(sbd == IGC_STATUS_SUCCESS || (sbd == IGC_STATUS_NOT_SUPPORTED && dt == IGC_DATA_BFLOAT16));
        if (sbd == IGC_STATUS_SUCCESS) {
            REQUIRE(igcGetConvolutionBackwardDataAddressReach(h, w, dy, c, dx, reach, extent) == IGC_STATUS_SUCCESS);
            for (int i = 0; i < 3; ++i) REQUIRE(reach[i] > 0 && reach[i] <= extent[i] && extent[i] < (1ll << 31));
        }
        igcFilterDescriptor_t dw = w;
        if (dt == IGC_DATA_BFLOAT16) {
            REQUIRE(igcCreateFilterDescriptor(&dw) == IGC_STATUS_SUCCESS);
            REQUIRE(igcSetFilter4dDescriptor(dw, IGC_DATA_FLOAT, K, C, R, S) == IGC_STATUS_SUCCESS);
        }
        const igcStatus sbf = igcGetConvolutionBackwardFilterWorkspaceSize(h, x, dy, c, dw, &bf);
        REQUIRE(sbf == IGC_STATUS_SUCCESS || (sbf == IGC_STATUS_NOT_SUPPORTED && dt == IGC_DATA_BFLOAT16));
        // every pass refuses null data pointers before anything else happens
        const float one = 1.f, zero = 0.f;
        const double one64 = 1.0, zero64 = 0.0;
        const void *al = dt == IGC_DATA_DOUBLE ? (const void *)&one64 : (const void *)&one;
        const void *be = dt == IGC_DATA_DOUBLE ? (const void *)&zero64 : (const void *)&zero;
        REQUIRE(igcConvolutionForward(h, al, x, nullptr, w, nullptr, c, nullptr, 0, be, y, nullptr) == IGC_STATUS_BAD_PARAM);
        REQUIRE(igcConvolutionBackwardData(h, al, w, nullptr, dy, nullptr, c, nullptr, 0, be, dx, nullptr) == IGC_STATUS_BAD_PARAM);
        REQUIRE(igcConvolutionBackwardFilter(h, al, x, nullptr, dy, nullptr, c, nullptr, 0, be, dw, nullptr) == IGC_STATUS_BAD_PARAM);
        // a y of the wrong size is refused by every query
        if (p > 1) {
            REQUIRE(igcSetTensor4dDescriptor(y, odt, n, k, p - 1, q, (long long)k * (p - 1) * q, (long long)(p - 1) * q, q, 1) == IGC_STATUS_SUCCESS);
            REQUIRE(igcGetConvolutionForwardPlan(h, x, w, c, y, &plan) == IGC_STATUS_BAD_PARAM);
        }
        if (dy != y) REQUIRE(igcDestroyTensorDescriptor(dy) == IGC_STATUS_SUCCESS);
        if (dw != w) REQUIRE(igcDestroyFilterDescriptor(dw) == IGC_STATUS_SUCCESS);
    }
    it = -2;
    REQUIRE(plans > 2500);
    // the division by multiply and shift, over divisors and numerators up to 2^31 - 1
    for (it = 0; it < 200000; ++it) {
        const unsigned d = (unsigned)draw(1, it % 2 ? 1 << 16 : 0x7fffffff), nn = (unsigned)draw(0, 0x7fffffff);
        unsigned mul = 0, shift = 0;
        REQUIRE(igcMagicDivisor(d, &mul, &shift) == IGC_STATUS_SUCCESS);
        REQUIRE(igcMagicDivide(nn, mul, shift) == nn / d);
    }
    it = -3;
    REQUIRE(igcDestroyTensorDescriptor(x) == IGC_STATUS_SUCCESS && igcDestroyTensorDescriptor(y) == IGC_STATUS_SUCCESS &&
            igcDestroyTensorDescriptor(dx) == IGC_STATUS_SUCCESS && igcDestroyFilterDescriptor(w) == IGC_STATUS_SUCCESS &&
            igcDestroyConvolutionDescriptor(c) == IGC_STATUS_SUCCESS && igcDestroy(h) == IGC_STATUS_SUCCESS);
    std::printf("host check ok (%lld plans)\n", plans);
    return 0;
}
