// Host-side descriptor objects behind the opaque handles of include/igconv.h, and small
// helpers shared by the translation units that implement entry points.  Internal.
#ifndef IGCONV_DESC_H_
#define IGCONV_DESC_H_

#include <algorithm>

#include "../../include/igconv.h"

struct igcContext {
    void *stream = nullptr;
    int kernelOverride = -1;
    int computeUnits = 256;   // of the device current when the handle was created (MI355X's 256 when there is none)
};

struct igcTensorStruct {
    bool set = false;
    igcDataType dtype = IGC_DATA_FLOAT;
    int dim[4] = {0, 0, 0, 0};           // n, c, h, w
    long long stride[4] = {0, 0, 0, 0};  // elements
};

struct igcFilterStruct {
    bool set = false;
    igcDataType dtype = IGC_DATA_FLOAT;
    int k = 0, c = 0, r = 0, s = 0;
};

struct igcConvolutionStruct {
    bool set = false;
    int pad_h = 0, pad_w = 0, u = 1, v = 1;
    igcConvolutionMode mode = IGC_CROSS_CORRELATION;
};

struct igcPoolingStruct {
    bool set = false;
    igcPoolingMode mode = IGC_POOLING_MAX;
    int win_h = 1, win_w = 1, pad_h = 0, pad_w = 0, u = 1, v = 1;
};

namespace igc {

inline int elem_size(igcDataType t) { return t == IGC_DATA_BFLOAT16 ? 2 : (t == IGC_DATA_DOUBLE ? 8 : 4); }

// Elements spanned by a strided 4-D tensor: 1 + sum (dim-1)*stride.
inline long long extent(const int dim[4], const long long stride[4]) {
    long long e = 1;
    for (int i = 0; i < 4; ++i) e += (long long)(dim[i] - 1) * stride[i];
    return e;
}

// True when every index tuple lands on its own element.  Sufficient test: with the
// dimensions of size > 1 sorted by stride, each stride must step over everything
// the smaller-stride dimensions span.
inline bool non_aliasing(const int dim[4], const long long stride[4]) {
    int idx[4], n = 0;
    for (int i = 0; i < 4; ++i)
        if (dim[i] > 1) idx[n++] = i;
    std::sort(idx, idx + n, [&](int a, int b) { return stride[a] < stride[b]; });
    long long span = 1;  // elements covered so far
    for (int t = 0; t < n; ++t) {
        const int i = idx[t];
        if (stride[i] < span) return false;
        span += (long long)(dim[i] - 1) * stride[i];
    }
    return true;
}

}  // namespace igc
#endif
