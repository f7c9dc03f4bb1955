/*
 * CPU oracle for the library's other functions (paper, Section 2.2 "Other functions"):
 * the three neuron activations (sigmoid, rectified linear, hyperbolic tangent), forward
 * and backward; softmax, computed the numerically stable way (every element shifted by
 * the maximum before exponentiation), per image over (feature map, height, width) or per
 * spatial location over the feature maps; max and average pooling; the addition of
 * tensors with optional broadcasting; and the gradient with respect to a bias added that
 * way (Section 4).  TEST INFRASTRUCTURE ONLY: used by the tests, the
 * smoke check and the bench's baseline leg; the HIP library never calls it and shares no
 * code with it.
 *
 * Each function is the plain definition, element by element, in double precision, and exists
 * for float inputs (pointwise_oracle_<f>) and for double inputs (pointwise_oracle_f64_<f>; paper,
 * Section 2: every routine in single and double precision);
 * tensors are logical (N,C,H,W) arrays addressed through four element strides; results
 * are blended as out = alpha * value + beta * old (Section 2.1.1's accumulate form).
 * Nothing is tiled, fused or reordered.
 */
#include <math.h>
#include <stddef.h>

enum { ACT_SIGMOID = 0, ACT_RELU = 1, ACT_TANH = 2 };
enum { SOFTMAX_INSTANCE = 0, SOFTMAX_CHANNEL = 1 };
enum { POOL_MAX = 0, POOL_AVERAGE = 1 };

static long long at(const long long *s, int n, int c, int h, int w)
{
    return n * s[0] + c * s[1] + h * s[2] + w * s[3];
}

static double act_value(int mode, double x)
{
    if (mode == ACT_SIGMOID) return 1.0 / (1.0 + exp(-x));
    if (mode == ACT_RELU) return x > 0.0 ? x : 0.0;
    return tanh(x);
}

#define IN_T float
#define NAME(f) pointwise_oracle_##f
#include "pointwise_oracle_impl.inc"
#undef IN_T
#undef NAME

#define IN_T double
#define NAME(f) pointwise_oracle_f64_##f
#include "pointwise_oracle_impl.inc"
#undef IN_T
#undef NAME
