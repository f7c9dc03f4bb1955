/*
 * CPU oracle for multichannel 2-D convolution forward.  TEST INFRASTRUCTURE ONLY:
 * it is used by the tests, the smoke check and the bench's cpu_baseline leg; the
 * product (the HIP library) never calls it and shares no code with it.
 *
 * It is the definition written out: the paper's Section 2.1.1 forward form, eq. 3,
 *
 *   O[n,k,p,q] = sum_c sum_r sum_s F[k,c,r,s] * D0[n,c,g(p,u,R,r,pad_h),g(q,v,S,s,pad_w)]
 *
 * with D0 the zero-extended input, the accessing function of eq. 2
 *   g(p,u,R,r,pad) = p*u + R - r - 1 - pad          (convolution: filter inverted)
 * or, for the cross-correlation variant the same section mentions,
 *   g'(p,u,r,pad)  = p*u + r - pad,
 * and the output size of eq. 1, P = ceil((H - R + 1 + 2*pad_h)/u), likewise Q.
 * The result is then scaled and accumulated, y = alpha*O + beta*y_old (the paper's
 * "return raw or accumulate" mode in its general BLAS-like form).
 *
 * Seven literal nested loops (four independent, three accumulating), double
 * accumulator, no tiling, no lowering, no reordering.  Inputs are float (fp32, or
 * bf16 values held exactly in a float); everything after the load is double.
 * Tensors are addressed through four element strides each, so any layout works.
 * OpenMP splits the (n,k) pairs over threads; that changes no arithmetic.
 */
#include <stddef.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* eq. 1: ceil((H - R + 1 + 2 pad)/u); returns 0 or less when no output exists. */
long long conv_oracle_output_dim(long long H, long long R, long long u, long long pad)
{
    long long num = H - R + 1 + 2 * pad;
    if (u < 1) return -1;
    if (num <= 0) return 0;
    return (num + u - 1) / u; /* ceiling of a positive quotient */
}

/* mode: 0 = convolution (eq. 2), 1 = cross-correlation.
 * xs, ys: element strides in the order n, c(k), h(p), w(q).  w is packed K,C,R,S.
 * y_old may be NULL when beta == 0 (then it is never read).
 * Returns 0, or a negative number when the arguments do not describe a problem. */
int conv_oracle_forward(const float *x, const long long *xs, int N, int C, int H, int W,
                        const float *w, int K, int R, int S,
                        int pad_h, int pad_w, int u, int v, int mode,
                        double alpha, double beta,
                        const double *y_old, double *y, const long long *ys,
                        int P, int Q, int nthreads)
{
    if (N < 1 || C < 1 || H < 1 || W < 1 || K < 1 || R < 1 || S < 1) return -1;
    if (u < 1 || v < 1 || pad_h < 0 || pad_w < 0) return -2;
    if (mode != 0 && mode != 1) return -3;
    if (conv_oracle_output_dim(H, R, u, pad_h) != P || P < 1) return -4;
    if (conv_oracle_output_dim(W, S, v, pad_w) != Q || Q < 1) return -5;
    if (beta != 0.0 && y_old == NULL) return -6;
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#else
    (void)nthreads;
#endif
    long long NK = (long long)N * K;
    long long nk;
#pragma omp parallel for schedule(dynamic, 1)
    for (nk = 0; nk < NK; ++nk) {
        int n = (int)(nk / K);
        int k = (int)(nk % K);
        for (int p = 0; p < P; ++p) {
            for (int q = 0; q < Q; ++q) {
                double acc = 0.0;
                for (int c = 0; c < C; ++c) {
                    for (int r = 0; r < R; ++r) {
                        int h = (mode == 0) ? p * u + R - r - 1 - pad_h : p * u + r - pad_h;
                        for (int s = 0; s < S; ++s) {
                            int ww = (mode == 0) ? q * v + S - s - 1 - pad_w : q * v + s - pad_w;
                            double d0 = 0.0; /* zero extension outside the image */
                            if (h >= 0 && h < H && ww >= 0 && ww < W)
                                d0 = (double)x[n * xs[0] + c * xs[1] + h * xs[2] + ww * xs[3]];
                            double f = (double)w[(((long long)k * C + c) * R + r) * S + s];
                            acc += f * d0;
                        }
                    }
                }
                long long yo = n * ys[0] + k * ys[1] + p * ys[2] + q * ys[3];
                double out = alpha * acc;
                if (beta != 0.0) out += beta * y_old[yo];
                y[yo] = out;
            }
        }
    }
    return 0;
}

int conv_oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
