/*
 * CPU oracle for multichannel 2-D convolution: forward, and (second half of the file)
 * the backward forms with respect to the input and the filters.  TEST INFRASTRUCTURE ONLY:
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

/*
 * The two backward forms (Section 2.1.1 calls them closely related to the forward form
 * and describes none of them; Section 2.1: one descriptor serves forward and backward,
 * results are returned raw or accumulated).  They are what back-propagation needs: with
 * O the forward result above and a given array dO of the shape of O,
 *
 *   dD[n,c,h,w] = sum over all (k,p,q,r,s) with (g(p,..,r,..), g(q,..,s,..)) = (h,w)
 *                 of F[k,c,r,s] * dO[n,k,p,q]            (derivative w.r.t. the input)
 *   dF[k,c,r,s] = sum_n sum_p sum_q dO[n,k,p,q] * D0[n,c,g(p,..,r,..),g(q,..,s,..)]
 *                                                          (derivative w.r.t. the filters)
 *
 * i.e. the transposes of the forward map, which is linear in D and in F.  Both are
 * written as the forward loop nest with the roles of the arrays exchanged, nothing else:
 * backward-data visits every (n,k,p,q,c,r,s) of the forward loops and ADDS F*dO to the
 * input element the forward loop READ there (taps in the zero border contribute to
 * nothing); backward-filter accumulates dO*D0 over (n,p,q) for each filter element.
 * Results are scaled and accumulated like the forward one: out = alpha*acc + beta*old.
 */

/* dx (N,C,H,W; strides dxs) from dy (N,K,P,Q; strides dys) and w (packed K,C,R,S). */
int conv_oracle_backward_data(const float *w, int K, int C, int R, int S,
                              const float *dy, const long long *dys, int N, int P, int Q,
                              int pad_h, int pad_w, int u, int v, int mode,
                              double alpha, double beta,
                              const double *dx_old, double *dx, const long long *dxs,
                              int H, int W, int nthreads)
{
    if (N < 1 || C < 1 || H < 1 || W < 1 || K < 1 || R < 1 || S < 1) return -1;
    if (u < 1 || v < 1 || pad_h < 0 || pad_w < 0) return -2;
    if (mode != 0 && mode != 1) return -3;
    if (conv_oracle_output_dim(H, R, u, pad_h) != P || P < 1) return -4;
    if (conv_oracle_output_dim(W, S, v, pad_w) != Q || Q < 1) return -5;
    if (beta != 0.0 && dx_old == NULL) return -6;
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#else
    (void)nthreads;
#endif
    long long NC = (long long)N * C;
    long long nc;
    /* one (n,c) plane of dx per iteration: no two iterations add to the same element */
#pragma omp parallel for schedule(dynamic, 1)
    for (nc = 0; nc < NC; ++nc) {
        int n = (int)(nc / C);
        int c = (int)(nc % C);
        for (int h = 0; h < H; ++h)
            for (int ww = 0; ww < W; ++ww) {
                long long o = n * dxs[0] + c * dxs[1] + h * dxs[2] + ww * dxs[3];
                dx[o] = 0.0;
            }
        for (int k = 0; k < K; ++k)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    double g = (double)dy[n * dys[0] + k * dys[1] + p * dys[2] + q * dys[3]];
                    for (int r = 0; r < R; ++r) {
                        int h = (mode == 0) ? p * u + R - r - 1 - pad_h : p * u + r - pad_h;
                        for (int s = 0; s < S; ++s) {
                            int ww = (mode == 0) ? q * v + S - s - 1 - pad_w : q * v + s - pad_w;
                            if (h >= 0 && h < H && ww >= 0 && ww < W) {
                                double f = (double)w[(((long long)k * C + c) * R + r) * S + s];
                                dx[n * dxs[0] + c * dxs[1] + h * dxs[2] + ww * dxs[3]] += f * g;
                            }
                        }
                    }
                }
        for (int h = 0; h < H; ++h)
            for (int ww = 0; ww < W; ++ww) {
                long long o = n * dxs[0] + c * dxs[1] + h * dxs[2] + ww * dxs[3];
                double out = alpha * dx[o];
                if (beta != 0.0) out += beta * dx_old[o];
                dx[o] = out;
            }
    }
    return 0;
}

/* dw (packed K,C,R,S) from x (N,C,H,W; strides xs) and dy (N,K,P,Q; strides dys). */
int conv_oracle_backward_filter(const float *x, const long long *xs, int N, int C, int H, int W,
                                const float *dy, const long long *dys, int K, int P, int Q,
                                int pad_h, int pad_w, int u, int v, int mode,
                                double alpha, double beta,
                                const double *dw_old, double *dw, int R, int S, int nthreads)
{
    if (N < 1 || C < 1 || H < 1 || W < 1 || K < 1 || R < 1 || S < 1) return -1;
    if (u < 1 || v < 1 || pad_h < 0 || pad_w < 0) return -2;
    if (mode != 0 && mode != 1) return -3;
    if (conv_oracle_output_dim(H, R, u, pad_h) != P || P < 1) return -4;
    if (conv_oracle_output_dim(W, S, v, pad_w) != Q || Q < 1) return -5;
    if (beta != 0.0 && dw_old == NULL) return -6;
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#else
    (void)nthreads;
#endif
    long long KC = (long long)K * C;
    long long kc;
#pragma omp parallel for schedule(dynamic, 1)
    for (kc = 0; kc < KC; ++kc) {
        int k = (int)(kc / C);
        int c = (int)(kc % C);
        for (int r = 0; r < R; ++r)
            for (int s = 0; s < S; ++s) {
                double acc = 0.0;
                for (int n = 0; n < N; ++n)
                    for (int p = 0; p < P; ++p) {
                        int h = (mode == 0) ? p * u + R - r - 1 - pad_h : p * u + r - pad_h;
                        for (int q = 0; q < Q; ++q) {
                            int ww = (mode == 0) ? q * v + S - s - 1 - pad_w : q * v + s - pad_w;
                            double d0 = 0.0;
                            if (h >= 0 && h < H && ww >= 0 && ww < W)
                                d0 = (double)x[n * xs[0] + c * xs[1] + h * xs[2] + ww * xs[3]];
                            acc += (double)dy[n * dys[0] + k * dys[1] + p * dys[2] + q * dys[3]] * d0;
                        }
                    }
                long long o = (((long long)k * C + c) * R + r) * S + s;
                double out = alpha * acc;
                if (beta != 0.0) out += beta * dw_old[o];
                dw[o] = out;
            }
    }
    return 0;
}
