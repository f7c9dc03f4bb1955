"""Second, independent CPU derivation: explicit lowering to one matrix product.

TEST INFRASTRUCTURE ONLY.  Follows the paper's Section 3 description of lowering
(Fig. 1): the filter tensor is reshaped to F_m (K x CRS), the input is duplicated
into D_m (CRS x NPQ), and O_m = F_m . D_m (K x NPQ).  This is the approach the paper
rejects for the GPU because D_m is large; here it only cross-checks the seven-loop
oracle.  numpy, float64, small problems only.
"""
import numpy as np

CONVOLUTION = 0
CROSS_CORRELATION = 1


def lower_filter(w):
    """F_m: K x (C*R*S), row k = filter k flattened with s fastest."""
    K = w.shape[0]
    return np.asarray(w, dtype=np.float64).reshape(K, -1)


def lower_data(x, R, S, pad, stride, mode, P, Q):
    """D_m: (C*R*S) x (N*P*Q); row (c,r,s), column (n,p,q); zeros where the tap
    falls in the zero border (D0 of eq. 3)."""
    x = np.asarray(x, dtype=np.float64)
    N, C, H, W = x.shape
    Dm = np.zeros((C * R * S, N * P * Q), dtype=np.float64)
    for c in range(C):
        for r in range(R):
            for s in range(S):
                row = (c * R + r) * S + s
                for n in range(N):
                    for p in range(P):
                        h = p * stride[0] + (R - r - 1 if mode == CONVOLUTION else r) - pad[0]
                        if h < 0 or h >= H:
                            continue
                        for q in range(Q):
                            ww = q * stride[1] + (S - s - 1 if mode == CONVOLUTION else s) - pad[1]
                            if 0 <= ww < W:
                                Dm[row, (n * P + p) * Q + q] = x[n, c, h, ww]
    return Dm


def conv_forward_lowered(x, w, pad=(0, 0), stride=(1, 1), mode=CROSS_CORRELATION):
    """Returns (O as (N,K,P,Q) float64, F_m, D_m)."""
    N, C, H, W = x.shape
    K, _, R, S = w.shape
    P = -((-(H - R + 1 + 2 * pad[0])) // stride[0])   # eq. 1, ceiling
    Q = -((-(W - S + 1 + 2 * pad[1])) // stride[1])
    Fm = lower_filter(w)
    Dm = lower_data(x, R, S, pad, stride, mode, P, Q)
    Om = Fm @ Dm
    return Om.reshape(K, N, P, Q).transpose(1, 0, 2, 3).copy(), Fm, Dm
