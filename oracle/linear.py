"""The compensated W3A16 linear in fp64.

Test infrastructure only (see the package docstring).

The compensated weight is the LoRC identity of Section 3.1.2,
W~ = Q^-1(W_q) + U V, with Q^-1 from Eq. wdq.  With the weight stored
[out N x in K] and the activations X [M x K], the layer output is

    Y = X W_dq^T + (X V^T) U^T,      U [N x r],  V [r x K].

Everything is evaluated in fp64 with no intermediate rounding; the inputs
(X, U, V, scales, zeros) are fp16 values widened exactly.
"""
import numpy as np

from .quantize import dequantize


def linear_from_dense(X, W_dq, U=None, V=None):
    X = np.asarray(X, dtype=np.float64)
    Y = X @ np.asarray(W_dq, dtype=np.float64).T
    if U is not None and V is not None and np.asarray(U).shape[1] > 0:
        T = X @ np.asarray(V, dtype=np.float64).T
        Y = Y + T @ np.asarray(U, dtype=np.float64).T
    return Y


def w3lr_linear(X, codes, scales, zeros, U=None, V=None):
    """X fp16 [M,K]; codes uint8 [N,K]; scales/zeros fp16 [N,K/64]; U [N,r]; V [r,K]."""
    return linear_from_dense(X, dequantize(codes, scales, zeros), U, V)
