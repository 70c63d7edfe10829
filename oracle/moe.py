"""Mixture-of-experts feed-forward layer built from compensated W3A16 linears.

Test infrastructure only (see the package docstring).

The paper runs its kernel inside the stock Mixtral / DeepSeek-MoE expert blocks
(Section 4.3.1) and does not restate them; the block is the standard SwiGLU
expert with top-k routing:

    y_t = sum_j g[t, j] * lin_w2^e( SiLU(lin_w1^e(x_t)) * lin_w3^e(x_t) ),  e = ids[t, j]

where every lin is the compensated linear of `linear.py`.  fp64 throughout; the
intermediate activation is *not* rounded to fp16 here.  Always-on shared
experts are expressed by the caller as extra routing columns with weight 1.
"""
import numpy as np

from .linear import w3lr_linear


def silu(a):
    return a / (1.0 + np.exp(-a))


def moe_forward(X, experts, ids, gates):
    """X fp16 [T,H]; experts: sequence of dicts with keys 'w1','w3','w2', each a dict
    (codes, scales, zeros, U, V) or a callable returning one (lazy materialisation);
    ids int [T,k]; gates float [T,k].  Returns fp64 [T,H]."""
    X64 = np.asarray(X, dtype=np.float64)
    ids = np.asarray(ids)
    gates = np.asarray(gates, dtype=np.float64)
    T = X64.shape[0]
    Y = None
    for e, ex in enumerate(experts):
        tok, slot = np.nonzero(ids == e)
        if tok.size == 0:
            continue
        ex = ex() if callable(ex) else ex
        xe = X64[tok]
        a = w3lr_linear(xe, **ex["w1"])
        b = w3lr_linear(xe, **ex["w3"])
        h = silu(a) * b
        o = w3lr_linear(h, **ex["w2"])
        if Y is None:
            Y = np.zeros((T, o.shape[1]), dtype=np.float64)
        np.add.at(Y, tok, gates[tok, slot][:, None] * o)
    if Y is None:
        raise ValueError("no token was routed to any expert")
    return Y
