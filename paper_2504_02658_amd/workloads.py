"""Seeded synthetic inputs shaped like the paper's workloads.

This module only draws random inputs (weights, activations, router outputs); it
contains none of the method's arithmetic (no quantizer, no packing, no GEMM).
Both the GPU tests / benchmark and the CPU oracle tests take their inputs from
here, so that the two sides see identical data without sharing any code of the
method itself.

The shapes stand in for the expert FFN matrices of Mixtral-8x7B (hidden 4096,
ffn 14336, 8 experts, top-2) and DeepSeek-MoE (hidden 2048, fine-grained experts
of ffn 1408, 64 routed with top-6 plus 2 shared) that the paper evaluates
(Section 4, appendix "Shape of GeMM in Throughput Tests").  The real
checkpoints are not available, so weights are N(0, 0.02^2) fp32 (optionally with
a few input channels scaled up, mimicking the channel-wise outliers of
Section 3.1.1) and activations are N(0, 1) fp16.
"""
from dataclasses import dataclass, field
from typing import Tuple

import numpy as np

WEIGHT_STD = 0.02


@dataclass(frozen=True)
class LinearCase:
    name: str
    M: int
    N: int
    K: int
    r: int
    seed: int
    outlier_frac: float = 0.0      # fraction of input channels (columns of W) scaled by outlier_gain
    outlier_gain: float = 8.0


@dataclass(frozen=True)
class MoECase:
    name: str
    T: int                          # tokens
    H: int                          # hidden size
    F: int                          # expert ffn size
    E: int                          # routed experts
    topk: int
    seed: int
    n_shared: int = 0               # always-on experts, appended after the routed ones
    rank_choices: Tuple[int, ...] = (16, 32, 64)   # one draw per routed expert
    shared_rank: int = 0
    renormalize: bool = True        # renormalise the top-k gate weights to sum to one
    zipf_s: float = 0.0             # >0: popularity skew via biased gate logits


# The five configurations of the build target.
C0 = LinearCase("c0_small", M=16, N=1024, K=1024, r=16, seed=1000)
C1 = {m: LinearCase(f"c1_mixtral_up_decode_M{m}", M=m, N=14336, K=4096, r=32, seed=1001,
                    outlier_frac=0.01) for m in (1, 4, 16)}
C2 = LinearCase("c2_mixtral_down_prefill", M=512, N=4096, K=14336, r=64, seed=1002)
C3 = MoECase("c3_mixtral_layer", T=512, H=4096, F=14336, E=8, topk=2, seed=1003,
             rank_choices=(16, 32, 64), renormalize=True)
C4 = MoECase("c4_deepseek_layer", T=4096, H=2048, F=1408, E=64, topk=6, seed=1004,
             n_shared=2, rank_choices=(8,), shared_rank=128, renormalize=False, zipf_s=1.2)


def _rng(*key):
    return np.random.default_rng(np.random.SeedSequence([int(k) for k in key]))


def gen_weight(N, K, seed, outlier_frac=0.0, outlier_gain=8.0, std=WEIGHT_STD):
    """fp32 [N, K] weight, N(0, std^2); floor(outlier_frac*K) distinct input channels scaled up."""
    rng = _rng(seed, 1)
    W = rng.standard_normal((N, K), dtype=np.float32)
    W *= np.float32(std)
    n_out = int(np.floor(outlier_frac * K))
    if n_out:
        cols = _rng(seed, 2).choice(K, size=n_out, replace=False)
        W[:, cols] *= np.float32(outlier_gain)
    return W


def gen_weight_lowrank(N, K, seed, modes=8, gain=6.0, decay=0.75, outlier_frac=0.0, std=WEIGHT_STD):
    """gen_weight plus `modes` rank-one components whose strengths fall off geometrically from `gain`
    times the top singular value of the Gaussian part: the spectrum with a few dominant directions
    over a flat bulk that the compressor's low-rank step is meant for."""
    W = gen_weight(N, K, seed, outlier_frac=outlier_frac, std=std)
    rng = _rng(seed, 4)
    bulk_top = std * (np.sqrt(N) + np.sqrt(K))
    for k in range(modes):
        a = rng.standard_normal(N).astype(np.float32)
        b = rng.standard_normal(K).astype(np.float32)
        a /= np.linalg.norm(a)
        b /= np.linalg.norm(b)
        W += np.float32(gain * decay ** k * bulk_top) * np.outer(a, b)
    return W


def gen_activations(M, K, seed):
    """fp16 [M, K], N(0, 1)."""
    return _rng(seed, 3).standard_normal((M, K), dtype=np.float32).astype(np.float16)


def linear_inputs(case: LinearCase):
    W = gen_weight(case.N, case.K, case.seed, case.outlier_frac, case.outlier_gain)
    X = gen_activations(case.M, case.K, case.seed)
    return X, W


# ---------------------------------------------------------------- MoE layers

def expert_ranks(case: MoECase):
    """Rank per expert (routed then shared); one seeded draw per routed expert."""
    rng = _rng(case.seed, 10)
    routed = rng.choice(np.asarray(case.rank_choices), size=case.E)
    return [int(r) for r in routed] + [int(case.shared_rank)] * case.n_shared


def expert_weight(case: MoECase, e: int, which: str):
    """fp32 weight of expert e; which in {'w1','w3'} -> [F, H], 'w2' -> [H, F]."""
    idx = {"w1": 0, "w3": 1, "w2": 2}[which]
    N, K = (case.F, case.H) if which in ("w1", "w3") else (case.H, case.F)
    rng = _rng(case.seed, 20, e, idx)
    W = rng.standard_normal((N, K), dtype=np.float32)
    W *= np.float32(WEIGHT_STD)
    return W


def moe_activations(case: MoECase):
    return _rng(case.seed, 3).standard_normal((case.T, case.H), dtype=np.float32).astype(np.float16)


def moe_routing(case: MoECase):
    """Router outputs for the layer: (ids int32 [T, topk + n_shared], gates fp32 [same]).

    The router itself (gate GEMM, softmax, top-k) is outside the library; here the
    gate logits are drawn directly.  Softmax over the routed experts, top-k with
    ties going to the lowest expert id, optional renormalisation (Mixtral style)
    and optional popularity skew: a seeded permutation pi of the experts and a
    bias -s*ln(pi_e + 1) on the logits (Zipf-like frequencies, standing in for the
    unbalanced expert activation the paper reports for DeepSeek-MoE).  Shared
    experts are appended as extra columns with weight 1.
    """
    rng = _rng(case.seed, 30)
    logits = rng.standard_normal((case.T, case.E)).astype(np.float64)
    if case.zipf_s > 0:
        perm = _rng(case.seed, 31).permutation(case.E)
        logits = logits - case.zipf_s * np.log(perm + 1.0)[None, :]
    p = np.exp(logits - logits.max(axis=1, keepdims=True))
    p /= p.sum(axis=1, keepdims=True)
    order = np.argsort(-p, axis=1, kind="stable")[:, : case.topk]
    gates = np.take_along_axis(p, order, axis=1)
    if case.renormalize:
        gates = gates / gates.sum(axis=1, keepdims=True)
    ids = order.astype(np.int32)
    gates = gates.astype(np.float32)
    if case.n_shared:
        sid = np.tile(np.arange(case.E, case.E + case.n_shared, dtype=np.int32), (case.T, 1))
        ids = np.concatenate([ids, sid], axis=1)
        gates = np.concatenate([gates, np.ones((case.T, case.n_shared), np.float32)], axis=1)
    return np.ascontiguousarray(ids), np.ascontiguousarray(gates)


def scaled(case, **kw):
    """A copy of a case with some fields replaced (used for reduced-size parity cases)."""
    d = {f: getattr(case, f) for f in case.__dataclass_fields__}
    d.update(kw)
    return type(case)(**d)
