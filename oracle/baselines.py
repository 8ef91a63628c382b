"""Accuracy baselines for the MRE report (Section 4.2, Tables 1-2) -- TEST/BENCH INFRASTRUCTURE ONLY.

Plain numpy emulations, for a subset of query rows of ONE head, of the two comparison precisions the
paper tabulates next to INT-FlashAttention: attention in fp16, and attention in FP8 with tensor-level
scales.  The paper gives neither their exact arithmetic nor its MRE formula, so these columns are
context, not pins: PARITY UNPINNED (the e4m3 rounding itself is pinned in tests/test_oracle_baselines.py
against the format's definition).
"""
from __future__ import annotations

import numpy as np

E4M3_MAX = 448.0          # OCP FP8 e4m3: 4 exponent bits (bias 7), 3 mantissa bits, no infinities


def round_e4m3(x):
    """Round fp64/fp32 values to the nearest e4m3 value (ties to even), saturating at +-448."""
    x = np.asarray(x, np.float64)
    ax = np.minimum(np.abs(x), E4M3_MAX)
    e = np.floor(np.log2(np.maximum(ax, 2.0 ** -20)))
    e = np.maximum(e, -6.0)                      # below 2^-6 the format is subnormal: fixed step 2^-9
    step = 2.0 ** (e - 3.0)
    return np.sign(x) * np.minimum(np.rint(ax / step) * step, E4M3_MAX)


def _scores(Qr, K, causal, rows, scale):
    S = (Qr.astype(np.float32) @ K.astype(np.float32).T) * np.float32(scale)
    if causal:
        S = np.where(np.arange(K.shape[0])[None, :] <= rows[:, None], S, -np.inf)
    return S


def attention_fp16(Q, K, V, rows, causal=False, scale=1.0):
    """fp16 inputs, fp32 accumulation, P~ cast to fp16 before the second product, fp16 output."""
    Q, K, V = (np.asarray(a).astype(np.float16) for a in (Q, K, V))
    S = _scores(Q[rows], K, causal, rows, scale)
    P = np.exp(S - S.max(-1, keepdims=True)).astype(np.float32)
    l = P.sum(-1, keepdims=True)
    O = (P.astype(np.float16).astype(np.float32) @ V.astype(np.float32)) / l
    return O.astype(np.float16).astype(np.float64)


def attention_fp8_tensor(Q, K, V, rows, causal=False, scale=1.0):
    """Q, K, V quantized to e4m3 with ONE scale per tensor (absmax / 448), fp32 scores,
    P~ in (0, 1] cast to e4m3 before the second product, fp32 accumulation."""
    out = []
    for X in (Q, K, V):
        X = np.asarray(X, np.float64)
        s = np.abs(X).max() / E4M3_MAX
        out.append((round_e4m3(X / s), s))
    (Q8, sq), (K8, sk), (V8, sv) = out
    S = _scores(Q8[rows], K8, causal, rows, scale * sq * sk)
    P = np.exp(S - S.max(-1, keepdims=True)).astype(np.float32)
    l = P.sum(-1, keepdims=True, dtype=np.float32)
    O = (round_e4m3(P).astype(np.float32) @ V8.astype(np.float32)) / l * np.float32(sv)
    return O.astype(np.float64)


def mre(O_hat, O_ref):
    """Two readings of the paper's 'mean relative error': sum|dO| / sum|O| (robust) and the mean of the
    element-wise relative error with a floor of 1e-6 max|O| on the denominator."""
    O_hat, O_ref = np.asarray(O_hat, np.float64), np.asarray(O_ref, np.float64)
    d = np.abs(O_hat - O_ref)
    eps = 1e-6 * np.abs(O_ref).max()
    return {"sum_ratio": float(d.sum() / np.abs(O_ref).sum()),
            "mean_elementwise": float(np.mean(d / np.maximum(np.abs(O_ref), eps)))}
