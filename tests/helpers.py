"""Shared test helpers: build quantized Algorithm-1 inputs from the seeded workloads using the
ORACLE's quantizer (never the HIP path's), so expected values depend on oracle/ alone."""
import numpy as np

import oracle
import workloads


def quantized_inputs(w, heads=None, scaled=False):
    """Real Q, K, V of workload `w` -> dict with int8 tensors and scales [heads, ...].
    scaled=True folds 1/sqrt(d) into s_Q (exact by the linearity remark of Section 3.2)."""
    Q = workloads.tensor(w, "Q", heads)
    K = workloads.tensor(w, "K", heads)
    V = workloads.tensor(w, "V", heads)
    Qq, sQ = oracle.quantize_tokenwise(Q)
    Kq, sK = oracle.quantize_tokenwise(K)
    Vq, sV = oracle.quantize_headwise(V)
    if scaled:
        sQ = (sQ * np.float32(1.0 / np.sqrt(w.d))).astype(np.float32)
    return {"Q": Q, "K": K, "V": V, "Qq": Qq, "Kq": Kq, "Vq": Vq, "sQ": sQ, "sK": sK, "sV": sV}


def dequant(q, s):
    return q.astype(np.float64) * np.asarray(s, np.float64)[..., None]


def random_int8_problem(rng, heads, N, d, score_sigma=1.0):
    """Random int8 Q, K, V with scales chosen so that scores have standard deviation ~score_sigma."""
    Qq = rng.integers(-127, 128, (heads, N, d), dtype=np.int8)
    Kq = rng.integers(-127, 128, (heads, N, d), dtype=np.int8)
    Vq = rng.integers(-127, 128, (heads, N, d), dtype=np.int8)
    base = score_sigma / (73.3 * 73.3 * np.sqrt(d))      # std of uniform int8 ~ 73.3
    sQ = (rng.uniform(0.5, 1.5, (heads, N)) * np.sqrt(base)).astype(np.float32)
    sK = (rng.uniform(0.5, 1.5, (heads, N)) * np.sqrt(base)).astype(np.float32)
    sV = rng.uniform(0.005, 0.02, heads).astype(np.float32)
    return Qq, Kq, Vq, sQ, sK, sV
