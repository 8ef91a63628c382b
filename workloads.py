"""Seeded synthetic inputs for the INT-FlashAttention forward path.

This module only draws random activations.  It holds none of the method's
arithmetic (no quantization, no attention), so that both the CPU oracle's tests
and the HIP path's tests / benchmark can take their inputs from it without
sharing any code of the method itself.

The paper evaluates on synthetic one-layer attention activations drawn from
N(0,1) and U(-0.5,0.5) (Section 4.2, Tables 1 and 2) at sequence lengths
1k..16k (Section 4.1); the five workloads below have those distributions and
lengths, plus an outlier-channel case and a heavy-tailed case.

Every (workload, tensor, head) triple has its own counter-free seed, so a single
head can be regenerated without materialising the whole tensor.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

TENSOR_IDS = {"Q": 0, "K": 1, "V": 2}


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    H: int
    N: int
    d: int
    causal: bool
    dist: str          # "normal" | "uniform" | "uniform_outlier" | "student_t3"
    in_dtype: str      # numpy dtype name of the real-valued Q, K, V
    out_dtype: str     # dtype the attention output is stored in
    seed: int

    @property
    def heads(self) -> int:
        return self.B * self.H

    @property
    def ops(self) -> float:
        """Integer operations (2 per multiply-accumulate) of both GEMMs; a causal
        workload counts only the lower triangle (N*(N+1)/2 score elements)."""
        score = self.N * (self.N + 1) / 2 if self.causal else float(self.N) * self.N
        return 4.0 * self.heads * score * self.d


WORKLOADS = {
    "c1": Workload("c1", 1, 1, 128, 64, False, "normal", "float32", "float32", 1),
    "c2": Workload("c2", 4, 16, 1024, 64, False, "normal", "float16", "float16", 2),
    "c3": Workload("c3", 4, 32, 4096, 128, True, "normal", "float16", "float16", 3),
    "c4": Workload("c4", 8, 32, 8192, 128, False, "uniform_outlier", "float16", "float16", 4),
    "c5": Workload("c5", 1, 32, 16384, 128, True, "student_t3", "float16", "float16", 5),
}


def head_tensor(w: Workload, tensor: str, head: int) -> np.ndarray:
    """Real-valued [N, d] activations of one (b, h) head of Q, K or V."""
    rng = np.random.default_rng([w.seed, TENSOR_IDS[tensor], head])
    if w.dist == "normal":
        x = rng.standard_normal((w.N, w.d), dtype=np.float32)
    elif w.dist == "uniform":                      # U(-0.5, 0.5), the second distribution of Section 4.2
        x = rng.random((w.N, w.d), dtype=np.float32) - np.float32(0.5)
    elif w.dist == "uniform_outlier":
        x = rng.random((w.N, w.d), dtype=np.float32) - np.float32(0.5)
        ch = rng.choice(w.d, size=4, replace=False)
        x[:, ch] *= np.float32(20.0)
    elif w.dist == "student_t3":
        x = (rng.standard_t(3.0, size=(w.N, w.d)) / np.sqrt(3.0)).astype(np.float32)
    else:
        raise ValueError(w.dist)
    return x.astype(w.in_dtype)


def tensor(w: Workload, name: str, heads=None) -> np.ndarray:
    """[len(heads), N, d] stack of heads (all B*H heads, in (b, h) order, by default)."""
    heads = range(w.heads) if heads is None else heads
    out = np.empty((len(heads), w.N, w.d), dtype=w.in_dtype)
    for i, h in enumerate(heads):
        out[i] = head_tensor(w, name, h)
    return out


def custom(name, B, H, N, d, causal, dist="normal", in_dtype="float16",
           out_dtype="float16", seed=1234) -> Workload:
    """A workload of any shape with one of the three distributions (parity-test sizes)."""
    return Workload(name, B, H, N, d, causal, dist, in_dtype, out_dtype, seed)


def sample_rows(w: Workload, full_heads=2, rows_per_head=64):
    """Deterministic (head, row) sample for the large workloads: every row of the first
    `full_heads` heads and `rows_per_head` seeded rows of every other head.  Rows of
    the attention output are independent, so evaluating only these is exact for them.
    Returns a list of (head, sorted int64 row array)."""
    rng = np.random.default_rng([w.seed, 99])
    out = []
    for h in range(w.heads):
        if h < full_heads:
            rows = np.arange(w.N, dtype=np.int64)
        else:
            rows = np.sort(rng.choice(w.N, size=min(rows_per_head, w.N), replace=False)).astype(np.int64)
        out.append((h, rows))
    return out
