"""ctypes front end of the CPU oracle (oracle/intfa_oracle.c) -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg import this package.
It imports nothing from the HIP package and shares no code with it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "intfa_oracle.c")
_LIB = os.path.join(_HERE, "_intfa_oracle.so")
_LIB_SANITIZED = os.path.join(_HERE, "_intfa_oracle_sanitized.so")

# No fast-math, no contraction: every fp32 operation in the C file rounds once, as written.
_CFLAGS = ["-O3", "-march=native", "-fopenmp", "-fPIC", "-shared", "-std=c11",
           "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra"]


def build(force: bool = False) -> str:
    """Compile the oracle with the host gcc.  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", *_CFLAGS, _SRC, "-o", _LIB, "-lm"])
    return _LIB


def build_sanitized() -> str:
    """The same source under AddressSanitizer and UndefinedBehaviorSanitizer (any report aborts), for the test that runs
    the pins against it in a child process (the sanitizer runtime has to be preloaded into that process)."""
    subprocess.check_call(["gcc", "-O1", "-g", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-ffp-contract=off", "-fno-fast-math",
                           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-Wall", "-Wextra",
                           _SRC, "-o", _LIB_SANITIZED, "-lm"])
    return _LIB_SANITIZED


_lib = None


def _load():
    global _lib
    if _lib is None:
        # INTFA_ORACLE_LIB: a prebuilt library to load instead (the sanitized build, in the child process of its test)
        lib = ctypes.CDLL(os.environ.get("INTFA_ORACLE_LIB") or build())
        vp, i64, i32, f64 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_double
        lib.orc_num_threads.restype = ctypes.c_int
        lib.orc_quantize_rows.argtypes = [vp, i64, i64, vp, vp]
        lib.orc_hadamard_rows.argtypes = [vp, i64, i64, vp]
        lib.orc_hadamard_rows.restype = None
        lib.orc_qk_i32.argtypes = [vp, vp, i64, i32, vp]
        lib.orc_pv_i32.argtypes = [vp, vp, i64, i32, vp]
        lib.orc_int_flash_attn_fwd.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, i64, i64, i32, i32, i32,
                                               i32, i32, vp, i64, vp, vp, vp, f64, f64, vp, vp, vp]
        lib.orc_attention_fp64.argtypes = [vp, vp, vp, i64, i64, i32, i32, f64, vp, i64, vp]
        lib.orc_round_to_half.argtypes = [ctypes.c_float]
        lib.orc_round_to_half.restype = ctypes.c_float
        lib.orc_int_flash_attn_fwd_half.argtypes = [vp, vp, vp, vp, vp, i32, i32, i64, i64, i32, i32, i32, vp, i64, vp, vp, vp]
        lib.orc_int_flash_attn_fwd_half.restype = None
        for f in (lib.orc_quantize_rows, lib.orc_qk_i32, lib.orc_pv_i32,
                  lib.orc_int_flash_attn_fwd, lib.orc_attention_fp64):
            f.restype = None
        _lib = lib
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


def num_threads() -> int:
    return _load().orc_num_threads()


def quantize_rows(X):
    """X: real [rows, cols] (fp16/fp32, widened exactly to fp32).  -> (int8 [rows, cols], fp32 [rows])."""
    X = _c(X, np.float32)
    rows, cols = X.shape
    q = np.empty((rows, cols), np.int8)
    s = np.empty(rows, np.float32)
    _load().orc_quantize_rows(_p(X), rows, cols, _p(q), _p(s))
    return q, s


def quantize_tokenwise(X):
    """Token-level scheme of Q and K (Section 3.2): X [..., d] -> int8 same shape, scale [...]."""
    X = np.asarray(X)
    q, s = quantize_rows(X.reshape(-1, X.shape[-1]))
    return q.reshape(X.shape), s.reshape(X.shape[:-1])


def hadamard_rows(X):
    """Unnormalized Walsh-Hadamard transform (Sylvester order) of the last axis, fp32 butterflies."""
    X = np.asarray(X)
    x2 = _c(X.reshape(-1, X.shape[-1]), np.float32)
    rows, cols = x2.shape
    assert cols & (cols - 1) == 0
    y = np.empty_like(x2)
    _load().orc_hadamard_rows(_p(x2), rows, cols, _p(y))
    return y.reshape(X.shape)


def quantize_tokenwise_hadamard(X, scale_mul=1.0):
    """Token-level quantization of the Hadamard-rotated rows: codes of H_d x, scale = max|H_d x| / 127 * scale_mul
    (scale_mul = 1/sqrt(d) makes the rotation orthonormal)."""
    q, s = quantize_tokenwise(hadamard_rows(X))
    return q, (s * np.float32(scale_mul)).astype(np.float32)


def quantize_headwise(X, global_scale=False):
    """Tensor-level scheme of V (Section 3.2): X [heads, N, d] -> int8 same shape, scale [heads].
    global_scale=True uses one scale for the whole array, replicated to every head."""
    X = np.asarray(X)
    heads = X.shape[0]
    if global_scale:
        q, s = quantize_rows(X.reshape(1, -1))
        return q.reshape(X.shape), np.full(heads, s[0], np.float32)
    q, s = quantize_rows(X.reshape(heads, -1))
    return q.reshape(X.shape), s


def quantize_blockwise(X, block):
    """Per-block scheme for V (the paper's stated future work): X [heads, N, d] -> int8 same shape and one scale
    per (head, block of `block` consecutive keys), shape [heads, ceil(N / block)].  Same rounding rule."""
    X = np.asarray(X)
    heads, N, d = X.shape
    Tc = -(-N // block)
    q = np.empty(X.shape, np.int8)
    s = np.empty((heads, Tc), np.float32)
    full = N // block
    if full:
        qq, ss = quantize_rows(X[:, :full * block].reshape(heads * full, block * d))
        q[:, :full * block] = qq.reshape(heads, full * block, d)
        s[:, :full] = ss.reshape(heads, full)
    if full < Tc:
        qq, ss = quantize_rows(X[:, full * block:].reshape(heads, -1))
        q[:, full * block:] = qq.reshape(heads, N - full * block, d)
        s[:, full] = ss
    return q, s


def qk_i32(Q, K):
    Q, K = _c(Q, np.int8), _c(K, np.int8)
    N, d = Q.shape
    S = np.empty((N, N), np.int32)
    _load().orc_qk_i32(_p(Q), _p(K), N, d, _p(S))
    return S


def pv_i32(P, V):
    P, V = _c(P, np.int8), _c(V, np.int8)
    N, d = V.shape
    out = np.empty((N, d), np.int32)
    _load().orc_pv_i32(_p(P), _p(V), N, d, _p(out))
    return out


def int_flash_attn_fwd(Q, K, V, sQ, sK, sV, causal, Bc, p_quant=True, row_idx=None,
                       tie_rel=0.0, tie_abs=0.0, want_P=False, tie_flip=None):
    """Algorithm 1.  Q int8 [heads, Nq, d], sQ fp32 [heads, Nq]; K, V int8 [heads, N, d], sK fp32 [heads, N]
    (Nq = N in the paper; with Nq != N the queries are the last Nq positions for the causal mask);
    sV fp32 [heads] (tensor-level scale of V) or [heads, ceil(N/Bc)] (one scale per key block, applied where
    P V_j enters O).
    tie_flip: optional uint64 [rows]; bit k rounds the k-th flagged near-tie entry of that row the other way.
    Returns a dict: O fp32 [rows, d], l, m fp32 [rows], n_tie int32 [rows], P int8 [rows, N] (if asked)."""
    Q, K, V = _c(Q, np.int8), _c(K, np.int8), _c(V, np.int8)
    heads, Nq, d = Q.shape
    N = K.shape[1]
    sQ, sK, sV = _c(sQ, np.float32), _c(sK, np.float32), _c(sV, np.float32)
    assert K.shape == (heads, N, d) and V.shape == K.shape
    assert not causal or N >= Nq
    sv_per_block = sV.ndim == 2
    assert sQ.shape == (heads, Nq) and sK.shape == (heads, N)
    assert sV.shape == ((heads, -(-N // int(Bc))) if sv_per_block else (heads,))
    if row_idx is not None:
        row_idx = _c(row_idx, np.int64)
        n = row_idx.size
        assert n == 0 or (row_idx.min() >= 0 and row_idx.max() < heads * Nq)
    else:
        n = heads * Nq
    O = np.empty((n, d), np.float32)
    l = np.empty(n, np.float32)
    m = np.empty(n, np.float32)
    n_tie = np.zeros(n, np.int32)
    P = np.empty((n, N), np.int8) if want_P else None
    if tie_flip is not None:
        tie_flip = _c(tie_flip, np.uint64)
        assert tie_flip.shape == (n,)
    if n:
        _load().orc_int_flash_attn_fwd(_p(Q), _p(K), _p(V), _p(sQ), _p(sK), _p(sV), 1, heads, Nq, N, d,
                                       int(bool(causal)), int(Bc), int(bool(p_quant)), int(sv_per_block),
                                       _p(row_idx), n, _p(O), _p(l), _p(m),
                                       float(tie_rel), float(tie_abs), _p(n_tie), _p(P), _p(tie_flip))
    return {"O": O, "l": l, "m": m, "n_tie": n_tie, "P": P}


def round_to_half(x):
    """Nearest fp16 value of each fp32 element (ties to even, gradual underflow), as fp32."""
    x = _c(x, np.float32)
    f = _load().orc_round_to_half
    return np.array([f(float(v)) for v in x.ravel()], np.float32).reshape(x.shape)


def int_flash_attn_fwd_half(Q, K, V, sQ, sK, causal, Bc, row_idx=None):
    """Half-INT8 variant (Section 4): INT8 Q, K with token-level scales, fp16 V, P~ = fp16(exp(S - m)).
    Q int8 [heads, Nq, d], sQ fp32 [heads, Nq]; K int8, V fp16 [heads, N, d], sK fp32 [heads, N].  Returns a dict O, l, m."""
    Q, K = _c(Q, np.int8), _c(K, np.int8)
    assert V.dtype == np.float16
    Vf = _c(V, np.float32)                      # exact widening
    heads, Nq, d = Q.shape
    N = K.shape[1]
    sQ, sK = _c(sQ, np.float32), _c(sK, np.float32)
    assert K.shape == (heads, N, d) and Vf.shape == K.shape and sQ.shape == (heads, Nq) and sK.shape == (heads, N)
    assert not causal or N >= Nq
    if row_idx is not None:
        row_idx = _c(row_idx, np.int64)
        n = row_idx.size
        assert n == 0 or (row_idx.min() >= 0 and row_idx.max() < heads * Nq)
    else:
        n = heads * Nq
    O = np.empty((n, d), np.float32)
    l = np.empty(n, np.float32)
    m = np.empty(n, np.float32)
    if n:
        _load().orc_int_flash_attn_fwd_half(_p(Q), _p(K), _p(Vf), _p(sQ), _p(sK), 1, heads, Nq, N, d,
                                            int(bool(causal)), int(Bc), _p(row_idx), n, _p(O), _p(l), _p(m))
    return {"O": O, "l": l, "m": m}


def attention_fp64(Q, K, V, causal=False, scale=1.0, row_idx=None):
    """Section 2.1 definition in fp64.  Q, K, V real [heads, N, d]."""
    Q, K, V = _c(Q, np.float64), _c(K, np.float64), _c(V, np.float64)
    heads, N, d = Q.shape
    if row_idx is not None:
        row_idx = _c(row_idx, np.int64)
        n = row_idx.size
    else:
        n = heads * N
    O = np.empty((n, d), np.float64)
    if n:
        _load().orc_attention_fp64(_p(Q), _p(K), _p(V), heads, N, d, int(bool(causal)), float(scale),
                                   _p(row_idx), n, _p(O))
    return O


def compare_up_to_ties(O_rows, Q, K, V, sQ, sK, sV, causal, Bc, row_idx=None, tie_rel=8 * 2.0 ** -24, tie_abs=2e-6,
                       tol=1e-3):
    """Compares O_rows [rows, d] (the implementation under test) with Algorithm 1 row by row.

    Line 11 rounds 127 exp(S - m) to an integer on an fp32 argument; where that argument lies within fp32 evaluation
    noise of a half-integer (tie_rel, tie_abs: see orc_int_flash_attn_fwd) either neighbour is a result of the
    algorithm.  A row passes if it is within tol * max|O| of the oracle's output for SOME resolution of its flagged
    entries: first the default one; for a row that misses it, the flagged entries are flipped one at a time
    (greedily, each step re-evaluating the row in the oracle) until the row matches or no flip helps.
    Returns a dict: err (per row, against the best resolution found), err_default (against the default one),
    n_tie, flips (per row, number of entries flipped), scale (= max|O| of the default result), l."""
    ref = int_flash_attn_fwd(Q, K, V, sQ, sK, sV, causal, Bc, row_idx=row_idx, tie_rel=tie_rel, tie_abs=tie_abs)
    O_ref = ref["O"].astype(np.float64)
    got = np.asarray(O_rows, np.float64)
    assert got.shape == O_ref.shape
    scale = float(np.abs(O_ref).max())
    err_default = np.abs(got - O_ref).max(axis=1)
    err = err_default.copy()
    flips = np.zeros(len(err), np.int32)
    rows = np.arange(len(err), dtype=np.int64) if row_idx is None else _c(row_idx, np.int64)
    for r in np.nonzero((err_default > tol * scale) & (ref["n_tie"] > 0))[0]:
        k = int(min(ref["n_tie"][r], 64))
        mask, best = np.uint64(0), err_default[r]
        for _ in range(k):
            cand = np.array([mask ^ np.uint64(1 << b) for b in range(k)], np.uint64)
            alt = int_flash_attn_fwd(Q, K, V, sQ, sK, sV, causal, Bc, row_idx=np.full(k, rows[r], np.int64),
                                     tie_rel=tie_rel, tie_abs=tie_abs, tie_flip=cand)["O"].astype(np.float64)
            e = np.abs(alt - got[r]).max(axis=1)
            b = int(e.argmin())
            if e[b] >= best:
                break
            mask, best = cand[b], e[b]
            if best <= tol * scale:
                break
        err[r] = best
        flips[r] = bin(int(mask)).count("1")
    return {"err": err, "err_default": err_default, "n_tie": ref["n_tie"], "flips": flips, "scale": scale, "l": ref["l"]}
