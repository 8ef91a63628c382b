"""ctypes binding of include/intfa.h.  Argument marshalling only."""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libintfa.so")

IFA_F32, IFA_F16, IFA_BF16 = 0, 1, 2

# every symbol include/intfa.h declares, with its C signature
_vp, _i, _l = ctypes.c_void_p, ctypes.c_int, ctypes.c_long
SIGNATURES = {
    "ifa_status_str": (ctypes.c_char_p, [_i]),
    "ifa_set_stream": (_i, [_vp]),
    "quantize_tokenwise": (_i, [_vp, _i, _l, _i, _vp, _vp]),
    "quantize_tokenwise_ex": (_i, [_vp, _i, _l, _i, _vp, _vp, ctypes.c_float, _vp]),
    "quantize_tokenwise_hadamard": (_i, [_vp, _i, _l, _i, _vp, _vp, ctypes.c_float, _vp]),
    "quantize_headwise": (_i, [_vp, _i, _l, _l, _i, _vp, _vp, _i]),
    "quantize_headwise_ex": (_i, [_vp, _i, _l, _l, _i, _vp, _vp, _i, _vp]),
    "quantize_qk": (_i, [_vp, _vp, _i, _l, _i, _vp, _vp, _vp, _vp, ctypes.c_float, _i, _vp]),
    "quantize_qkv": (_i, [_vp, _vp, _vp, _i, _l, _l, _i, _vp, _vp, _vp, _vp, _vp, _vp, ctypes.c_float, _vp]),
    "int_flash_attn_fwd": (_i, [_vp] * 6 + [_i] * 5 + [_vp]),
    "int_flash_attn_fwd_ex": (_i, [_vp] * 6 + [_i] * 5 + [_vp, _i, _vp]),
    "int_flash_attn_fwd_rect": (_i, [_vp] * 6 + [_i] * 6 + [_vp, _i, _vp]),
    "ifa_splitk_workspace_bytes": (_l, [_i] * 5),
    "int_flash_attn_fwd_splitk": (_i, [_vp] * 6 + [_i] * 6 + [_vp, _i, _vp, _l, _vp]),
    "ifa_static_workspace_bytes": (_l, []),
    "int_flash_attn_fwd_splitk_static": (_i, [_vp] * 6 + [_i] * 6 + [_vp, _i, _vp]),
    "quantize_blockwise": (_i, [_vp, _i, _l, _l, _i, _i, _vp, _vp, _vp]),
    "int_flash_attn_fwd_vblock": (_i, [_vp] * 6 + [_i] * 5 + [_vp, _i, _vp]),
    "int_flash_attn_fwd_vblock_rect": (_i, [_vp] * 6 + [_i] * 6 + [_vp, _i, _vp]),
    "ifa_block_cols": (_i, [_i, _i]),
    "int_flash_attn_fwd_half": (_i, [_vp] * 5 + [_i] * 5 + [_vp, _i, _vp]),
    "int_flash_attn_fwd_half_rect": (_i, [_vp] * 5 + [_i] * 6 + [_vp, _i, _vp]),
    "ifa_block_cols_half": (_i, [_i, _i]),
    "ifa_debug_fwd": (_i, [_vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _vp, _vp, _vp, _vp, _vp, _vp]),
}


class IntfaError(RuntimeError):
    pass


_lib = None


def lib_path() -> str:
    return _LIB_PATH


def lib():
    """The loaded C library.  Raises if it has not been built (no fallback of any kind)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise IntfaError(f"{_LIB_PATH} is missing: build it with `python -m paper_2409_16997_amd.build` "
                             "or __graft_entry__.build(); there is no CPU fallback")
        handle = ctypes.CDLL(_LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(handle, name)
            fn.restype, fn.argtypes = res, args
        _lib = handle
    return _lib


def status_str(code: int) -> str:
    return lib().ifa_status_str(int(code)).decode()


def _check(code: int, what: str):
    if code != 0:
        raise IntfaError(f"{what}: {status_str(code)} ({code})")


def _dtype_enum(t):
    import torch
    try:
        return {torch.float32: IFA_F32, torch.float16: IFA_F16, torch.bfloat16: IFA_BF16}[t.dtype]
    except KeyError:
        raise IntfaError(f"unsupported dtype {t.dtype}") from None


def _dev(t, dtype=None):
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda or not t.is_contiguous():
        raise IntfaError("expected a contiguous tensor in GPU memory")
    if dtype is not None and t.dtype != dtype:
        raise IntfaError(f"expected dtype {dtype}, got {t.dtype}")
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def quantize_tokenwise(X, scale_mul=1.0, hadamard=False):
    """X [..., d] fp32/fp16/bf16 on the GPU -> (int8 [..., d], fp32 scale [...] times scale_mul).
    hadamard=True quantizes the Walsh-Hadamard transform H_d x of every row instead of x."""
    import torch
    d = X.shape[-1]
    rows = X.numel() // d
    Xq = torch.empty(X.shape, dtype=torch.int8, device=X.device)
    scale = torch.empty(X.shape[:-1], dtype=torch.float32, device=X.device)
    fn = lib().quantize_tokenwise_hadamard if hadamard else lib().quantize_tokenwise_ex
    _check(fn(_dev(X), _dtype_enum(X), rows, d, _dev(Xq), _dev(scale), float(scale_mul), _stream()), "quantize_tokenwise")
    return Xq, scale


def quantize_headwise(X, global_scale=False):
    """X [B, H, N, d] (or [heads, N, d]) -> (int8 same shape, fp32 scale [B, H] (or [heads]))."""
    import torch
    N, d = X.shape[-2], X.shape[-1]
    heads = X.numel() // (N * d)
    Xq = torch.empty(X.shape, dtype=torch.int8, device=X.device)
    scale = torch.empty(X.shape[:-2], dtype=torch.float32, device=X.device)
    _check(lib().quantize_headwise_ex(_dev(X), _dtype_enum(X), heads, N, d, _dev(Xq), _dev(scale), int(bool(global_scale)),
                                      _stream()), "quantize_headwise_ex")
    return Xq, scale


def quantize_qkv(Q, K, V, s_Q_mul=1.0, out=None):
    """The input preparation of one attention call in three launches: Q, K token-level, V tensor-level.
    Q, K, V [B, H, N, d] -> (Q_i8, K_i8, V_i8, s_Q [B, H, N] (times s_Q_mul), s_K [B, H, N], s_V [B, H]);
    out: optional tuple of those six tensors to write into."""
    import torch
    assert Q.shape == K.shape == V.shape and Q.dtype == K.dtype == V.dtype
    N, d = Q.shape[-2], Q.shape[-1]
    heads = Q.numel() // (N * d)
    if out is None:
        q8, k8, v8 = (torch.empty(Q.shape, dtype=torch.int8, device=Q.device) for _ in range(3))
        sq, sk = (torch.empty(Q.shape[:-1], dtype=torch.float32, device=Q.device) for _ in range(2))
        sv = torch.empty(Q.shape[:-2], dtype=torch.float32, device=Q.device)
    else:
        q8, k8, v8, sq, sk, sv = out
    _check(lib().quantize_qkv(_dev(Q), _dev(K), _dev(V), _dtype_enum(Q), heads, N, d, _dev(q8, torch.int8), _dev(k8, torch.int8),
                              _dev(v8, torch.int8), _dev(sq, torch.float32), _dev(sk, torch.float32), _dev(sv, torch.float32),
                              float(s_Q_mul), _stream()), "quantize_qkv")
    return q8, k8, v8, sq, sk, sv


def quantize_qk(Q, K, s_Q_mul=1.0, hadamard=False, out=None):
    """Q and K token-level in one launch.  Q, K [..., d] of one shape -> (Q_i8, K_i8, s_Q [...] (times s_Q_mul), s_K [...]);
    out: optional tuple of those four tensors to write into."""
    import torch
    assert Q.shape == K.shape and Q.dtype == K.dtype
    d = Q.shape[-1]
    rows = Q.numel() // d
    if out is None:
        q8, k8 = (torch.empty(Q.shape, dtype=torch.int8, device=Q.device) for _ in range(2))
        sq, sk = (torch.empty(Q.shape[:-1], dtype=torch.float32, device=Q.device) for _ in range(2))
    else:
        q8, k8, sq, sk = out
    _check(lib().quantize_qk(_dev(Q), _dev(K), _dtype_enum(Q), rows, d, _dev(q8, torch.int8), _dev(k8, torch.int8),
                             _dev(sq, torch.float32), _dev(sk, torch.float32), float(s_Q_mul), int(bool(hadamard)), _stream()),
           "quantize_qk")
    return q8, k8, sq, sk


def quantize_blockwise(X, block_keys):
    """X [B, H, N, d] (or [heads, N, d]) -> (int8 same shape, fp32 scale [B, H, ceil(N/block_keys)])."""
    import torch
    N, d = X.shape[-2], X.shape[-1]
    heads = X.numel() // (N * d)
    Xq = torch.empty(X.shape, dtype=torch.int8, device=X.device)
    scale = torch.empty(tuple(X.shape[:-2]) + (-(-N // block_keys),), dtype=torch.float32, device=X.device)
    _check(lib().quantize_blockwise(_dev(X), _dtype_enum(X), heads, N, d, int(block_keys), _dev(Xq), _dev(scale), _stream()),
           "quantize_blockwise")
    return Xq, scale


def int_flash_attn_fwd(Q_i8, K_i8, V_i8, s_Q, s_K, s_V, causal=False, out_dtype=None, out=None):
    """Algorithm 1 on int8 tensors Q [B, H, Nq, d], K, V [B, H, Nk, d] (Nq = Nk in the paper; under the causal mask
    the queries are the last Nq positions).  Returns O [B, H, Nq, d] (fp16 unless out_dtype/out says otherwise).
    s_V [B, H] is the tensor-level scale of V; a 3-d s_V [B, H, ceil(N/B_c)] selects the per-block V scales."""
    import torch
    B, H, N, d = Q_i8.shape
    Nk = K_i8.shape[2]
    if out is None:
        out = torch.empty((B, H, N, d), dtype=out_dtype or torch.float16, device=Q_i8.device)
    args = (_dev(Q_i8, torch.int8), _dev(K_i8, torch.int8), _dev(V_i8, torch.int8),
            _dev(s_Q, torch.float32), _dev(s_K, torch.float32), _dev(s_V, torch.float32))
    tail = (d, int(bool(causal)), _dev(out), _dtype_enum(out), _stream())
    if K_i8.shape != (B, H, Nk, d) or V_i8.shape != K_i8.shape or s_K.shape != (B, H, Nk) or s_Q.shape != (B, H, N):
        raise IntfaError("Q/K/V/scale shapes do not agree")
    if s_V.dim() == 3:
        if s_V.shape != (B, H, -(-Nk // block_cols(d, causal))):
            raise IntfaError(f"per-block s_V has shape {tuple(s_V.shape)}")
        code = (lib().int_flash_attn_fwd_vblock(*args, B, H, N, *tail) if Nk == N else
                lib().int_flash_attn_fwd_vblock_rect(*args, B, H, N, Nk, *tail))
    elif Nk != N:
        code = lib().int_flash_attn_fwd_rect(*args, B, H, N, Nk, *tail)
    else:
        code = lib().int_flash_attn_fwd_ex(*args, B, H, N, *tail)
    _check(code, "int_flash_attn_fwd")
    return out


def splitk_workspace_bytes(B: int, H: int, Nq: int, Nk: int, d: int) -> int:
    """Bytes of workspace int_flash_attn_fwd_splitk needs for this shape (0: the shape is not one it takes)."""
    return int(lib().ifa_splitk_workspace_bytes(int(B), int(H), int(Nq), int(Nk), int(d)))


def int_flash_attn_fwd_splitk(Q_i8, K_i8, V_i8, s_Q, s_K, s_V, causal=False, out_dtype=None, out=None, workspace=None):
    """Algorithm 1 for at most 32 queries per head against many keys (a decode step, a short chunk), the key axis split over the
    whole chip: same shapes and mask convention as int_flash_attn_fwd.  `workspace`: a uint8 device tensor of at least
    splitk_workspace_bytes(...) bytes (allocated here if not given), or the string "static": the library's built-in
    16 MiB workspace (no allocation at all; calls that overlap on one GPU must not share it)."""
    import torch
    B, H, N, d = Q_i8.shape
    Nk = K_i8.shape[2]
    if K_i8.shape != (B, H, Nk, d) or V_i8.shape != K_i8.shape or s_K.shape != (B, H, Nk) or s_Q.shape != (B, H, N) \
            or s_V.shape != (B, H):
        raise IntfaError("Q/K/V/scale shapes do not agree")
    if out is None:
        out = torch.empty((B, H, N, d), dtype=out_dtype or torch.float16, device=Q_i8.device)
    need = splitk_workspace_bytes(B, H, N, Nk, d)
    if need == 0:
        raise IntfaError("int_flash_attn_fwd_splitk: shape not supported (at most 32 queries per head, d in {64, 128})")
    if isinstance(workspace, str):
        if workspace != "static":
            raise IntfaError("workspace: a uint8 device tensor, None or 'static'")
        code = lib().int_flash_attn_fwd_splitk_static(_dev(Q_i8, torch.int8), _dev(K_i8, torch.int8), _dev(V_i8, torch.int8),
                                                      _dev(s_Q, torch.float32), _dev(s_K, torch.float32), _dev(s_V, torch.float32),
                                                      B, H, N, Nk, d, int(bool(causal)), _dev(out), _dtype_enum(out), _stream())
        _check(code, "int_flash_attn_fwd_splitk_static")
        return out
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=Q_i8.device)
    code = lib().int_flash_attn_fwd_splitk(_dev(Q_i8, torch.int8), _dev(K_i8, torch.int8), _dev(V_i8, torch.int8),
                                           _dev(s_Q, torch.float32), _dev(s_K, torch.float32), _dev(s_V, torch.float32),
                                           B, H, N, Nk, d, int(bool(causal)), _dev(out), _dtype_enum(out),
                                           _dev(workspace, torch.uint8), workspace.numel(), _stream())
    _check(code, "int_flash_attn_fwd_splitk")
    return out


def block_cols(d: int, causal: bool) -> int:
    return lib().ifa_block_cols(int(d), int(bool(causal)))


def int_flash_attn_fwd_half(Q_i8, K_i8, V_f16, s_Q, s_K, causal=False, out_dtype=None, out=None):
    """Half-INT8 variant: int8 Q [B, H, Nq, d], K [B, H, Nk, d] with token-level scales, fp16 V [B, H, Nk, d] as is
    (Nq = Nk in the paper; under the mask the queries are the last Nq positions).  Returns O [B, H, Nq, d]."""
    import torch
    B, H, N, d = Q_i8.shape
    if out is None:
        out = torch.empty((B, H, N, d), dtype=out_dtype or torch.float16, device=Q_i8.device)
    Nk = K_i8.shape[2]
    if K_i8.shape != (B, H, Nk, d) or V_f16.shape != K_i8.shape or s_K.shape != (B, H, Nk) or s_Q.shape != (B, H, N):
        raise IntfaError("Q/K/V/scale shapes do not agree")
    code = lib().int_flash_attn_fwd_half_rect(_dev(Q_i8, torch.int8), _dev(K_i8, torch.int8), _dev(V_f16, torch.float16),
                                              _dev(s_Q, torch.float32), _dev(s_K, torch.float32),
                                              B, H, N, Nk, d, int(bool(causal)), _dev(out), _dtype_enum(out), _stream())
    _check(code, "int_flash_attn_fwd_half")
    return out


def block_cols_half(d: int, causal: bool) -> int:
    return lib().ifa_block_cols_half(int(d), int(bool(causal)))


def debug_fwd(Q_i8, K_i8, V_i8, s_Q, s_K, s_V, causal=False, P_in=None, fill=-1):
    """One head [N, d] through the production kernel with its integer stages written out.  Returns a dict with
    S [N, N] int32, P [N, N] int8, PV [N / B_c, N, d] int32 and O [N, d] fp32; entries the kernel does not compute
    (key tiles and blocks wholly above the causal diagonal) keep the value `fill`."""
    import torch
    N, d = Q_i8.shape
    Bc = block_cols(d, causal)
    dev = Q_i8.device
    S = torch.full((N, N), fill, dtype=torch.int32, device=dev)
    P = torch.full((N, N), fill, dtype=torch.int8, device=dev)
    PV = torch.full((max(N // max(Bc, 1), 1), N, d), fill, dtype=torch.int32, device=dev)
    O = torch.empty((N, d), dtype=torch.float32, device=dev)
    _check(lib().ifa_debug_fwd(_dev(Q_i8, torch.int8), _dev(K_i8, torch.int8), _dev(V_i8, torch.int8), _dev(s_Q, torch.float32),
                               _dev(s_K, torch.float32), _dev(s_V, torch.float32), N, d, int(bool(causal)),
                               None if P_in is None else _dev(P_in, torch.int8), _dev(S), _dev(P), _dev(PV), _dev(O), _stream()),
           "ifa_debug_fwd")
    return {"S": S, "P": P, "PV": PV, "O": O}
