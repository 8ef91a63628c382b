"""CPU-side checks of the boundary: the library loads, exports every symbol include/intfa.h declares,
and rejects bad arguments on the host before any launch (no GPU needed: validation comes first)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    import paper_2409_16997_amd as ifa
    if not os.path.exists(ifa.lib_path()):
        from paper_2409_16997_amd import build
        build.build()
    return ifa.lib()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "intfa.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(?:int|long|const char \*)\s*\*?\s*(\w+)\s*\(", text)))


def test_header_declares_the_north_star_calls():
    names = declared_symbols()
    for must in ("quantize_tokenwise", "quantize_headwise", "int_flash_attn_fwd", "int_flash_attn_fwd_ex",
                 "quantize_tokenwise_ex", "quantize_headwise_ex", "quantize_qk", "quantize_qkv", "quantize_tokenwise_hadamard", "quantize_blockwise", "int_flash_attn_fwd_vblock", "int_flash_attn_fwd_vblock_rect", "int_flash_attn_fwd_half", "int_flash_attn_fwd_half_rect", "ifa_block_cols_half", "int_flash_attn_fwd_rect", "int_flash_attn_fwd_splitk", "ifa_splitk_workspace_bytes", "ifa_block_cols", "ifa_debug_fwd", "ifa_set_stream", "ifa_status_str"):
        assert must in names


def test_library_exports_every_declared_symbol(L):
    from paper_2409_16997_amd.binding import SIGNATURES
    names = declared_symbols()
    assert sorted(SIGNATURES) == names
    for n in names:
        assert getattr(L, n) is not None


def test_status_strings(L):
    assert L.ifa_status_str(0) == b"IFA_OK"
    for c in (-1, -2, -3, -4, -5, -6):
        assert L.ifa_status_str(c).startswith(b"IFA_ERR_")
    assert L.ifa_status_str(7) == b"unknown ifa_status"


def test_block_cols(L):
    assert L.ifa_block_cols(128, 1) == 128 and L.ifa_block_cols(64, 0) == 128
    assert L.ifa_block_cols(96, 0) == 0
    assert L.ifa_block_cols_half(128, 1) == 64 and L.ifa_block_cols_half(64, 0) == 64
    assert L.ifa_block_cols_half(32, 0) == 0


def test_argument_validation_happens_on_the_host(L):
    p = ctypes.c_void_p(0x1000)            # non-null, 16-byte aligned, never dereferenced by validation
    null = ctypes.c_void_p(0)
    odd = ctypes.c_void_p(0x1004)
    f = L.int_flash_attn_fwd_ex
    ok_tail = (p, 1, None)
    assert f(null, p, p, p, p, p, 1, 1, 128, 128, 0, *ok_tail) == -1
    assert f(p, p, p, p, p, p, 1, 1, 128, 128, 0, null, 1, None) == -1
    assert f(p, p, p, p, p, p, 0, 1, 128, 128, 0, *ok_tail) == -2
    assert f(p, p, p, p, p, p, 1, 1, -128, 128, 0, *ok_tail) == -2
    assert f(p, p, p, p, p, p, 1, 1, 128, 128, 0, p, 9, None) == -3
    assert f(p, p, p, p, p, p, 1, 1, 128, 96, 0, *ok_tail) == -4      # head dim not built
    assert f(p, p, p, p, p, p, 1, 1, 1 << 30, 128, 0, *ok_tail) == -4  # one head must stay below 2 GiB
    assert f(odd, p, p, p, p, p, 1, 1, 128, 128, 0, *ok_tail) == -4   # misaligned
    assert f(p, p, p, p, p, p, 1, 1, 0x7ff00000 // 128 + 1, 128, 0, *ok_tail) == -4   # first N past the per-head limit
    assert L.int_flash_attn_fwd(null, p, p, p, p, p, 1, 1, 128, 128, 0, p) == -1
    q = L.quantize_tokenwise
    assert q(null, 1, 10, 128, p, p) == -1
    assert q(p, 1, 0, 128, p, p) == -2
    assert q(p, 5, 10, 128, p, p) == -3
    assert q(p, 1, 10, 100, p, p) == -4
    qx = L.quantize_tokenwise_ex
    assert qx(p, 1, 10, 128, p, p, 0.0, None) == -2 and qx(p, 1, 10, 128, p, p, float("nan"), None) == -2
    assert qx(p, 1, 10, 128, null, p, 1.0, None) == -1
    qk = L.quantize_qk
    assert qk(p, null, 1, 10, 128, p, p, p, p, 1.0, 0, None) == -1 and qk(p, p, 1, 10, 128, p, p, p, null, 1.0, 1, None) == -1
    assert qk(p, p, 1, 0, 128, p, p, p, p, 1.0, 0, None) == -2 and qk(p, p, 1, 10, 128, p, p, p, p, -1.0, 0, None) == -2
    assert qk(p, p, 4, 10, 128, p, p, p, p, 1.0, 0, None) == -3 and qk(p, odd, 1, 10, 128, p, p, p, p, 1.0, 0, None) == -4
    h = L.quantize_headwise
    assert h(p, 1, 4, 128, 64, p, null, 0) == -1
    assert h(p, 1, 0, 128, 64, p, p, 0) == -2
    assert h(p, 3, 4, 128, 64, p, p, 0) == -3
    assert h(p, 1, 4, 3, 3, p, p, 0) == -4
    b = L.quantize_blockwise
    assert b(p, 1, 4, 256, 128, 128, p, null, None) == -1 and b(p, 1, 4, 256, 128, 0, p, p, None) == -2
    assert b(p, 7, 4, 256, 128, 128, p, p, None) == -3 and b(p, 1, 4, 256, 128, 256, p, p, None) == -4
    assert L.int_flash_attn_fwd_vblock(p, p, p, p, p, null, 1, 1, 128, 128, 0, p, 1, None) == -1
    assert L.int_flash_attn_fwd_vblock(p, p, p, p, p, p, 1, 1, 128, 96, 0, p, 1, None) == -4
    vr = L.int_flash_attn_fwd_vblock_rect
    assert vr(p, p, p, p, p, p, 1, 1, 256, 64, 128, 1, p, 1, None) == -4 and vr(p, p, p, p, p, null, 1, 1, 8, 64, 128, 0, p, 1, None) == -1
    rc = L.int_flash_attn_fwd_rect
    assert rc(p, p, p, p, p, p, 1, 1, 256, 64, 128, 1, p, 1, None) == -4             # causal with Nk < Nq
    assert rc(p, p, p, p, p, p, 1, 1, 0, 64, 128, 0, p, 1, None) == -2 and rc(p, p, p, p, p, null, 1, 1, 8, 64, 128, 0, p, 1, None) == -1
    sk, wb = L.int_flash_attn_fwd_splitk, L.ifa_splitk_workspace_bytes
    ws = ctypes.c_void_p(0x10000)
    assert wb(1, 8, 1, 16384, 128) > 4 * 8 * 16384 and wb(1, 8, 33, 16384, 128) == 0 and 0 < wb(1, 8, 32, 16384, 128) < wb(1, 8, 8, 16384, 128) + (16 << 20) and wb(1, 8, 1, 16384, 96) == 0
    need = wb(1, 8, 4, 1000, 128)
    assert sk(p, p, p, p, p, p, 1, 8, 33, 1000, 128, 0, p, 1, ws, 1 << 30, None) == -4      # more than 32 queries
    assert sk(p, p, p, p, p, p, 1, 8, 4, 1000, 128, 0, p, 1, null, need, None) == -1
    assert sk(p, p, p, p, p, p, 1, 8, 4, 1000, 128, 0, p, 1, ws, need - 1, None) == -6       # workspace too small
    assert sk(p, p, p, p, p, p, 1, 8, 4, 1000, 128, 0, p, 1, odd, need, None) == -4          # workspace not 256-byte aligned
    assert sk(p, p, p, p, p, p, 1, 8, 4, 2, 128, 1, p, 1, ws, need, None) == -4              # causal with Nk < Nq
    assert sk(p, p, p, p, p, p, 1, 8, 4, 1000, 128, 0, p, 5, ws, need, None) == -3
    assert L.ifa_static_workspace_bytes() == 16 << 20                                         # also without a GPU: the set-up part is skipped
    assert L.int_flash_attn_fwd_splitk_static(p, p, p, p, p, p, 4, 32, 8, 16384, 128, 1, p, 1, None) == -6   # 86 MB needed
    hf = L.int_flash_attn_fwd_half
    assert hf(p, p, null, p, p, 1, 1, 128, 128, 0, p, 1, None) == -1 and hf(p, p, p, p, p, 1, 0, 128, 128, 0, p, 1, None) == -2
    assert hf(p, p, p, p, p, 1, 1, 128, 128, 0, p, -1, None) == -3 and hf(p, p, p, p, p, 1, 1, 128, 256, 0, p, 1, None) == -4
    assert hf(p, p, p, p, p, 1, 1, 1 << 29, 128, 0, p, 1, None) == -4   # one head of fp16 V must stay below 2 GiB
    assert hf(p, p, p, p, p, 1, 1, 0x7ff00000 // 256 + 1, 128, 0, p, 1, None) == -4   # first N past that limit
    assert L.int_flash_attn_fwd_half_rect(p, p, p, p, p, 1, 1, 256, 64, 128, 1, p, 1, None) == -4   # causal with Nk < Nq
    assert L.ifa_debug_fwd(p, p, p, p, p, p, 100, 128, 0, null, p, p, p, p, null) == -4
    assert L.ifa_debug_fwd(p, null, p, p, p, p, 128, 128, 0, null, p, p, p, p, null) == -1


def test_bench_refuses_more_than_one_gpu():
    # the build is single-GPU by design: bench.py says so instead of running
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "ONE GPU" in r.stderr
