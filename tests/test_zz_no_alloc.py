"""The key-split entry point that allocates nothing (its workspace is an array in the library's device image),
called through the C ABI and compared with the entry point it is a variant of, which takes the caller's workspace:
same kernels on the same inputs, so the outputs must be equal bit for bit -- on two calls in a row, the second
with a smaller input (the array keeps the first call's contents)."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from helpers import random_int8_problem

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def L():
    import paper_2409_16997_amd as ifa
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    return ifa.lib()


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr())


def _case(L, H, Nq, Nk, d, causal, seed):
    rng = np.random.default_rng(seed)
    Qq, Kq, Vq, sQ, sK, sV = random_int8_problem(rng, H, max(Nq, Nk), d, score_sigma=2.0)
    Qq, sQ = np.ascontiguousarray(Qq[:, :Nq]), np.ascontiguousarray(sQ[:, :Nq])
    Kq, Vq, sK = np.ascontiguousarray(Kq[:, :Nk]), np.ascontiguousarray(Vq[:, :Nk]), np.ascontiguousarray(sK[:, :Nk])
    t = [torch.from_numpy(x).cuda() for x in (Qq, Kq, Vq, sQ, sK, sV)]
    need = L.ifa_splitk_workspace_bytes(1, H, Nq, Nk, d)
    assert 0 < need <= L.ifa_static_workspace_bytes()
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    guard = 32
    ref = torch.full((H * Nq + guard, d), 777.0, dtype=torch.float32, device="cuda")
    got = torch.full((H * Nq + guard, d), 777.0, dtype=torch.float32, device="cuda")
    st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    rc = L.int_flash_attn_fwd_splitk(*map(_ptr, t), 1, H, Nq, Nk, d, causal, _ptr(ref), 0, _ptr(ws), need, st)
    assert rc == 0
    rc = L.int_flash_attn_fwd_splitk_static(*map(_ptr, t), 1, H, Nq, Nk, d, causal, _ptr(got), 0, st)
    assert rc == 0
    torch.cuda.synchronize()
    assert torch.equal(got, ref), (H, Nq, Nk, d, causal)
    assert bool((got[H * Nq:] == 777.0).all())
    # and the result is Algorithm 1: the strict parity bar against the oracle
    res = oracle.compare_up_to_ties(got[:H * Nq].cpu().numpy(), Qq, Kq, Vq, sQ, sK, sV, bool(causal), L.ifa_block_cols(d, causal))
    assert np.all(res["err"] <= 1e-3 * res["scale"])


def test_static_workspace_entry_point_equals_the_caller_workspace_one(L):
    _case(L, 8, 3, 9000, 128, 1, seed=1)          # first call: 71 key blocks per head
    _case(L, 5, 1, 700, 64, 0, seed=2)            # second call, smaller: the array still holds the first call's words
    _case(L, 8, 3, 9000, 128, 1, seed=1)
    _case(L, 4, 20, 5000, 128, 1, seed=3)         # 9 .. 32 queries: the second pass recomputes the scores


def test_static_workspace_entry_point_refuses_what_does_not_fit(L):
    p = ctypes.c_void_p(0x1000)
    B, H, Nq, Nk, d = 4, 32, 8, 16384, 128         # 86 MB of workspace
    assert L.ifa_splitk_workspace_bytes(B, H, Nq, Nk, d) > L.ifa_static_workspace_bytes()
    assert L.int_flash_attn_fwd_splitk_static(p, p, p, p, p, p, B, H, Nq, Nk, d, 1, p, 1, None) == -6
    assert L.ifa_status_str(-6).startswith(b"IFA_ERR_WORKSPACE")
    assert L.int_flash_attn_fwd_splitk_static(p, p, p, p, p, p, 1, 8, 33, 1000, d, 0, p, 1, None) == -4
