"""Pins for the oracle's attention functions against what the paper and the mathematics fix:
Section 2.1 (standard attention), Section 3.1 (online softmax equals standard softmax),
Algorithm 1 and Section 3.2 (INT8 P with S_P = 1/R cancelling in diag(l)^-1)."""
import itertools
import math

import numpy as np
import pytest
import scipy.special

import oracle
from helpers import dequant, random_int8_problem


# ---------------------------------------------------------------- integer GEMMs (exact)

@pytest.mark.parametrize("N,d", [(96, 64), (128, 128)])
def test_int32_gemms_match_int64_numpy(N, d):
    rng = np.random.default_rng(10)
    Q = rng.integers(-128, 128, (N, d), dtype=np.int8)
    K = rng.integers(-128, 128, (N, d), dtype=np.int8)
    V = rng.integers(-128, 128, (N, d), dtype=np.int8)
    P = rng.integers(0, 128, (N, N), dtype=np.int8)
    S = oracle.qk_i32(Q, K)
    assert np.array_equal(S.astype(np.int64), Q.astype(np.int64) @ K.astype(np.int64).T)
    assert np.abs(S).max() <= 128 * 128 * d
    PV = oracle.pv_i32(P, V)
    assert np.array_equal(PV.astype(np.int64), P.astype(np.int64) @ V.astype(np.int64))
    # a transposed operand would pass a symmetric input only; use an asymmetric one
    e = np.zeros((N, d), np.int8); e[3, 5] = 7
    f = np.zeros((N, d), np.int8); f[9, 5] = 11
    assert oracle.qk_i32(e, f)[3, 9] == 77 and oracle.qk_i32(e, f).sum() == 77


# ---------------------------------------------------------------- fp64 brute force == library softmax

@pytest.mark.parametrize("causal", [False, True])
def test_fp64_attention_matches_scipy_softmax(causal):
    rng = np.random.default_rng(11)
    Q, K, V = (rng.standard_normal((3, 40, 16)) for _ in range(3))
    O = oracle.attention_fp64(Q, K, V, causal=causal, scale=0.25).reshape(3, 40, 16)
    S = 0.25 * np.einsum("hik,hjk->hij", Q, K)
    if causal:
        S = np.where(np.tril(np.ones((40, 40), bool)), S, -np.inf)
    ref = np.einsum("hij,hjc->hic", scipy.special.softmax(S, axis=-1), V)
    assert np.allclose(O, ref, rtol=1e-12, atol=1e-13)
    rows = np.array([5, 41, 119], np.int64)
    assert np.array_equal(oracle.attention_fp64(Q, K, V, causal=causal, scale=0.25, row_idx=rows),
                          O.reshape(-1, 16)[rows])


# ---------------------------------------------------------------- Section 3.1: online == standard

@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("N,Bc", [(64, 16), (100, 32), (128, 128), (130, 64)])
def test_online_softmax_without_p_quant_equals_standard_attention(N, Bc, causal):
    rng = np.random.default_rng(12)
    Qq, Kq, Vq, sQ, sK, sV = random_int8_problem(rng, 2, N, 32, score_sigma=2.0)
    got = oracle.int_flash_attn_fwd(Qq, Kq, Vq, sQ, sK, sV, causal, Bc, p_quant=False)
    ref = oracle.attention_fp64(dequant(Qq, sQ), dequant(Kq, sK),
                                Vq.astype(np.float64) * sV[:, None, None].astype(np.float64), causal=causal)
    assert np.abs(got["O"] - ref).max() <= 1e-5 * np.abs(ref).max()
    # l is the softmax denominator on the grid of the final max: sum_j exp(S_j - m)
    S = np.einsum("hik,hjk->hij", dequant(Qq, sQ), dequant(Kq, sK))
    if causal:
        S = np.where(np.tril(np.ones((N, N), bool)), S, -np.inf)
    assert np.allclose(got["m"], S.max(-1).reshape(-1), rtol=1e-6)
    assert np.allclose(got["l"], np.exp(S - S.max(-1, keepdims=True)).sum(-1).reshape(-1), rtol=1e-5)


# ---------------------------------------------------------------- Algorithm 1, single block: closed form

@pytest.mark.parametrize("causal", [False, True])
def test_single_block_closed_form(causal):
    # With Bc = N there is one inner iteration: P = rint(127 exp(S - rowmax S)),
    # O = s_V (P V) / rowsum(P)   (Section 3.2, first block of the two-block derivation).
    rng = np.random.default_rng(13)
    N, d = 48, 32
    Qq, Kq, Vq, sQ, sK, sV = random_int8_problem(rng, 1, N, d, score_sigma=1.5)
    out = oracle.int_flash_attn_fwd(Qq, Kq, Vq, sQ, sK, sV, causal, N, want_P=True)
    acc = Qq[0].astype(np.int64) @ Kq[0].astype(np.int64).T
    S = (acc.astype(np.float32) * sQ[0][:, None]) * sK[0][None, :]
    if causal:
        S = np.where(np.tril(np.ones((N, N), bool)), S, -np.inf)
    t = (S - S.max(-1, keepdims=True)).astype(np.float32)
    P = np.rint(127.0 * np.exp(t.astype(np.float64))).astype(np.int64)
    assert np.array_equal(out["P"].astype(np.int64), P)
    O = (P @ Vq[0].astype(np.int64)).astype(np.float64) / P.sum(-1, keepdims=True) * float(sV[0])
    assert np.allclose(out["O"], O, rtol=3e-7, atol=0)
    assert np.array_equal(out["l"], P.sum(-1).astype(np.float32))
    # range invariant (P~ in (0,1], P in I_8) and the maximum is attained
    assert out["P"].min() >= 0 and np.all(out["P"].max(-1) == 127)


def test_p_range_and_row_max_with_many_blocks():
    rng = np.random.default_rng(14)
    N, Bc = 96, 16
    Qq, Kq, Vq, sQ, sK, sV = random_int8_problem(rng, 2, N, 64, score_sigma=3.0)
    out = oracle.int_flash_attn_fwd(Qq, Kq, Vq, sQ, sK, sV, False, Bc, want_P=True)
    P = out["P"].reshape(2, N, N)
    assert P.min() >= 0 and P.max() <= 127
    S = np.einsum("hik,hjk->hij", dequant(Qq, sQ), dequant(Kq, sK))
    jstar = S.argmax(-1)                       # the block holding the running max has a 127 there
    assert np.all(np.take_along_axis(P, jstar[..., None], -1) == 127)
    # keys in blocks before the arg-max block are rounded on an earlier (smaller) max: P there is
    # not determined by the final max, which is exactly the B_c dependence of Algorithm 1.


# ---------------------------------------------------------------- closed forms

@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("Bc", [8, 32])
def test_uniform_scores_give_the_mean_of_v(causal, Bc):
    # Q = 0 => S = 0 => every P = 127 => O[i] = mean of V^ (prefix mean under the causal mask).
    rng = np.random.default_rng(15)
    N, d = 64, 16
    _, Kq, Vq, sQ, sK, sV = random_int8_problem(rng, 1, N, d)
    Qq = np.zeros((1, N, d), np.int8)
    out = oracle.int_flash_attn_fwd(Qq, Kq, Vq, sQ, sK, sV, causal, Bc, want_P=True)
    Vh = Vq[0].astype(np.float64) * float(sV[0])
    if causal:
        ref = np.cumsum(Vh, 0) / np.arange(1, N + 1)[:, None]
        assert np.array_equal(out["P"], 127 * np.tril(np.ones((N, N), np.int8)))
        assert np.array_equal(out["l"], 127.0 * np.arange(1, N + 1, dtype=np.float32))
    else:
        ref = np.broadcast_to(Vh.mean(0), (N, d))
        assert np.all(out["P"] == 127)
        assert np.all(out["l"] == 127.0 * N)
    assert np.allclose(out["O"], ref, rtol=1e-6, atol=1e-9)


def test_one_hot_row_returns_that_value_row():
    # One key in block 0 whose score is > 6 above all others: 127 exp(-6) < 1/2 so every other
    # P is 0 and O[i] = V^[j*] exactly.
    N, d, Bc = 32, 16, 8
    rng = np.random.default_rng(16)
    Vq = rng.integers(-127, 128, (1, N, d), dtype=np.int8)
    Qq = np.zeros((1, N, d), np.int8); Qq[0, :, 0] = 100
    Kq = np.zeros((1, N, d), np.int8); Kq[0, 3, 0] = 100          # key 3 is in block 0
    sQ = np.full((1, N), 0.03, np.float32)
    sK = np.full((1, N), 0.03, np.float32)                       # S = 9 at key 3, 0 elsewhere
    sV = np.array([0.5], np.float32)
    out = oracle.int_flash_attn_fwd(Qq, Kq, Vq, sQ, sK, sV, False, Bc, want_P=True)
    assert np.array_equal(out["P"][:, 3], np.full(N, 127, np.int8)) and out["P"].sum() == 127 * N
    assert np.array_equal(out["O"], np.broadcast_to(Vq[0, 3].astype(np.float32) * 0.5, (N, d)))
    assert np.all(out["l"] == 127.0)


def test_two_block_worked_example():
    # Hand evaluation of the two-block derivation in Section 3.2 with d = 1, B_c = 1.
    # Scores (0, -1): m stays 0, alpha = 1, P = (127, rint(127/e) = 47), l = 174.
    # Scores (-1, 0): block 1 is rounded on the grid of m = -1 (P = 127), then rescaled by
    # alpha = 1/e when the max moves to 0: l = 127/e + 127, O~ = (127/e) V0 + 127 V1.
    V = np.array([[[100], [-50]]], np.int8)
    sV = np.array([0.01], np.float32)
    one = np.ones((1, 1), np.float32)
    Kq = np.array([[[0], [100]]], np.int8)
    Qq = np.array([[[-100]]], np.int8)            # acc = (0, -10000); s_Q s_K = 1e-4 -> S = (0, -1)
    out = oracle.int_flash_attn_fwd(np.repeat(Qq, 2, 1), Kq, V, np.full((1, 2), 1e-2, np.float32),
                                    np.full((1, 2), 1e-2, np.float32), sV, False, 1, want_P=True)
    assert out["P"][0].tolist() == [127, 47] and out["l"][0] == 174.0
    assert math.isclose(out["O"][0, 0], (127 * 100 - 47 * 50) / 174 * 0.01, rel_tol=1e-6)
    Kq2 = np.array([[[100], [0]]], np.int8)       # S = (-1, 0)
    out = oracle.int_flash_attn_fwd(np.repeat(Qq, 2, 1), Kq2, V, np.full((1, 2), 1e-2, np.float32),
                                    np.full((1, 2), 1e-2, np.float32), sV, False, 1, want_P=True)
    a = math.exp(-1.0)
    assert out["P"][0].tolist() == [127, 127]
    assert math.isclose(out["l"][0], 127 * a + 127, rel_tol=1e-6)
    assert math.isclose(out["O"][0, 0], (127 * a * 100 - 127 * 50) / (127 * a + 127) * 0.01, rel_tol=1e-5)
    # with one block of two keys the same scores round on the final grid instead: P = (47, 127)
    out = oracle.int_flash_attn_fwd(np.repeat(Qq, 2, 1), Kq2, V, np.full((1, 2), 1e-2, np.float32),
                                    np.full((1, 2), 1e-2, np.float32), sV, False, 2, want_P=True)
    assert out["P"][0].tolist() == [47, 127] and out["l"][0] == 174.0
    del one


# ---------------------------------------------------------------- causal mask (extension)

def test_causal_properties():
    rng = np.random.default_rng(17)
    N, d, Bc = 64, 32, 16
    Qq, Kq, Vq, sQ, sK, sV = random_int8_problem(rng, 2, N, d, score_sigma=2.0)
    out = oracle.int_flash_attn_fwd(Qq, Kq, Vq, sQ, sK, sV, True, Bc)
    O = out["O"].reshape(2, N, d)
    # row 0 attends to key 0 only
    assert np.array_equal(O[:, 0], Vq[:, 0].astype(np.float32) * sV[:, None])
    # changing K, V rows after i leaves O[i] bit-identical
    K2, V2 = Kq.copy(), Vq.copy()
    K2[:, 40:] = rng.integers(-127, 128, K2[:, 40:].shape, dtype=np.int8)
    V2[:, 40:] = rng.integers(-127, 128, V2[:, 40:].shape, dtype=np.int8)
    O2 = oracle.int_flash_attn_fwd(Qq, K2, V2, sQ, sK, sV, True, Bc)["O"].reshape(2, N, d)
    assert np.array_equal(O[:, :40], O2[:, :40]) and not np.array_equal(O[:, 40:], O2[:, 40:])
    # row i under the mask == last row of the unmasked problem on the prefix of length i+1
    for i in (15, 31, 47):                          # (i+1) % Bc == 0: same block boundaries
        n = i + 1
        pre = oracle.int_flash_attn_fwd(Qq[:, :n], Kq[:, :n], Vq[:, :n], sQ[:, :n], sK[:, :n], sV,
                                        False, Bc)["O"].reshape(2, n, d)
        assert np.array_equal(pre[:, i], O[:, i])


# ---------------------------------------------------------------- linearity of the scales (Section 3.2)

def test_scale_linearity():
    rng = np.random.default_rng(18)
    N, d, Bc = 64, 32, 16
    Qq, Kq, Vq, sQ, sK, sV = random_int8_problem(rng, 1, N, d, score_sigma=1.0)
    base = oracle.int_flash_attn_fwd(Qq, Kq, Vq, sQ, sK, sV, False, Bc)
    # s_V -> 4 s_V scales O by exactly 4 (power of two)
    o4 = oracle.int_flash_attn_fwd(Qq, Kq, Vq, sQ, sK, sV * 4, False, Bc)["O"]
    assert np.array_equal(o4, base["O"] * 4)
    # moving a power-of-two factor from s_Q to s_K changes nothing at all
    o2 = oracle.int_flash_attn_fwd(Qq, Kq, Vq, sQ * 8, sK / 8, sV, False, Bc)["O"]
    assert np.array_equal(o2, base["O"])
    # a general factor changes S only by fp32 rounding: P may move by one step at near-ties
    o3 = oracle.int_flash_attn_fwd(Qq, Kq, Vq, sQ * np.float32(1.7), sK / np.float32(1.7), sV, False, Bc)["O"]
    assert np.abs(o3 - base["O"]).max() <= 2e-3 * np.abs(base["O"]).max()


# ---------------------------------------------------------------- P rounding: error bound

@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("sigma", [0.5, 3.0])
def test_p_rounding_error_bound(causal, sigma):
    # Effective weight of key j: w_j = P_j exp(m^(jb) - m_final) = 127 p~_j + eps_j, |eps_j| <= 1/2,
    # and sum_j p~_j (v_j - O*) = 0, hence |O - O*| <= (1/2) sum_j |v_j - O*| / sum_j w_j = ... / l.
    rng = np.random.default_rng(19)
    N, d = 96, 16
    Qq, Kq, Vq, sQ, sK, sV = random_int8_problem(rng, 2, N, d, score_sigma=sigma)
    ref = oracle.attention_fp64(dequant(Qq, sQ), dequant(Kq, sK),
                                Vq.astype(np.float64) * sV[:, None, None].astype(np.float64),
                                causal=causal).reshape(2, N, d)
    Vh = Vq.astype(np.float64) * sV[:, None, None].astype(np.float64)
    mask = np.tril(np.ones((N, N), bool)) if causal else np.ones((N, N), bool)
    dev = np.abs(Vh[:, None, :, :] - ref[:, :, None, :]) * mask[None, :, :, None]   # [h, i, j, c]
    outs = {}
    for Bc in (16, 32, 96):
        out = oracle.int_flash_attn_fwd(Qq, Kq, Vq, sQ, sK, sV, causal, Bc)
        bound = 0.5 * dev.sum(2) / out["l"].reshape(2, N, 1)
        err = np.abs(out["O"].reshape(2, N, d) - ref)
        assert np.all(err <= bound * (1 + 1e-4) + 1e-6 * np.abs(ref).max())
        outs[Bc] = out["O"]
    # the result depends on B_c (different rounding grids) but only at the rounding-noise level
    assert not np.array_equal(outs[16], outs[96])


def test_l_is_R_times_the_float_denominator():
    # Section 3.2: l^(2) = R x l, so O needs no explicit S_P: l / 127 ~ sum_j exp(S_j - m).
    rng = np.random.default_rng(20)
    N = 128
    Qq, Kq, Vq, sQ, sK, sV = random_int8_problem(rng, 1, N, 32, score_sigma=1.0)
    a = oracle.int_flash_attn_fwd(Qq, Kq, Vq, sQ, sK, sV, False, 32)
    b = oracle.int_flash_attn_fwd(Qq, Kq, Vq, sQ, sK, sV, False, 32, p_quant=False)
    assert np.array_equal(a["m"], b["m"])
    assert np.all(np.abs(a["l"] / 127.0 - b["l"]) <= 0.5 * N / 127.0)


def test_tie_counter_flags_exact_half():
    # 127 exp(t) within the stated relative window of k + 1/2 is flagged; others are not.
    V = np.array([[[1], [1]]], np.int8)
    sV = np.ones(1, np.float32)
    Qq = np.array([[[100], [100]]], np.int8)
    Kq = np.array([[[0], [-100]]], np.int8)
    t = np.float32(math.log(46.5 / 127.0))            # 127 exp(t) ~ 46.5
    s = np.float32(math.sqrt(-float(t) / 10000.0))
    out = oracle.int_flash_attn_fwd(Qq, Kq, V, np.full((1, 2), s, np.float32), np.full((1, 2), s, np.float32),
                                    sV, False, 2, tie_rel=0.0, tie_abs=1e-5)
    assert out["n_tie"].tolist() == [1, 1]
    out = oracle.int_flash_attn_fwd(Qq, Kq, V, np.full((1, 2), s, np.float32), np.full((1, 2), s, np.float32),
                                    sV, False, 2, tie_rel=0.0, tie_abs=1e-9)
    assert out["n_tie"].tolist() == [0, 0]


def test_row_subset_equals_full():
    rng = np.random.default_rng(21)
    Qq, Kq, Vq, sQ, sK, sV = random_int8_problem(rng, 3, 64, 32)
    full = oracle.int_flash_attn_fwd(Qq, Kq, Vq, sQ, sK, sV, True, 16)
    rows = np.array([0, 63, 64, 100, 191], np.int64)
    sub = oracle.int_flash_attn_fwd(Qq, Kq, Vq, sQ, sK, sV, True, 16, row_idx=rows)
    assert np.array_equal(sub["O"], full["O"][rows]) and np.array_equal(sub["l"], full["l"][rows])


# ---------------------------------------------------------------- per-block V scales (the paper's stated future work)

def test_blockwise_v_quantizer():
    rng = np.random.default_rng(30)
    V = rng.standard_normal((3, 200, 16)).astype(np.float32)
    V[1, 64:128] *= 50.0                                  # one loud block
    q, s = oracle.quantize_blockwise(V, 64)
    assert q.shape == V.shape and s.shape == (3, 4)
    for h in range(3):
        for jb in range(4):
            blk = V[h, 64 * jb:64 * (jb + 1)]
            assert s[h, jb] == np.abs(blk).max() / np.float32(127.0)
            qb = q[h, 64 * jb:64 * (jb + 1)]
            assert np.abs(qb).max() == 127
            assert np.abs(blk - qb.astype(np.float64) * float(s[h, jb])).max() <= 0.5 * s[h, jb] * (1 + 1e-5)
    # a loud block no longer costs the quiet blocks their resolution
    qh, sh = oracle.quantize_headwise(V)
    quiet = slice(128, 200)
    err_block = np.abs(V[1, quiet] - q[1, quiet] * s[1, 2:4].repeat([64, 8])[:, None]).max()
    err_head = np.abs(V[1, quiet] - qh[1, quiet] * sh[1]).max()
    assert err_block < 0.1 * err_head


@pytest.mark.parametrize("causal", [False, True])
def test_blockwise_v_reduces_to_tensor_level_when_scales_are_equal(causal):
    rng = np.random.default_rng(31)
    N, d, Bc = 96, 16, 32
    Qq, Kq, Vq, sQ, sK, sV = random_int8_problem(rng, 2, N, d, score_sigma=1.5)
    a = oracle.int_flash_attn_fwd(Qq, Kq, Vq, sQ, sK, sV, causal, Bc)
    b = oracle.int_flash_attn_fwd(Qq, Kq, Vq, sQ, sK, np.repeat(sV[:, None], 3, 1), causal, Bc)
    assert np.array_equal(a["l"], b["l"]) and np.array_equal(a["m"], b["m"])
    assert np.allclose(a["O"], b["O"], rtol=2e-6, atol=1e-7 * np.abs(a["O"]).max())
    # power-of-two scales commute exactly with every fp32 rounding
    a = oracle.int_flash_attn_fwd(Qq, Kq, Vq, sQ, sK, np.full(2, 0.25, np.float32), causal, Bc)
    b = oracle.int_flash_attn_fwd(Qq, Kq, Vq, sQ, sK, np.full((2, 3), 0.25, np.float32), causal, Bc)
    assert np.array_equal(a["O"], b["O"])


@pytest.mark.parametrize("causal", [False, True])
def test_blockwise_v_closed_forms_and_error_bound(causal):
    rng = np.random.default_rng(32)
    N, d, Bc = 80, 16, 32                                 # ragged: blocks of 32, 32, 16 keys
    Qq, Kq, Vq, sQ, sK, _ = random_int8_problem(rng, 2, N, d, score_sigma=1.0)
    sVb = rng.uniform(0.01, 0.2, (2, 3)).astype(np.float32)
    Vhat = Vq.astype(np.float64) * np.repeat(sVb.astype(np.float64), Bc, axis=1)[:, :N, None]
    # uniform scores: O is the (prefix) mean of the block-wise dequantized V
    Z = np.zeros_like(Qq)
    out = oracle.int_flash_attn_fwd(Z, Kq, Vq, sQ, sK, sVb, causal, Bc)["O"].reshape(2, N, d)
    ref = np.cumsum(Vhat, 1) / np.arange(1, N + 1)[None, :, None] if causal else np.broadcast_to(Vhat.mean(1, keepdims=True), (2, N, d))
    assert np.allclose(out, ref, rtol=2e-6, atol=1e-8)
    # general scores: p_quant=0 equals fp64 attention of the dequantized inputs, and the P-rounding bound holds
    ref = oracle.attention_fp64(dequant(Qq, sQ), dequant(Kq, sK), Vhat, causal=causal).reshape(2, N, d)
    nq = oracle.int_flash_attn_fwd(Qq, Kq, Vq, sQ, sK, sVb, causal, Bc, p_quant=False)["O"].reshape(2, N, d)
    assert np.abs(nq - ref).max() <= 1e-5 * np.abs(ref).max()
    got = oracle.int_flash_attn_fwd(Qq, Kq, Vq, sQ, sK, sVb, causal, Bc)
    mask = np.tril(np.ones((N, N), bool)) if causal else np.ones((N, N), bool)
    dev_ = np.abs(Vhat[:, None, :, :] - ref[:, :, None, :]) * mask[None, :, :, None]
    bound = 0.5 * dev_.sum(2) / got["l"].reshape(2, N, 1)
    assert np.all(np.abs(got["O"].reshape(2, N, d) - ref) <= bound * (1 + 1e-4) + 1e-6 * np.abs(ref).max())


# ---------------------------------------------------------------- N_q != N_k (queries = the last N_q positions)

@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("Nq,N,Bc", [(1, 200, 64), (40, 100, 32), (64, 192, 64), (37, 37, 16), (5, 130, 128)])
def test_rectangular_without_p_quant_equals_standard_attention(Nq, N, Bc, causal):
    # fp64 reference with the library softmax; causal: query i sees keys j <= i + (N - Nq)
    rng = np.random.default_rng(30)
    Qq, Kq, Vq, sQ, sK, sV = random_int8_problem(rng, 2, N, 32, score_sigma=2.0)
    Qq, sQ = Qq[:, :Nq], sQ[:, :Nq]                      # any Nq rows will do as queries
    got = oracle.int_flash_attn_fwd(Qq, Kq, Vq, sQ, sK, sV, causal, Bc, p_quant=False)["O"].reshape(2, Nq, 32)
    S = np.einsum("hik,hjk->hij", dequant(Qq, sQ), dequant(Kq, sK))
    if causal:
        vis = np.arange(N)[None, :] <= (np.arange(Nq)[:, None] + (N - Nq))
        S = np.where(vis[None], S, -np.inf)
    ref = np.einsum("hij,hjc->hic", scipy.special.softmax(S, axis=-1),
                    Vq.astype(np.float64) * sV[:, None, None].astype(np.float64))
    assert np.allclose(got, ref, rtol=2e-5, atol=2e-6 * np.abs(ref).max())


@pytest.mark.parametrize("Bc", [32, 128])
def test_rectangular_rows_are_rows_of_the_square_problem(Bc):
    # Rows are independent (Algorithm 1 treats each Q_i block alone): the last Nq rows of the square causal
    # problem ARE the causal rectangular problem, bit for bit; without a mask any subset of rows is.
    rng = np.random.default_rng(31)
    N, Nq, d = 160, 48, 32
    Qq, Kq, Vq, sQ, sK, sV = random_int8_problem(rng, 2, N, d, score_sigma=2.0)
    sVb = rng.uniform(0.01, 0.2, (2, -(-N // Bc))).astype(np.float32)      # one V scale per key block
    for causal, sv in itertools.product((False, True), (sV, sVb)):
        full = oracle.int_flash_attn_fwd(Qq, Kq, Vq, sQ, sK, sv, causal, Bc, want_P=True)
        rect = oracle.int_flash_attn_fwd(Qq[:, N - Nq:], Kq, Vq, sQ[:, N - Nq:], sK, sv, causal, Bc, want_P=True)
        pick = (np.arange(2)[:, None] * N + np.arange(N - Nq, N)[None, :]).ravel()
        for key in ("O", "l", "m", "P"):
            assert np.array_equal(rect[key], full[key][pick]), key
    # a single query (decode): the mask changes nothing, and it sees every key
    one = oracle.int_flash_attn_fwd(Qq[:, -1:], Kq, Vq, sQ[:, -1:], sK, sV, True, Bc, want_P=True)
    assert np.array_equal(one["O"], oracle.int_flash_attn_fwd(Qq[:, -1:], Kq, Vq, sQ[:, -1:], sK, sV, False, Bc)["O"])
    assert (one["P"] > 0).sum() > 0 and one["P"].shape == (2, N)
    # first of the Nq causal rows sees exactly N - Nq + 1 keys
    P0 = oracle.int_flash_attn_fwd(Qq[:, N - Nq:], Kq, Vq, sQ[:, N - Nq:], sK, sV, True, Bc, want_P=True)["P"][0]
    assert not P0[N - Nq + 1:].any()


def test_forced_tie_resolution_by_hand():
    # One query, two keys, one block.  S = [0, -x] with x = fp32(ln 2): 127 exp(-x) = 63.4999999 lies 1e-7 below the
    # half-integer 63.5, so line 11 gives P = [127, 63] and the entry is flagged as a near-tie; resolved the other
    # way it is 64.  With V = [100, -50] and s_V = 1 line 16 gives (127*100 - 63*50) / 190 = 50.2631578...
    # and, flipped, (127*100 - 64*50) / 191 = 49.7382198...
    Q = np.array([[[1]]], np.int8); K = np.array([[[0], [-1]]], np.int8); V = np.array([[[100], [-50]]], np.int8)
    sQ = np.ones((1, 1), np.float32); sK = np.array([[1.0, np.float32(np.log(2.0))]], np.float32); sV = np.ones(1, np.float32)
    kw = dict(tie_rel=8 * 2.0 ** -24, tie_abs=2e-6, want_P=True)
    r0 = oracle.int_flash_attn_fwd(Q, K, V, sQ, sK, sV, False, 128, **kw)
    assert r0["n_tie"][0] == 1 and r0["P"].tolist() == [[127, 63]]
    assert abs(r0["O"][0, 0] - 9550.0 / 190.0) < 1e-5
    r1 = oracle.int_flash_attn_fwd(Q, K, V, sQ, sK, sV, False, 128, tie_flip=np.array([1], np.uint64), **kw)
    assert r1["P"].tolist() == [[127, 64]] and abs(r1["O"][0, 0] - 9500.0 / 191.0) < 1e-5 and r1["l"][0] == 191.0
    r2 = oracle.int_flash_attn_fwd(Q, K, V, sQ, sK, sV, False, 128, tie_flip=np.array([2], np.uint64), **kw)   # no second tie
    assert r2["P"].tolist() == [[127, 63]] and r2["O"][0, 0] == r0["O"][0, 0]
    # an entry that is not near a half-integer is never flipped: x = 1 gives 127 / e = 46.72
    sK2 = np.array([[1.0, 1.0]], np.float32)
    r3 = oracle.int_flash_attn_fwd(Q, K, V, sQ, sK2, sV, False, 128, tie_flip=np.array([1], np.uint64), **kw)
    assert r3["n_tie"][0] == 0 and r3["P"].tolist() == [[127, 47]]


def test_compare_up_to_ties_accepts_the_other_valid_result_and_nothing_else():
    Q = np.array([[[1]]], np.int8); K = np.array([[[0], [-1]]], np.int8); V = np.array([[[100], [-50]]], np.int8)
    sQ = np.ones((1, 1), np.float32); sK = np.array([[1.0, np.float32(np.log(2.0))]], np.float32); sV = np.ones(1, np.float32)
    args = (Q, K, V, sQ, sK, sV, False, 128)
    same = oracle.compare_up_to_ties(np.array([[9550.0 / 190.0]]), *args)
    assert same["err"][0] < 1e-5 and same["flips"][0] == 0
    other = oracle.compare_up_to_ties(np.array([[9500.0 / 191.0]]), *args)          # the entry rounded the other way
    assert other["err_default"][0] > 0.5 and other["err"][0] < 1e-5 and other["flips"][0] == 1
    wrong = oracle.compare_up_to_ties(np.array([[50.0]]), *args)                    # between the two: neither result
    assert wrong["err"][0] > 0.2
    # a larger random problem compared with itself: nothing to resolve, zero error
    rng = np.random.default_rng(3)
    Qr, Kr, Vr = (rng.integers(-127, 128, (2, 256, 64), dtype=np.int8) for _ in range(3))
    sq = rng.uniform(0.002, 0.004, (2, 256)).astype(np.float32); sk = rng.uniform(0.002, 0.004, (2, 256)).astype(np.float32)
    sv = np.array([0.01, 0.02], np.float32)
    O = oracle.int_flash_attn_fwd(Qr, Kr, Vr, sq, sk, sv, True, 128)["O"]
    res = oracle.compare_up_to_ties(O, Qr, Kr, Vr, sq, sk, sv, True, 128)
    assert res["err"].max() == 0.0 and res["flips"].sum() == 0
    # ... and with one row replaced by the result of flipping its first flagged entry (if it has one)
    ref = oracle.int_flash_attn_fwd(Qr, Kr, Vr, sq, sk, sv, True, 128, tie_rel=8 * 2.0 ** -24, tie_abs=2e-6)
    flagged = np.nonzero(ref["n_tie"] > 0)[0]
    if flagged.size:
        r = int(flagged[0])
        alt = oracle.int_flash_attn_fwd(Qr, Kr, Vr, sq, sk, sv, True, 128, row_idx=np.array([r]), tie_rel=8 * 2.0 ** -24,
                                        tie_abs=2e-6, tie_flip=np.array([1], np.uint64))["O"]
        O2 = O.copy(); O2[r] = alt[0]
        res2 = oracle.compare_up_to_ties(O2, Qr, Kr, Vr, sq, sk, sv, True, 128, tol=1e-7)
        assert res2["err"].max() <= 1e-7 * res2["scale"] and res2["flips"][r] == 1
