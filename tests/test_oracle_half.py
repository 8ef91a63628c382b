"""Pins for the oracle's half-INT8 variant (Section 4: INT8 Q and K, FP16 V; the weights P~ = fp16(exp(S - m))
take the place of the INT8 P of Algorithm 1) and for its fp16 rounding helper."""
import numpy as np
import pytest
import scipy.special

import oracle
from helpers import dequant, random_int8_problem


# ---------------------------------------------------------------- fp16 rounding helper == numpy's float16 cast

def test_round_to_half_matches_the_library_cast():
    rng = np.random.default_rng(60)
    mant = rng.standard_normal(4000).astype(np.float32)
    x = mant * np.float32(2.0) ** rng.integers(-30, 17, 4000).astype(np.float32)        # normals, subnormals, underflow, overflow
    # exact ties between neighbouring halfs, normal and subnormal, and the overflow threshold
    ties = np.array([1 + 2.0 ** -11, 1 + 3 * 2.0 ** -11, 2.0 ** -25, 3 * 2.0 ** -25, 5 * 2.0 ** -25, 2.0 ** -14 - 2.0 ** -25,
                     65504.0, 65519.996, 65520.0, 0.0, -0.0, 2.0 ** -24, 2.0 ** -14, 0.1, -0.1, 1.0, 1023.5, 2047.0, 2049.0],
                    np.float32)
    x = np.concatenate([x, ties, -ties])
    with np.errstate(over="ignore"):
        ref = x.astype(np.float16).astype(np.float32)
    got = oracle.round_to_half(x)
    assert np.array_equal(got, ref)
    assert np.array_equal(np.signbit(got), np.signbit(ref))


# ---------------------------------------------------------------- against fp64 attention of the same operands

def _problem(rng, heads, N, d, sigma):
    Qq, Kq, _, sQ, sK, _ = random_int8_problem(rng, heads, N, d, score_sigma=sigma)
    V = rng.standard_normal((heads, N, d)).astype(np.float16)
    return Qq, Kq, V, sQ, sK


def _fp64_reference(Qq, Kq, V, sQ, sK, causal):
    """softmax(Q K^T) V in fp64 with the library softmax, on the dequantized Q, K and the fp16 V as given."""
    S = np.einsum("hik,hjk->hij", dequant(Qq, sQ), dequant(Kq, sK))
    if causal:
        N = S.shape[-1]
        S = np.where(np.tril(np.ones((N, N), bool)), S, -np.inf)
    return np.einsum("hij,hjc->hic", scipy.special.softmax(S, axis=-1), V.astype(np.float64))


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("N,Bc,sigma", [(64, 16, 1.0), (100, 32, 2.0), (128, 64, 4.0), (130, 64, 1.0), (96, 128, 8.0)])
def test_half_variant_is_standard_attention_up_to_the_fp16_rounding_of_the_weights(N, Bc, sigma, causal):
    # Each weight carries a relative error <= 2^-11 (or an absolute 2^-25 once subnormal), in numerator and
    # denominator alike: |O - O_exact| <= 2 * 2^-11 * max|V| + fp32 accumulation noise.  Q, K enter exactly
    # (same integers, same scales), so a wrong index, a dropped rescale or a transposed operand shows at O(1).
    rng = np.random.default_rng(61)
    Qq, Kq, V, sQ, sK = _problem(rng, 2, N, 32, sigma)
    got = oracle.int_flash_attn_fwd_half(Qq, Kq, V, sQ, sK, causal, Bc)["O"].reshape(2, N, 32)
    ref = _fp64_reference(Qq, Kq, V, sQ, sK, causal)
    vmax = float(np.abs(V.astype(np.float64)).max())
    err = np.abs(got - ref).max()
    assert err <= 2 * 2.0 ** -11 * vmax + 1e-5 * vmax
    # and far from a systematic error: the rounding errors are independent, so the typical error is much smaller
    assert np.abs(got - ref).mean() <= 2.0 ** -13 * vmax


def test_single_block_equals_the_definition_with_the_library_fp16_cast():
    # One key block (Bc >= N): O = sum_j h_j V_j / sum_j h_j with h = float16(exp(S - rowmax S)), written with
    # numpy's own float16 cast and fp64 sums.  fp32 accumulation over 80 terms: <= 80 * 2^-24 relative.
    rng = np.random.default_rng(62)
    N, d = 80, 32
    Qq, Kq, V, sQ, sK = _problem(rng, 1, N, d, 3.0)
    got = oracle.int_flash_attn_fwd_half(Qq, Kq, V, sQ, sK, False, 128)
    acc = Qq[0].astype(np.int64) @ Kq[0].astype(np.int64).T
    S = (acc.astype(np.float32) * sQ[0][:, None]) * sK[0][None, :]                      # line 9, fp32, this order
    m = S.max(axis=1)
    h = np.exp((S - m[:, None]).astype(np.float64)).astype(np.float32).astype(np.float16).astype(np.float64)
    ref = (h @ V[0].astype(np.float64)) / h.sum(axis=1, keepdims=True)
    assert np.array_equal(got["m"], m)
    assert np.allclose(got["l"], h.sum(axis=1), rtol=1e-5)
    assert np.abs(got["O"] - ref).max() <= 1e-5 * np.abs(V.astype(np.float64)).max()


def test_uniform_scores_give_the_mean_and_a_dominant_key_gives_its_row():
    rng = np.random.default_rng(63)
    N, d = 96, 16
    V = rng.standard_normal((1, N, d)).astype(np.float16)
    Kq = rng.integers(-127, 128, (1, N, d), dtype=np.int8)
    ones = np.full((1, N), 0.01, np.float32)
    # Q = 0: every score is 0, every weight is exactly 1, l = N
    out = oracle.int_flash_attn_fwd_half(np.zeros((1, N, d), np.int8), Kq, V, ones, ones, False, 32)
    assert np.all(out["l"] == N) and np.all(out["m"] == 0)
    assert np.allclose(out["O"], V[0].astype(np.float64).mean(axis=0)[None, :], rtol=0, atol=1e-5)
    # one key 40 above the rest: its weight is 1, the others underflow fp16 (exp(-40) < 2^-25) and what earlier
    # blocks accumulated is rescaled by exp(-40), below half an ulp of fp32: O is exactly that row of V
    Qq = np.zeros((1, N, d), np.int8); Qq[0, :, 0] = 100
    Kq = np.zeros((1, N, d), np.int8); Kq[0, 37, 0] = 100
    s = np.full((1, N), np.sqrt(40.0 / 10000.0), np.float32)                            # score of key 37 is 40
    out = oracle.int_flash_attn_fwd_half(Qq, Kq, V, s, s, False, 32)
    assert np.all(out["l"] == 1.0)
    assert np.array_equal(out["O"], np.repeat(V[0, 37].astype(np.float32)[None, :], N, axis=0))


def test_causal_rows_see_exactly_their_prefix():
    rng = np.random.default_rng(64)
    N, d, Bc = 96, 32, 32
    Qq, Kq, V, sQ, sK = _problem(rng, 1, N, d, 2.0)
    full = oracle.int_flash_attn_fwd_half(Qq, Kq, V, sQ, sK, True, Bc)["O"]
    assert np.array_equal(full[0], V[0, 0].astype(np.float32))                          # row 0: one key, weight 1
    for i in (31, 32, 70, 95):                                                          # block edges and interiors
        n = i + 1
        pre = oracle.int_flash_attn_fwd_half(Qq[:, :n], Kq[:, :n], V[:, :n], sQ[:, :n], sK[:, :n], False, Bc,
                                             row_idx=np.array([i]))["O"][0]
        assert np.array_equal(full[i], pre)


def test_row_subset_and_block_size_dependence():
    rng = np.random.default_rng(65)
    N, d = 128, 32
    Qq, Kq, V, sQ, sK = _problem(rng, 2, N, d, 2.0)
    full = oracle.int_flash_attn_fwd_half(Qq, Kq, V, sQ, sK, False, 64)["O"]
    rows = np.array([0, 5, 127, 128, 200, 255], np.int64)
    sub = oracle.int_flash_attn_fwd_half(Qq, Kq, V, sQ, sK, False, 64, row_idx=rows)["O"]
    assert np.array_equal(sub, full[rows])
    # unlike Algorithm 1 proper the weights are not on a coarse grid: two block sizes agree to fp16 rounding noise
    other = oracle.int_flash_attn_fwd_half(Qq, Kq, V, sQ, sK, False, 16)["O"]
    assert np.abs(other - full).max() <= 2.0 ** -10 * float(np.abs(V.astype(np.float64)).max())


def test_rectangular_rows_are_rows_of_the_square_problem():
    # rows are independent: the last Nq rows of the square causal problem are the causal rectangular problem
    rng = np.random.default_rng(66)
    N, Nq, d = 160, 48, 32
    Qq, Kq, V, sQ, sK = _problem(rng, 2, N, d, 2.0)
    pick = (np.arange(2)[:, None] * N + np.arange(N - Nq, N)[None, :]).ravel()
    for causal in (False, True):
        full = oracle.int_flash_attn_fwd_half(Qq, Kq, V, sQ, sK, causal, 64)
        rect = oracle.int_flash_attn_fwd_half(Qq[:, N - Nq:], Kq, V, sQ[:, N - Nq:], sK, causal, 64)
        for key in ("O", "l", "m"):
            assert np.array_equal(rect[key], full[key][pick]), key
    # and against fp64 attention with the library softmax under the shifted mask
    Nq2 = 40
    got = oracle.int_flash_attn_fwd_half(Qq[:, :Nq2], Kq, V, sQ[:, :Nq2], sK, True, 32)["O"].reshape(2, Nq2, d)
    S = np.einsum("hik,hjk->hij", dequant(Qq[:, :Nq2], sQ[:, :Nq2]), dequant(Kq, sK))
    vis = np.arange(N)[None, :] <= (np.arange(Nq2)[:, None] + (N - Nq2))
    ref = np.einsum("hij,hjc->hic", scipy.special.softmax(np.where(vis[None], S, -np.inf), axis=-1), V.astype(np.float64))
    assert np.abs(got - ref).max() <= (2 * 2.0 ** -11 + 1e-5) * float(np.abs(V.astype(np.float64)).max())
