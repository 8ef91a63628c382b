"""Pins for the oracle's quantizers (Section 3.2: linear symmetric quantization with
S = rowmax|X| / R for Q, K and S_V = max|V| / R for V; R = 127 as in Algorithm 1)."""
import numpy as np
import pytest

import oracle


def test_identity_on_the_int8_grid():
    # x = k * s0 with integer k in [-127, 127], some |k| = 127, s0 a power of two
    # => quantization returns k and s0 exactly.
    rng = np.random.default_rng(0)
    for s0 in (2.0 ** -7, 2.0 ** -3, 1.0, 4.0):
        k = rng.integers(-127, 128, (64, 128)).astype(np.int8)
        k[:, 5] = 127 * np.where(rng.random(64) < 0.5, 1, -1)
        q, s = oracle.quantize_tokenwise((k.astype(np.float32) * np.float32(s0)))
        assert np.array_equal(q, k)
        assert np.all(s == np.float32(s0))


def test_half_step_error_bound_and_full_range():
    rng = np.random.default_rng(1)
    for x in (rng.standard_normal((200, 64)).astype(np.float32),
              (rng.standard_t(3, (200, 128)) / np.sqrt(3)).astype(np.float16),
              (rng.random((50, 128)) - 0.5).astype(np.float16)):
        q, s = oracle.quantize_tokenwise(x)
        xf = x.astype(np.float64)
        err = np.abs(xf - q.astype(np.float64) * s.astype(np.float64)[:, None])
        assert np.all(err <= 0.5 * s[:, None] * (1 + 1e-5))
        assert np.all(np.abs(q).max(axis=1) == 127)          # absmax element maps to +-127
        assert q.min() >= -127                                   # symmetric grid: never -128
        # the scale is the fp32 quotient absmax / 127
        assert np.array_equal(s, (np.abs(x.astype(np.float32)).max(axis=1) / np.float32(127.0)))


def test_sign_symmetry():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((100, 64)).astype(np.float32)
    q1, s1 = oracle.quantize_tokenwise(x)
    q2, s2 = oracle.quantize_tokenwise(-x)
    assert np.array_equal(q1, -q2) and np.array_equal(s1, s2)


def test_round_half_to_even():
    # absmax = 127 => x * (127/absmax) = x exactly, so halves are exact ties.
    x = np.array([[127.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 3.5, 126.5, -126.5]], np.float32)
    q, s = oracle.quantize_tokenwise(x)
    assert s[0] == 1.0
    assert q[0].tolist() == [127, 0, 2, 2, 0, -2, -2, 4, 126, -126]


def test_zero_row_has_unit_scale():
    x = np.zeros((3, 64), np.float32)
    x[1, 7] = -3.0
    q, s = oracle.quantize_tokenwise(x)
    assert s[0] == 1.0 and s[2] == 1.0 and s[1] == np.float32(3.0) / np.float32(127.0)
    assert not q[0].any() and not q[2].any() and q[1, 7] == -127


def test_headwise_is_rowwise_over_the_whole_head():
    rng = np.random.default_rng(3)
    V = rng.standard_normal((5, 32, 64)).astype(np.float16)
    q, s = oracle.quantize_headwise(V)
    for h in range(5):
        a = np.abs(V[h].astype(np.float32)).max()
        assert s[h] == a / np.float32(127.0)
        assert np.abs(q[h]).max() == 127
        err = np.abs(V[h].astype(np.float64) - q[h].astype(np.float64) * float(s[h]))
        assert err.max() <= 0.5 * s[h] * (1 + 1e-5)
    qg, sg = oracle.quantize_headwise(V, global_scale=True)
    assert np.all(sg == np.abs(V.astype(np.float32)).max() / np.float32(127.0))
    assert (np.abs(qg).reshape(5, -1).max(axis=1) == 127).sum() >= 1


@pytest.mark.parametrize("d", [64, 128])
def test_monotone_and_idempotent(d):
    # Quantizing the dequantized values again returns the same codes (grid points are fixed points
    # up to the fp32 rounding of q*s, which cannot move a code by a full step).
    rng = np.random.default_rng(4)
    x = rng.standard_normal((64, d)).astype(np.float32)
    q, s = oracle.quantize_tokenwise(x)
    q2, s2 = oracle.quantize_tokenwise(q.astype(np.float32) * s[:, None])
    assert np.array_equal(q, q2)
    assert np.allclose(s, s2, rtol=2e-7)
    # order preserving within a row
    i = np.argsort(x, axis=1)
    assert np.all(np.diff(np.take_along_axis(q.astype(np.int32), i, axis=1), axis=1) >= 0)


# ---------------------------------------------------------------- Hadamard rotation (the paper's stated future work)

@pytest.mark.parametrize("d", [32, 64, 128])
def test_hadamard_matches_the_library_matrix_and_is_an_involution(d):
    import scipy.linalg
    rng = np.random.default_rng(40)
    x = rng.integers(-100, 101, (50, d)).astype(np.float32)        # small integers: every butterfly is exact
    y = oracle.hadamard_rows(x)
    H = scipy.linalg.hadamard(d).astype(np.float64)
    assert np.array_equal(y.astype(np.float64), x.astype(np.float64) @ H)
    assert np.array_equal(oracle.hadamard_rows(y), x * d)           # H H = d I
    xr = rng.standard_normal((50, d)).astype(np.float32)
    assert np.allclose(oracle.hadamard_rows(xr), xr.astype(np.float64) @ H, rtol=1e-5, atol=1e-4)


def test_hadamard_rotation_leaves_scores_unchanged_and_tames_outlier_channels():
    rng = np.random.default_rng(41)
    d = 128
    Q = rng.integers(-50, 51, (40, d)).astype(np.float32)
    K = rng.integers(-50, 51, (40, d)).astype(np.float32)
    S = Q.astype(np.float64) @ K.astype(np.float64).T
    Sr = oracle.hadamard_rows(Q).astype(np.float64) @ oracle.hadamard_rows(K).astype(np.float64).T
    assert np.array_equal(Sr, S * d)                                 # (QH)(KH)^T = d QK^T, exactly on integers
    # outlier channels: quantization error of the scores drops once the rotation spreads them out
    X = (rng.random((256, d)) - 0.5).astype(np.float32)
    Y = (rng.random((256, d)) - 0.5).astype(np.float32)
    X[:, [3, 17, 90, 101]] *= 20; Y[:, [5, 17, 64, 120]] *= 20
    S = X.astype(np.float64) @ Y.astype(np.float64).T
    def scores(qf):
        (qx, sx), (qy, sy) = qf(X), qf(Y)
        return (qx.astype(np.float64) * sx[:, None]) @ (qy.astype(np.float64) * sy[:, None]).T
    e_plain = np.abs(scores(oracle.quantize_tokenwise) - S).mean()
    e_rot = np.abs(scores(lambda a: oracle.quantize_tokenwise_hadamard(a, d ** -0.5)) - S).mean()
    assert e_rot < 0.5 * e_plain
