"""The e4m3 rounding used by the FP8 accuracy baseline, pinned against the format's definition
(OCP FP8: 1-4-3, bias 7, max 448, subnormal step 2^-9), and sanity of the MRE helper."""
import itertools

import numpy as np

from oracle import baselines


def all_e4m3_values():
    vals = []
    for e, m in itertools.product(range(16), range(8)):
        if e == 15 and m == 7:
            continue                                   # NaN encoding
        vals.append((m / 8.0) * 2.0 ** -6 if e == 0 else (1 + m / 8.0) * 2.0 ** (e - 7))
    return np.array(sorted(set(vals)))


def test_e4m3_grid_points_are_fixed_and_midpoints_tie_to_even():
    g = all_e4m3_values()
    assert g.max() == 448.0 and g[1] == 2.0 ** -9 and len(g) == 127
    assert np.array_equal(baselines.round_e4m3(g), g)
    assert np.array_equal(baselines.round_e4m3(-g), -g)
    # nearest-value property against brute force on random points
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.uniform(-460, 460, 4000), rng.uniform(-0.05, 0.05, 4000)])
    full = np.concatenate([-g[::-1], g])
    brute = full[np.abs(x[:, None] - full[None, :]).argmin(1)]
    got = baselines.round_e4m3(x)
    assert np.all(np.abs(got - x) <= np.abs(brute - x) + 1e-15)
    # exact midpoints go to the even mantissa
    assert baselines.round_e4m3(1.0625) == 1.0 and baselines.round_e4m3(1.1875) == 1.25
    assert baselines.round_e4m3(1000.0) == 448.0


def test_mre_helper():
    a = np.array([[1.0, -2.0], [4.0, 0.0]])
    assert baselines.mre(a, a) == {"sum_ratio": 0.0, "mean_elementwise": 0.0}
    r = baselines.mre(a * 1.1, a)
    assert abs(r["sum_ratio"] - 0.1) < 1e-12


def test_baselines_track_fp64_attention():
    import oracle
    rng = np.random.default_rng(1)
    Q, K, V = (rng.standard_normal((256, 64)) for _ in range(3))
    rows = np.arange(0, 256, 8)
    for causal in (False, True):
        ref = oracle.attention_fp64(Q[None], K[None], V[None], causal=causal, scale=0.125, row_idx=rows)
        e16 = baselines.mre(baselines.attention_fp16(Q, K, V, rows, causal, 0.125), ref)["sum_ratio"]
        e8 = baselines.mre(baselines.attention_fp8_tensor(Q, K, V, rows, causal, 0.125), ref)["sum_ratio"]
        assert e16 < 5e-3 and 5e-3 < e8 < 0.2


# ------------------------------------------------------------------------------------------------
# Pins of the two comparison-precision emulations (the FP16 and FP8 columns of Tables 1-2, Section 4.2;
# FP8 = tensor-level scales, Section 3 opening).  Every expected value below is worked out by hand from
# the formats' definitions, not by re-running the emulation's own operations.

LN_0P3 = 1.2039728043259361        # -ln(0.3): a score gap that makes the second softmax weight exactly 0.3


def _two_key_problem(v1, v2, big):
    """One query, two keys, scores [0, ln 0.3] after `scale`: Q.K1 = 0, Q.K2 = -big^2 ... all entries on both
    the fp16 and the e4m3 grid, each tensor's absmax exactly `big`."""
    Q = np.array([[big, 0.0]])
    K = np.array([[0.0, big], [-1.0, 0.0]])
    V = np.array([v1, v2], dtype=np.float64)
    return Q, K, V, LN_0P3 / big


def test_fp8_baseline_two_key_row_by_hand():
    # Inputs on the e4m3 grid with absmax exactly 448: every tensor scale is 1 and quantization is the identity.
    # Softmax weights before rounding: [1, 0.3], row sum l = 1.3 (the UNROUNDED weights are summed).
    # e4m3 neighbours of 0.3 in the binade [0.25, 0.5) (step 2^-5): 0.28125 and 0.3125 -> 0.3125 is nearer.
    # O = (1 * V1 + 0.3125 * V2) / 1.3.
    Q, K, V, scale = _two_key_problem([448.0, 16.0], [-448.0, 32.0], 448.0)
    O = baselines.attention_fp8_tensor(Q, K, V, np.array([0]), False, scale)
    want = np.array([(448.0 - 0.3125 * 448.0) / 1.3, (16.0 + 0.3125 * 32.0) / 1.3])
    assert np.allclose(O[0], want, rtol=2e-6, atol=0)
    # ... and it is NOT the value without the e4m3 cast of the weights (0.3 instead of 0.3125)
    assert abs(O[0, 1] - (16.0 + 0.3 * 32.0) / 1.3) > 0.2


def test_fp8_baseline_tensor_scales():
    # The same problem with every tensor multiplied by a constant whose product with 448 is exact:
    # Q8, K8, V8 are the same codes, the scales are the constants, so O(c) = c_V * O(1) when the softmax scale
    # is divided by c_Q c_K.  Dropping or misplacing any one of the three scales breaks this.
    Q, K, V, scale = _two_key_problem([448.0, 16.0], [-448.0, 32.0], 448.0)
    O1 = baselines.attention_fp8_tensor(Q, K, V, np.array([0]), False, scale)
    cq, ck, cv = 0.375, 1.5, 0.75
    Oc = baselines.attention_fp8_tensor(Q * cq, K * ck, V * cv, np.array([0]), False, scale / (cq * ck))
    assert np.allclose(Oc, cv * O1, rtol=2e-6, atol=0)
    # a scale that does not cancel: without s_q * s_k in the scores the second weight would be 0.3^(1/(cq ck))
    Ou = baselines.attention_fp8_tensor(Q * cq, K * ck, V * cv, np.array([0]), False, scale)
    w2 = 0.3 ** (cq * ck)                                   # = 0.5080..., e4m3 neighbours 0.5 and 0.5625 -> 0.5
    assert np.allclose(Ou[0, 1], cv * (16.0 + 0.5 * 32.0) / (1.0 + w2), rtol=2e-6)


def test_fp8_baseline_uniform_scores_give_mean_of_rounded_v():
    # All scores equal (the query's only non-zero entry meets a zero column of K): every weight is exactly 1, an
    # e4m3 value, so O = mean over keys of the e4m3-quantized V.  448 in each tensor fixes the scales at 1.
    # V is off the grid on purpose:
    #   300: step 32 in [256, 512) -> neighbours 288 and 320 -> 288 (12 away against 20)
    #   100: step 8 in [64, 128) -> 96 and 104, a tie -> even mantissa: 96 (1.100b x 64; 104 = 1.101b x 64)
    #    17: step 2 in [16, 32) -> 16 and 18, a tie -> even mantissa: 16 (1.000b x 16; 18 = 1.001b x 16)
    V = np.array([[448.0, 300.0], [0.0, 100.0], [-448.0, 17.0]])
    K = np.array([[0.0, 448.0], [0.0, 3.0], [0.0, 5.0]])
    Q = np.array([[448.0, 0.0]])
    O = baselines.attention_fp8_tensor(Q, K, V, np.array([0]), False, 1.0)
    assert np.allclose(O[0], [0.0, (288.0 + 96.0 + 16.0) / 3.0], rtol=2e-6, atol=1e-4)


def test_fp8_baseline_one_hot_row():
    # one key 40 above the others in score: the other weights (e^-40) vanish below the e4m3 subnormal step
    # and below fp32 resolution of l, so O is exactly that key's quantized V row
    Q = np.array([[448.0, 0.0]])
    K = np.array([[0.0, 448.0], [-448.0, 0.0], [-448.0, 0.0]])
    V = np.array([[448.0, -300.0], [7.0, 448.0], [-9.0, 100.0]])
    O = baselines.attention_fp8_tensor(Q, K, V, np.array([0]), False, 40.0 / (448.0 * 448.0))
    assert np.array_equal(O[0], [448.0, -288.0])
    # causal row 1 sees keys 0 and 1 only; with equal scores both weights are 1: the mean of two quantized rows
    K2 = np.array([[0.0, 448.0], [0.0, 448.0], [448.0, 0.0]])
    Oc = baselines.attention_fp8_tensor(np.array([[0.0, 0.0], [448.0, 0.0], [1.0, 1.0]]), K2, V, np.array([1]), True, 1.0)
    assert np.allclose(Oc[0], [(448.0 + 7.0) / 2.0, (-288.0 + 448.0) / 2.0], rtol=2e-6)


def test_fp16_baseline_two_key_row_by_hand():
    # fp16-exact inputs, scores [0, ln 0.3]: weights [1, 0.3], l = 1.3 (unrounded weights, fp32).
    # fp16 of 0.3: binade [0.25, 0.5) has step 2^-12; 0.3 / 2^-12 = 1228.8 -> 1229 * 2^-12 = 0.300048828125.
    # Column 0: V = [1, 0]: O = 1 / 1.3 = 0.769230...; fp16 step in [0.5, 1) is 2^-11: 1575.38 -> 1575 * 2^-11
    #           = 0.76904296875 (the output cast).
    # Column 1: V = [0, 1024]: O = 0.300048828125 * 1024 / 1.3 = 236.3461...; fp16 step in [128, 256) is 0.125:
    #           236.375.  Without the fp16 cast of the weight it would be 0.3 * 1024 / 1.3 = 236.3077 -> 236.25.
    Q, K, V, scale = _two_key_problem([1.0, 0.0], [0.0, 1024.0], 1.0)
    O = baselines.attention_fp16(Q, K, V, np.array([0]), False, scale)
    assert np.array_equal(O[0], [0.76904296875, 236.375])


def test_fp16_baseline_inputs_are_cast_to_fp16():
    # K = [1.0004, 1]: fp16 has step 2^-10 just above 1, so both keys become 1.0 and, whatever the softmax scale,
    # their scores are equal: weights [1, 1], O = (0 + 8) / 2 = 4.  Without the input cast the scores would differ
    # by 0.0004 * 5000 = 2 and O would be 8 e^-2 / (1 + e^-2) = 0.95.
    Q = np.array([[1.0]]); K = np.array([[1.0004], [1.0]]); V = np.array([[0.0], [8.0]])
    O = baselines.attention_fp16(Q, K, V, np.array([0]), False, 5000.0)
    assert np.array_equal(O[0], [4.0])
    # V is cast too: 0.1 -> fp16 0.0999755859375 (1638 * 2^-14; 0.1 / 2^-14 = 1638.4) and 24.1 -> 24.09375
    # (step 2^-6 in [16, 32): 1542.4 -> 1542); with Q = 0 the weights are 1, 1:
    # O = (0.0999755859375 + 24.09375) / 2 = 12.09686279296875 -> output cast, step 2^-7 in [8, 16): 1548.4 -> 1548
    # -> 12.09375.  With V left in fp64 it would be 12.1 -> 1548.8 -> 1549 -> 12.1015625.
    V2 = np.array([[0.1], [24.1]])
    O2 = baselines.attention_fp16(np.zeros((1, 1)), np.ones((2, 1)), V2, np.array([0]), False, 1.0)
    assert np.array_equal(O2[0], [12.09375])


def test_fp16_baseline_one_hot_and_causal():
    Q = np.array([[1.0, 0.0], [1.0, 0.0]])
    K = np.array([[0.0, 1.0], [-1.0, 0.0]])
    V = np.array([[3.0, -5.0], [100.0, 200.0]])
    # row 0 under the causal mask sees key 0 only: exactly V[0]
    O = baselines.attention_fp16(Q, K, V, np.array([0, 1]), True, 40.0)
    assert np.array_equal(O[0], [3.0, -5.0])
    # row 1 sees both, key 1 is 40 below: weight e^-40 ~ 4e-18 is below the smallest fp16 subnormal -> exactly V[0]
    assert np.array_equal(O[1], [3.0, -5.0])
