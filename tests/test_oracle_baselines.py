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
