"""Seeded random shapes through every attention entry point, every row compared with the oracle at the strict bar
(and, in the second test, through every quantizer entry point, bit for bit):
the fused kernel (square and N_q != N_k), the few-query kernel, per-block V scales, the key-split path and the
half-INT8 variant; d in {64, 128}, 1-8 heads, ragged N_q, N_k up to 1500, with and without the causal mask, flat
to peaked score distributions.  The committed parity cases fix their shapes by hand; this one draws them."""
import numpy as np
import pytest
import torch

import oracle

pytestmark = pytest.mark.gpu

KINDS = ["square", "rect", "few", "vblock", "half", "splitk"]


@pytest.fixture(scope="module")
def ifa():
    import paper_2409_16997_amd as m
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    m.lib()
    return m


def _draw(rng, ifa):
    d = int(rng.choice([64, 128]))
    H = int(rng.choice([1, 2, 3, 5, 8]))
    kind = str(rng.choice(KINDS))
    causal = bool(rng.integers(0, 2))
    Nk = int(rng.choice([rng.integers(1, 140), rng.integers(140, 700), rng.integers(700, 1500)]))
    if kind in ("square", "vblock", "half") and rng.integers(0, 2):
        Nq = Nk
    elif kind == "few":
        Nq = int(rng.integers(1, 65))
    elif kind == "splitk":
        Nq = int(rng.integers(1, 33))
    else:
        Nq = int(rng.integers(1, 500))
    if causal and Nk < Nq:
        Nk = Nq + int(rng.integers(0, 200))
    sigma = float(rng.choice([0.3, 1.0, 3.0]))                      # standard deviation of the scores
    Qq = rng.integers(-127, 128, (H, Nq, d), dtype=np.int8)
    Kq = rng.integers(-127, 128, (H, Nk, d), dtype=np.int8)
    Vq = rng.integers(-127, 128, (H, Nk, d), dtype=np.int8)
    base = sigma / (73.3 * 73.3 * np.sqrt(d))                       # uniform int8 has standard deviation ~73.3
    sQ = (rng.uniform(0.5, 1.5, (H, Nq)) * np.sqrt(base) * np.log2(np.e)).astype(np.float32)
    sK = (rng.uniform(0.5, 1.5, (H, Nk)) * np.sqrt(base)).astype(np.float32)
    Bc = ifa.block_cols(d, causal)
    sV = rng.uniform(0.005, 0.02, (H, -(-Nk // Bc)) if kind == "vblock" else H).astype(np.float32)
    return dict(kind=kind, d=d, H=H, Nq=Nq, Nk=Nk, causal=causal, sigma=sigma), (Qq, Kq, Vq, sQ, sK, sV), Bc


@pytest.mark.parametrize("seed", [101, 102, 103, 104])
def test_random_shapes_meet_the_strict_bar_on_every_row(ifa, seed):
    rng = np.random.default_rng(seed)
    dev = lambda a: torch.from_numpy(a).cuda()[None]
    for case in range(60):
        desc, (Qq, Kq, Vq, sQ, sK, sV), Bc = _draw(rng, ifa)
        d, causal = desc["d"], desc["causal"]
        if desc["kind"] == "half":
            Vh = (Vq.astype(np.float32) * 0.01).astype(np.float16)
            O = ifa.int_flash_attn_fwd_half(dev(Qq), dev(Kq), dev(Vh), dev(sQ), dev(sK), causal=causal, out_dtype=torch.float32)
            ref = oracle.int_flash_attn_fwd_half(Qq, Kq, Vh, sQ, sK, causal, ifa.block_cols_half(d, causal))["O"]
            got = O[0].reshape(-1, d).cpu().numpy()
            assert np.abs(got - ref).max() <= 1e-3 * np.abs(ref).max(), (seed, case, desc)
            continue
        fn = ifa.int_flash_attn_fwd_splitk if desc["kind"] == "splitk" else ifa.int_flash_attn_fwd
        O = fn(dev(Qq), dev(Kq), dev(Vq), dev(sQ), dev(sK), dev(sV), causal=causal, out_dtype=torch.float32)
        got = O[0].reshape(-1, d).cpu().numpy()
        assert np.isfinite(got).all(), (seed, case, desc)
        res = oracle.compare_up_to_ties(got, Qq, Kq, Vq, sQ, sK, sV, causal, Bc)
        assert np.all(res["err"] <= 1e-3 * res["scale"]), (seed, case, desc, float((res["err"] / res["scale"]).max()))


def _widen(t):
    return t.float().cpu().numpy()


@pytest.mark.parametrize("seed", [201, 202])
def test_random_quantizer_calls_equal_the_oracle_bit_for_bit(ifa, seed):
    # every quantizer entry point on drawn shapes, dtypes and value distributions (outlier channels, values near the
    # bottom of the fp32 range of the scale, all-zero rows): codes and scales against the oracle's, bit for bit
    rng = np.random.default_rng(seed)
    dtypes = [torch.float32, torch.float16, torch.bfloat16]
    for case in range(70):
        kind = str(rng.choice(["token", "hadamard", "head", "global", "block", "qkv", "qk"]))
        d = int(rng.choice([32, 64, 128, 256, 512])) if kind in ("token", "hadamard", "qk") else int(rng.choice([64, 128]))
        H = int(rng.choice([1, 2, 3, 7, 32, 40]))
        N = int(rng.choice([1, 5, 64, 129, 1000, 2051]))
        if kind in ("head", "global", "qkv") and (N * d) % 8:
            N += 1
        dt = dtypes[int(rng.integers(0, 3))]
        dist = str(rng.choice(["normal", "outlier", "tiny", "zero_rows"]))
        g = torch.Generator(device="cpu").manual_seed(1000 * seed + case)

        def draw():
            x = torch.randn((H, N, d), generator=g)
            if dist == "outlier":
                x[..., :: max(1, d // 4)] *= 50
            if dist == "tiny":
                x *= 1e-6
            if dist == "zero_rows":
                x[:, ::3] = 0
            return x.to(dt).cuda()

        X = draw()
        desc = (seed, case, kind, d, H, N, str(dt), dist)
        half = np.float32(0.5)
        if kind == "token":
            got = ifa.quantize_tokenwise(X, scale_mul=0.5)
            rq, rs = oracle.quantize_tokenwise(_widen(X))
            ref = (rq, (rs * half).astype(np.float32))
        elif kind == "hadamard":
            got = ifa.quantize_tokenwise(X, scale_mul=d ** -0.5, hadamard=True)
            ref = oracle.quantize_tokenwise_hadamard(_widen(X), scale_mul=d ** -0.5)
        elif kind in ("head", "global"):
            got = ifa.quantize_headwise(X, global_scale=(kind == "global"))
            ref = oracle.quantize_headwise(_widen(X), global_scale=(kind == "global"))
        elif kind == "block":
            got = ifa.quantize_blockwise(X, 128)
            ref = oracle.quantize_blockwise(_widen(X), 128)
        elif kind == "qkv":
            K, V = draw(), draw()
            got = ifa.quantize_qkv(X, K, V, s_Q_mul=0.5)
            got = ifa.quantize_qkv(X, K, V, s_Q_mul=0.5, out=got)           # again, into what the first call left
            (rq, rsq), (rk, rsk), (rv, rsv) = (oracle.quantize_tokenwise(_widen(X)), oracle.quantize_tokenwise(_widen(K)),
                                               oracle.quantize_headwise(_widen(V)))
            ref = (rq, rk, rv, (rsq * half).astype(np.float32), rsk, rsv)
        else:
            K = draw()
            got = ifa.quantize_qk(X, K, s_Q_mul=0.5)
            (rq, rsq), (rk, rsk) = oracle.quantize_tokenwise(_widen(X)), oracle.quantize_tokenwise(_widen(K))
            ref = (rq, rk, (rsq * half).astype(np.float32), rsk)
        for a, b in zip(got, ref):
            assert np.array_equal(a.cpu().numpy(), b), desc
