"""The library's calls under HIP graph capture: no entry point allocates, clears memory with a memset node or
synchronises, so a whole step (quantize_qkv + attention, or a key-split decode call on the static workspace) can be
recorded once and replayed.  Every replay is compared bit for bit with the same calls made eagerly on the same
inputs, with eager work and synchronisations between the replays and the inputs changed in place in between."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ifa():
    import paper_2409_16997_amd as m
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    m.lib()
    return m


def _inputs(seed, shape, sigma):
    g = torch.Generator(device="cpu").manual_seed(seed)
    return [(sigma * torch.randn(shape, generator=g)).to(torch.float16).cuda() for _ in range(3)]


def _capture(fn):
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        fn()
        fn()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        fn()
    return graph


@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("shape", [(2, 4, 640, 128), (1, 3, 333, 64), (2, 32, 512, 128)])
def test_a_captured_step_replays_to_the_eager_result(ifa, shape, causal):
    B, H, N, d = shape
    fold = float(np.log2(np.e) / np.sqrt(d))
    Q, K, V = _inputs(1, shape, 1.0)                                   # the graph's input buffers
    bufs = ifa.quantize_qkv(Q, K, V, s_Q_mul=fold)                     # its intermediate buffers
    O = torch.empty(shape, dtype=torch.float16, device="cuda")

    def step(q=Q, k=K, v=V, out=bufs, o=O):
        t = ifa.quantize_qkv(q, k, v, s_Q_mul=fold, out=out)
        ifa.int_flash_attn_fwd(*t, causal=causal, out=o)

    graph = _capture(step)
    for rep, seed in enumerate([1, 2, 3, 2]):
        q, k, v = _inputs(seed, shape, 1.0 + 0.5 * rep)
        ebufs = ifa.quantize_qkv(q, k, v, s_Q_mul=fold)                # eager, into buffers of its own
        want = ifa.int_flash_attn_fwd(*ebufs, causal=causal)
        torch.cuda.synchronize()
        Q.copy_(q), K.copy_(k), V.copy_(v)
        O.fill_(7.0)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(O, want), (shape, causal, rep)
        for a, b in zip(bufs, ebufs):
            assert torch.equal(a, b), (shape, causal, rep)


@pytest.mark.parametrize("Nq,Nk", [(1, 5000), (4, 2100), (20, 3000)])
def test_a_captured_key_split_call_on_the_static_workspace_replays_to_the_eager_result(ifa, Nq, Nk):
    B, H, d = 1, 8, 128
    rng = np.random.default_rng(Nq + Nk)

    def problem():
        Qq = torch.from_numpy(rng.integers(-127, 128, (B, H, Nq, d), dtype=np.int8)).cuda()
        Kq = torch.from_numpy(rng.integers(-127, 128, (B, H, Nk, d), dtype=np.int8)).cuda()
        Vq = torch.from_numpy(rng.integers(-127, 128, (B, H, Nk, d), dtype=np.int8)).cuda()
        sQ = torch.from_numpy(rng.uniform(2e-3, 4e-3, (B, H, Nq)).astype(np.float32)).cuda()
        sK = torch.from_numpy(rng.uniform(1e-2, 3e-2, (B, H, Nk)).astype(np.float32)).cuda()
        sV = torch.from_numpy(rng.uniform(1e-2, 3e-2, (B, H)).astype(np.float32)).cuda()
        return [Qq, Kq, Vq, sQ, sK, sV]

    static = problem()
    O = torch.empty((B, H, Nq, d), dtype=torch.float16, device="cuda")
    graph = _capture(lambda: ifa.int_flash_attn_fwd_splitk(*static, causal=True, out=O, workspace="static"))
    for rep in range(3):
        cur = problem()
        want = ifa.int_flash_attn_fwd_splitk(*cur, causal=True)        # eager, workspace of its own
        torch.cuda.synchronize()
        for a, b in zip(static, cur):
            a.copy_(b)
        O.fill_(7.0)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(O, want), (Nq, Nk, rep)
