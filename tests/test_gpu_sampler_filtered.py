"""`sample_tokens_filtered` (min-p, top-k, then top-p) against the CPU checker: bit-exact tokens
except where a uniform sits within 1e-6 of a CDF boundary or a threshold within 1e-6 (relative) of
a probability that fp32 and fp64 may order differently."""
import numpy as np
import pytest

from gpu_checks import compare_tokens
from paper_2502_02534_amd import workloads as W

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def dev():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    from paper_2502_02534_amd import binding, device
    binding.load()
    return device


def _run(dev, x, T, top_p, top_k, min_p, u):
    from paper_2502_02534_amd import binding as B
    rows, vocab = x.shape
    to = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()
    xd, td, pd, ud = to(x), to(T), to(top_p), to(u)
    kd, md = to(top_k), to(min_p)
    tokens = torch.full((rows,), -7, dtype=torch.int32, device="cuda")
    ws = torch.empty(max(256, B.sample_tokens_workspace_size(rows, vocab)), dtype=torch.uint8, device="cuda")
    B.sample_tokens_filtered(xd, B.SPD_F32, rows, vocab, vocab, td, pd, kd, md, ud, tokens, ws)
    torch.cuda.synchronize()
    return tokens.cpu().numpy()


def _check(dev, oracle, x, T, top_p, top_k, min_p, u):
    tok = _run(dev, x, T, top_p, top_k, min_p, u)
    o = oracle.sample_tokens_filtered(x, T, top_p, u, top_k, min_p)
    compare_tokens(tok, o, u, x.shape[1])
    print(f"  kept min/median/max {o['kept'].min()}/{int(np.median(o['kept']))}/{o['kept'].max()}")


CASES = [
    dict(rows=32, vocab=32000, sigma=3.0, ties=False),
    dict(rows=16, vocab=128256, sigma=3.0, ties=False),
    dict(rows=24, vocab=50257, sigma=2.0, ties=True),     # bf16-valued logits: many exact ties
    dict(rows=40, vocab=4099, sigma=6.0, ties=False),
    dict(rows=9, vocab=5, sigma=1.0, ties=True),
    dict(rows=5, vocab=1, sigma=1.0, ties=False),
    # rows the sliced kernels take (vocabulary a multiple of 4), at a size that fills the chip, and with
    # bf16-valued logits: exact ties at the k-th element and at the thresholds
    dict(rows=96, vocab=128256, sigma=3.0, ties=False),
    dict(rows=24, vocab=50256, sigma=2.0, ties=True),
    dict(rows=300, vocab=32000, sigma=4.0, ties=True),
    # more than eight slices per row: rows with a filter leave the sliced kernels for the whole-row routine
    dict(rows=6, vocab=200004, sigma=3.0, ties=False),
]


@pytest.mark.parametrize("i", range(len(CASES)))
def test_filtered_sampling(dev, oracle, i):
    c = CASES[i]
    print(f"filtered sampler case {i}: {c}", flush=True)
    rng = np.random.default_rng(7000 + i)
    rows, vocab = c["rows"], c["vocab"]
    x = (rng.standard_normal((rows, vocab)) * c["sigma"]).astype(np.float32)
    if c["ties"]:
        x = W.bf16_bits_to_f32(W.f32_to_bf16_bits(x))
    T = rng.choice([0.0, 0.3, 0.7, 1.0, 1.3], rows).astype(np.float32)
    top_p = rng.choice([0.3, 0.9, 0.95, 1.0], rows).astype(np.float32)
    top_k = rng.choice([0, 1, 2, 7, 50, 1000, 200000], rows).astype(np.int32)
    min_p = rng.choice([0.0, 1e-4, 0.01, 0.1, 0.7, 1.0], rows).astype(np.float32)
    u = rng.random(rows, dtype=np.float32)
    _check(dev, oracle, x, T, top_p, top_k, min_p, u)


def test_filters_off_equals_sample_tokens(dev, oracle):
    rng = np.random.default_rng(7100)
    x = (rng.standard_normal((16, 20011)) * 3).astype(np.float32)
    T = np.full(16, 0.8, np.float32)
    top_p = np.full(16, 0.9, np.float32)
    u = rng.random(16, dtype=np.float32)
    a = _run(dev, x, T, top_p, None, None, u)                                   # sliced kernels
    b = _run(dev, x, T, top_p, np.zeros(16, np.int32), np.zeros(16, np.float32), u)  # whole-row kernel
    o = oracle.sample_tokens(x, T, top_p, u)
    assert np.array_equal(a, o["token"]) and np.array_equal(b, o["token"])


def test_only_one_filter_given(dev, oracle):
    rng = np.random.default_rng(7200)
    x = (rng.standard_normal((12, 9001)) * 3).astype(np.float32)
    T = np.full(12, 1.0, np.float32)
    top_p = np.full(12, 1.0, np.float32)
    u = rng.random(12, dtype=np.float32)
    _check(dev, oracle, x, T, top_p, np.full(12, 10, np.int32), None, u)
    _check(dev, oracle, x, T, top_p, None, np.full(12, 0.05, np.float32), u)
