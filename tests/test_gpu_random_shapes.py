"""Seeded sweep over random small attention problems (group size, head counts, samples per prompt,
ragged prefix and suffix lengths including empty ones, contiguous and paged KV): every path of the
attention call (plain, tiled prefix and suffix, the fused launch with one to three row tiles) must
match the CPU checker."""
import numpy as np
import pytest

from gpu_checks import check_attention, check_tokens
from paper_2502_02534_amd import workloads as W

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _random_spec(rng):
    hkv = int(rng.choice([1, 2, 4, 8]))
    g = int(rng.choice([1, 2, 4, 8]))
    prompts = int(rng.integers(1, 5))
    # rows per KV head from a handful to three 128-row tiles
    spp = int(rng.choice([1, 3, 9, 17, 33, 40, 70]))
    spp = max(1, min(spp, 320 // g))
    lp_hi = int(rng.choice([0, 1, 63, 64, 65, 200, 777, 1300]))
    lp_lo = int(rng.integers(0, lp_hi + 1))
    ls_hi = int(rng.choice([0, 1, 31, 33, 150, 400]))
    ls_lo = int(rng.integers(0, ls_hi + 1))
    dtype = "bf16" if rng.random() < 0.8 else "f32"
    d = 128 if dtype == "bf16" and rng.random() < 0.85 else 64
    page = 16 if rng.random() < 0.4 else 0
    return dict(dtype=dtype, num_q_heads=hkv * g, num_kv_heads=hkv, head_dim=d, num_prompts=prompts,
                samples_per_prompt=spp, prefix_len=(lp_lo, lp_hi), suffix_len=(ls_lo, ls_hi), page_size=page)


SPECS = [_random_spec(np.random.default_rng([77, i])) for i in range(40)]


@pytest.fixture(scope="module")
def dev():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    from paper_2502_02534_amd import binding, device
    binding.load()
    return device


@pytest.mark.parametrize("i", range(len(SPECS)))
def test_random_shape(dev, oracle, i):
    print(f"random shape {i}: {SPECS[i]}", flush=True)
    inp = W.make_attn_inputs(0, spec=W.small_spec(**SPECS[i]), seed=5000 + i, poison_padding=True)
    check_attention(dev, oracle, inp)


def _random_sampler(rng):
    rows = int(rng.choice([1, 2, 7, 31, 64, 130]))
    vocab = int(rng.choice([3, 4, 100, 2047, 2048, 4099, 16385, 32000, 50257, 70001, 128256]))
    if rows * vocab > 6_000_000:
        rows = max(1, 6_000_000 // vocab)
    return dict(rows=rows, vocab=vocab, sigma=float(rng.choice([0.5, 1.0, 3.0, 6.0])),
                T=float(rng.choice([0.0, 0.2, 0.7, 1.0, 1.5])), top_p=float(rng.choice([0.05, 0.5, 0.9, 0.95, 0.999, 1.0])),
                ties=bool(rng.random() < 0.25))


SAMPLERS = [_random_sampler(np.random.default_rng([78, i])) for i in range(30)]


@pytest.mark.parametrize("i", range(len(SAMPLERS)))
def test_random_sampler(dev, oracle, i):
    c = SAMPLERS[i]
    print(f"random sampler {i}: {c}", flush=True)
    rng = np.random.default_rng(6000 + i)
    x = (rng.standard_normal((c["rows"], c["vocab"])) * c["sigma"]).astype(np.float32)
    if c["ties"]:
        x = W.bf16_bits_to_f32(W.f32_to_bf16_bits(x))
    t = np.full(c["rows"], c["T"], np.float32)
    tp = np.full(c["rows"], c["top_p"], np.float32)
    sin = W.SamplerInputs(x, t, tp, rng.random(c["rows"], dtype=np.float32))
    check_tokens(dev, oracle, sin)
