"""GPU parity: the HIP library (through its C ABI) against the fp64 checker on the
same seeded inputs.

Tolerances and exemption rules: tests/gpu_checks.py.
"""
import numpy as np
import pytest

from gpu_checks import check_attention, check_tokens
from paper_2502_02534_amd import workloads as W

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2502_02534_amd import binding
    binding.load()          # raises if the HIP library is missing: no fallback
    from paper_2502_02534_amd import device
    return device


@pytest.mark.parametrize("cfg", [1, 2])
def test_attention_small_configs(dev, oracle, cfg):
    print(f"attention cfg{cfg}", flush=True)
    check_attention(dev, oracle, W.make_attn_inputs(cfg, poison_padding=True))


@pytest.mark.parametrize("cfg", [1, 2])
def test_sampler_small_configs(dev, oracle, cfg):
    print(f"sampler cfg{cfg}", flush=True)
    check_tokens(dev, oracle, W.make_sampler_inputs(cfg))


RAGGED = [
    dict(dtype="f32", num_q_heads=6, num_kv_heads=3, head_dim=64, num_prompts=2, samples_per_prompt=5,
         prefix_len=(1, 300), suffix_len=(0, 70)),
    dict(dtype="f32", num_q_heads=4, num_kv_heads=1, head_dim=128, num_prompts=1, samples_per_prompt=3,
         prefix_len=(0, 0), suffix_len=(0, 9)),
    dict(dtype="bf16", num_q_heads=8, num_kv_heads=2, head_dim=128, num_prompts=3, samples_per_prompt=7,
         prefix_len=(1, 700), suffix_len=(0, 300)),
    dict(dtype="bf16", num_q_heads=8, num_kv_heads=1, head_dim=128, num_prompts=1, samples_per_prompt=5,
         prefix_len=(513, 513), suffix_len=(0, 0)),
    dict(dtype="bf16", num_q_heads=16, num_kv_heads=2, head_dim=64, num_prompts=2, samples_per_prompt=9,
         prefix_len=(65, 400), suffix_len=(1, 130)),
    dict(dtype="bf16", num_q_heads=8, num_kv_heads=2, head_dim=128, num_prompts=3, samples_per_prompt=6,
         prefix_len=(1, 500), suffix_len=(0, 200), page_size=16),
    dict(dtype="bf16", num_q_heads=4, num_kv_heads=4, head_dim=128, num_prompts=2, samples_per_prompt=33,
         prefix_len=(100, 200), suffix_len=(0, 40), page_size=16),
    # more than 64 query rows per KV head: prefix and suffix pass share one launch (128-row tiles;
    # 80 rows = one partial tile, 160 rows = one full + one partial, 264 rows = three tiles)
    dict(dtype="bf16", num_q_heads=32, num_kv_heads=8, head_dim=128, num_prompts=3, samples_per_prompt=20,
         prefix_len=(1, 700), suffix_len=(0, 300)),
    dict(dtype="bf16", num_q_heads=16, num_kv_heads=4, head_dim=128, num_prompts=2, samples_per_prompt=40,
         prefix_len=(63, 1100), suffix_len=(0, 400), page_size=16),
    dict(dtype="bf16", num_q_heads=8, num_kv_heads=1, head_dim=128, num_prompts=2, samples_per_prompt=33,
         prefix_len=(64, 129), suffix_len=(1, 33)),
    dict(dtype="bf16", num_q_heads=16, num_kv_heads=2, head_dim=128, num_prompts=1, samples_per_prompt=24,
         prefix_len=(2049, 2049), suffix_len=(0, 0)),
    # more prefix workgroups than CUs (6 prompts x 8 KV heads x 2 row tiles x 3 splits = 288): the fused
    # launch spreads them through the grid
    dict(dtype="bf16", num_q_heads=32, num_kv_heads=8, head_dim=128, num_prompts=6, samples_per_prompt=40,
         prefix_len=(600, 900), suffix_len=(0, 150)),
]


@pytest.mark.parametrize("i", range(len(RAGGED)))
def test_attention_ragged_and_degenerate(dev, oracle, i):
    print(f"ragged attention case {i}: {RAGGED[i]}", flush=True)
    inp = W.make_attn_inputs(0, spec=W.small_spec(**RAGGED[i]), seed=100 + i, poison_padding=True)
    check_attention(dev, oracle, inp)


def test_stage_masks_compose(dev, oracle):
    """Running the stages one call at a time gives the same bits as one full call."""
    from paper_2502_02534_amd import binding as B
    inp = W.make_attn_inputs(2)
    d = dev.upload_attn(inp)
    d.run()
    torch.cuda.synchronize()
    full = d.out.clone()
    d.out.zero_()
    for st in (B.STAGE_PREFIX, B.STAGE_SUFFIX, B.STAGE_MERGE):
        d.run(st)
    torch.cuda.synchronize()
    assert torch.equal(full.view(torch.int16), d.out.view(torch.int16))


def _sampler_case(rows, vocab, sigma, T, top_p, seed, ties=False):
    rng = np.random.default_rng(seed)
    x = (rng.standard_normal((rows, vocab)) * sigma).astype(np.float32)
    if ties:
        x = W.bf16_bits_to_f32(W.f32_to_bf16_bits(x))     # bf16-valued logits: many exact ties
    t = np.broadcast_to(np.asarray(T, np.float32), (rows,)).copy()
    tp = np.broadcast_to(np.asarray(top_p, np.float32), (rows,)).copy()
    return W.SamplerInputs(x, t, tp, rng.random(rows, dtype=np.float32))


SAMPLER_CASES = [
    dict(rows=7, vocab=1, sigma=3, T=0.7, top_p=0.9),
    dict(rows=9, vocab=5, sigma=3, T=0.7, top_p=0.9),
    dict(rows=33, vocab=4097, sigma=3, T=1.0, top_p=0.95),
    dict(rows=16, vocab=32000, sigma=3, T=0.4, top_p=0.9),
    dict(rows=16, vocab=50257, sigma=3, T=1.0, top_p=1.0),
    dict(rows=16, vocab=50257, sigma=3, T=0.0, top_p=0.9),
    dict(rows=16, vocab=32000, sigma=3, T=0.7, top_p=0.9, ties=True),
    dict(rows=8, vocab=128256, sigma=3, T=1.2, top_p=0.95),
    dict(rows=8, vocab=128256, sigma=3, T=0.2, top_p=0.5),
    dict(rows=8, vocab=1000, sigma=0, T=1.0, top_p=0.9),           # all logits equal
    dict(rows=8, vocab=1000, sigma=3, T=1.0, top_p=1e-6),          # nucleus = argmax only
    dict(rows=4, vocab=262144, sigma=3, T=0.9, top_p=0.92),        # the largest vocabulary the call takes (16 slices)
    dict(rows=3, vocab=200003, sigma=3, T=1.1, top_p=0.97),        # 13 slices and a 3-logit tail
]


@pytest.mark.parametrize("i", range(len(SAMPLER_CASES)))
def test_sampler_cases(dev, oracle, i):
    print(f"sampler case {i}: {SAMPLER_CASES[i]}", flush=True)
    check_tokens(dev, oracle, _sampler_case(seed=500 + i, **SAMPLER_CASES[i]))


@pytest.mark.parametrize("vocab,row_stride", [(20011, 20016), (20011, 20021), (32000, 32768), (4097, 4099)])
def test_sampler_strided_rows(dev, oracle, vocab, row_stride):
    """Rows that sit in a wider matrix: 16-byte aligned strides take the sliced kernels, the others
    the whole-row kernel; the padding columns hold 1e30 and must never be read as logits."""
    print(f"sampler strided vocab {vocab} stride {row_stride}", flush=True)
    check_tokens(dev, oracle, _sampler_case(24, vocab, 3, 0.8, 0.9, 900 + row_stride), row_stride=row_stride)


def test_temperature_sweep_in_one_batch(dev, oracle):
    """The paper samples 64 completions at each of three temperatures from one prompt (App.,
    experiment settings): 192 samples share the prefix, the temperature is per sample."""
    print("temperature sweep batch", flush=True)
    spec = W.small_spec(dtype="bf16", num_q_heads=32, num_kv_heads=8, head_dim=128, num_prompts=1,
                        samples_per_prompt=192, prefix_len=(3000, 3000), suffix_len=(1, 600))
    check_attention(dev, oracle, W.make_attn_inputs(0, spec=spec, seed=4242, poison_padding=True))
    T = np.repeat(np.asarray([0.4, 0.7, 1.0], np.float32), 64)
    check_tokens(dev, oracle, _sampler_case(192, 32000, 3, T, 0.95, 4243))


def test_sampler_mixed_per_row_parameters(dev, oracle):
    rows = 64
    rng = np.random.default_rng(77)
    T = rng.choice([0.0, 0.2, 0.4, 0.7, 1.0, 1.2], size=rows)
    tp = rng.choice([0.1, 0.5, 0.9, 0.95, 1.0], size=rows)
    check_tokens(dev, oracle, _sampler_case(rows, 20011, 3, T, tp, 78))


def test_sampler_is_deterministic(dev):
    sin = W.make_sampler_inputs(2)
    ds = dev.upload_sampler(sin)
    ds.run()
    torch.cuda.synchronize()
    a = ds.tokens.clone()
    ds.run()
    torch.cuda.synchronize()
    assert torch.equal(a, ds.tokens)


@pytest.mark.parametrize("vocab,rows", [(20011, 24), (50257, 16), (200003, 3), (20011, 1100)])
@pytest.mark.parametrize("heavy_tail", [False, True])
def test_sampler_no_cut_with_tail_logits(dev, oracle, vocab, rows, heavy_tail):
    """top_p = 1 (the paper sets a temperature and nothing else), a vocabulary that is not a multiple
    of four inside 16-byte aligned rows: the last one to three logits of a row are handled apart
    from the vector loads and must still count in the normaliser.  With `heavy_tail` the last token
    carries most of the mass (end-of-sequence ids sit at the end of a vocabulary)."""
    print(f"sampler top_p=1 vocab {vocab} rows {rows} heavy_tail {heavy_tail}", flush=True)
    sin = _sampler_case(rows, vocab, 3, 0.9, 1.0, 1300 + vocab % 97 + rows)
    if heavy_tail:
        sin.logits[:, -1] = sin.logits.max(axis=1) + 8.0
        sin.logits[::2, -2] = sin.logits[::2, -1] - 1.0
    check_tokens(dev, oracle, sin, row_stride=(vocab + 3) // 4 * 4)
    # and with a cut, same rows
    sin.top_p[:] = 0.9
    check_tokens(dev, oracle, sin, row_stride=(vocab + 3) // 4 * 4)
