"""Closed forms and peaked softmaxes on the device.

With N(0,1) queries, keys and values and thousands of keys the attention output is an average of
magnitude 0.03, far below the contractual 2e-2; these cases make the outputs large (|o| of order
1): a dominant key (output = that key's value row), identical keys (output = mean of the value
rows), a value constant per KV head (output = the head's constant: pins the head mapping) and
random inputs with the queries scaled up.  Each runs on the fused prefix+suffix launch
(contiguous KV, more than 64 query rows per KV head), on paged KV, and on a tree of shared
prefixes; the result is compared with the closed form itself and with the fp64 checker."""
import copy

import numpy as np
import pytest

from gpu_checks import attention_errors, check_attention, lse_errors
from paper_2502_02534_amd import workloads as W

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

SHAPES = {
    "fused": dict(dtype="bf16", num_q_heads=32, num_kv_heads=8, head_dim=128, num_prompts=2, samples_per_prompt=24,
                  prefix_len=(700, 1500), suffix_len=(1, 300)),
    "paged": dict(dtype="bf16", num_q_heads=16, num_kv_heads=4, head_dim=128, num_prompts=2, samples_per_prompt=40,
                  prefix_len=(300, 1100), suffix_len=(1, 400), page_size=16),
    "small": dict(dtype="bf16", num_q_heads=8, num_kv_heads=2, head_dim=128, num_prompts=1, samples_per_prompt=3,
                  prefix_len=(513, 513), suffix_len=(5, 70)),
}


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2502_02534_amd import binding, device
    binding.load()
    return device


def _bits(x):
    return W.f32_to_bf16_bits(np.asarray(x, np.float32))


def _f(b):
    return W.bf16_bits_to_f32(b).astype(np.float64)


def _run(dev, inp):
    d = dev.upload_attn(inp)
    d.out.fill_(float("nan"))
    d.run()
    torch.cuda.synchronize()
    return d.out.float().cpu().numpy().astype(np.float64), d.lse.cpu().numpy().astype(np.float64)


def _tokens_of(inp, n):
    """(K, V) of sample n over [prefix of its prompt | its suffix], fp64, shape [L, Hkv, D]."""
    sp = inp.spec
    b = int(np.searchsorted(inp.sample_indptr, n, side="right") - 1)
    if sp.page_size == 0:
        p0 = inp.prefix_indptr[b]
        ks = [inp.k_prefix[p0:p0 + inp.prefix_lens[b]], inp.k_suffix[n, :inp.suffix_lens[n]]]
        vs = [inp.v_prefix[p0:p0 + inp.prefix_lens[b]], inp.v_suffix[n, :inp.suffix_lens[n]]]
    else:
        P = sp.page_size

        def seq(pool, pages, L):
            return np.stack([pool[pages[t // P], :, t % P, :] for t in range(L)]) if L else pool[:0, :, 0, :]

        pp = inp.prefix_page_indices[inp.prefix_indptr[b]:]
        sg = inp.suffix_page_indices[inp.suffix_page_indptr[n]:]
        ks = [seq(inp.k_prefix, pp, inp.prefix_lens[b]), seq(inp.k_suffix, sg, inp.suffix_lens[n])]
        vs = [seq(inp.v_prefix, pp, inp.prefix_lens[b]), seq(inp.v_suffix, sg, inp.suffix_lens[n])]
    return _f(np.concatenate(ks)), _f(np.concatenate(vs))


@pytest.mark.parametrize("shape", list(SHAPES))
def test_identical_keys_give_the_mean_of_the_value_rows(dev, oracle, shape):
    print(f"uniform keys, {shape}", flush=True)
    inp = W.make_attn_inputs(0, spec=W.small_spec(**SHAPES[shape]), seed=11, poison_padding=False)
    key = _bits(np.random.default_rng(1).standard_normal(128))
    inp.k_prefix[...] = key
    if inp.k_suffix is not inp.k_prefix:
        inp.k_suffix[...] = key
    out, lse = _run(dev, inp)
    sp = inp.spec
    for n in range(sp.num_samples):
        K, V = _tokens_of(inp, n)
        mean = V.mean(axis=0)                           # [Hkv, D]
        want = np.repeat(mean, sp.group, axis=0)        # query head h reads KV head h // G
        attention_errors(out[n], want, "bf16")
        s = (_f(inp.q[n]) @ _f(key)) / np.sqrt(128.0)   # the one score every key has, per head
        np.testing.assert_allclose(lse[n], s + np.log(len(K)), atol=2.1e-3)
    check_attention(dev, oracle, inp)


@pytest.mark.parametrize("shape", list(SHAPES))
@pytest.mark.parametrize("where", ["prefix", "suffix"])
def test_dominant_key_returns_its_value_row(dev, oracle, shape, where):
    """Every query is 2 * ones; one key per sequence is 2 * ones (score 4 sqrt(128) = 45, every other
    key scores about N(0, 4)), so the softmax weight of the rest is below 1e-12 and the output is the
    dominant key's value row, which is a bf16 vector and therefore must come back exactly."""
    print(f"dominant key in the {where}, {shape}", flush=True)
    inp = W.make_attn_inputs(0, spec=W.small_spec(**SHAPES[shape]), seed=12)
    sp = inp.spec
    inp.q[...] = _bits(2.0)
    two = _bits(np.full(128, 2.0))
    rng = np.random.default_rng(2)
    want = np.zeros((sp.num_samples, sp.num_q_heads, 128))
    P = sp.page_size
    for b in range(sp.num_prompts):
        samples = range(inp.sample_indptr[b], inp.sample_indptr[b + 1])
        if where == "prefix":
            t = int(rng.integers(0, inp.prefix_lens[b]))
            if P == 0:
                row = (inp.prefix_indptr[b] + t,)
            else:
                row = (inp.prefix_page_indices[inp.prefix_indptr[b] + t // P], slice(None), t % P)
            inp.k_prefix[row] = two
            v = _f(inp.v_prefix[row])                   # [Hkv, D]
            for n in samples:
                want[n] = np.repeat(v, sp.group, axis=0)
        else:
            for n in samples:
                t = int(rng.integers(0, inp.suffix_lens[n]))
                if P == 0:
                    row = (n, t)
                else:
                    row = (inp.suffix_page_indices[inp.suffix_page_indptr[n] + t // P], slice(None), t % P)
                inp.k_suffix[row] = two
                want[n] = np.repeat(_f(inp.v_suffix[row]), sp.group, axis=0)
    out, _ = _run(dev, inp)
    assert np.abs(out - want).max() <= 1e-6, np.abs(out - want).max()
    check_attention(dev, oracle, inp)


@pytest.mark.parametrize("shape", list(SHAPES))
def test_value_constant_per_kv_head_pins_the_head_mapping(dev, oracle, shape):
    print(f"constant V per KV head, {shape}", flush=True)
    inp = W.make_attn_inputs(0, spec=W.small_spec(**SHAPES[shape]), seed=13)
    sp = inp.spec
    for j in range(sp.num_kv_heads):
        c = _bits(float(j + 1))
        if sp.page_size == 0:
            inp.v_prefix[:, j, :] = c
            inp.v_suffix[:, :, j, :] = c
        else:
            inp.v_prefix[:, j, :, :] = c
    out, _ = _run(dev, inp)
    want = np.broadcast_to((np.arange(sp.num_q_heads) // sp.group + 1.0)[None, :, None], out.shape)
    assert np.array_equal(out, want), np.abs(out - want).max()


@pytest.mark.parametrize("shape", list(SHAPES))
@pytest.mark.parametrize("gain", [4.0, 16.0])
def test_peaked_softmax_against_the_checker(dev, oracle, shape, gain):
    """Queries scaled up (exact in bf16): scores of standard deviation 4 and 16, so a handful of keys
    carry the softmax and |o| is of order 1."""
    print(f"peaked softmax x{gain}, {shape}", flush=True)
    inp = W.make_attn_inputs(0, spec=W.small_spec(**SHAPES[shape]), seed=14, poison_padding=True)
    inp.q = _bits(W.bf16_bits_to_f32(inp.q) * np.float32(gain))
    err = check_attention(dev, oracle, inp)
    ref, _ = oracle.attention_inputs(inp)
    print(f"  max |ref| {np.abs(ref).max():.2f}, max err {err:.3e}")
    assert np.abs(ref).max() > 1.0


TREES = [
    dict(group_sizes=[[72], [40, 32], [20, 20, 16, 16]], len_ranges=[(1500, 1500), (100, 700), (1, 300)],
         num_q_heads=32, num_kv_heads=8, suffix_len=(1, 200)),
    dict(group_sizes=[[12], [5, 4, 3]], len_ranges=[(300, 300), (1, 200)], suffix_len=(1, 60)),
]


def _run_tree(dev, inp):
    d = dev.DeviceCascade(inp)
    d.out.fill_(float("nan"))
    d.run()
    torch.cuda.synchronize()
    return d.out.float().cpu().numpy().astype(np.float64), d.lse.cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("i", range(len(TREES)))
def test_tree_of_prefixes_peaked_and_constant_value(dev, oracle, i):
    print(f"tree of prefixes, closed forms, case {i}", flush=True)
    inp = W.make_cascade_inputs(seed=950 + i, **TREES[i])
    # peaked: the queries (shared by the tree and its flattened form) scaled by 4
    q4 = _bits(W.bf16_bits_to_f32(inp.q) * np.float32(4.0))
    inp.q = q4
    inp.flat.q = q4
    out, lse = _run_tree(dev, inp)
    ref, ref_lse = oracle.attention_inputs(inp.flat)
    err = attention_errors(out, ref, "bf16")
    lse_errors(lse, ref_lse, "bf16")
    print(f"  peaked: max |ref| {np.abs(ref).max():.2f}, max err {err:.3e}")
    # value constant per KV head at every level and in the suffix, with the queries as drawn (the row sum
    # l adds up unrounded probabilities while the second product multiplies with their bf16 roundings,
    # so with a peaked softmax a constant comes back within one bf16 unit, not exactly)
    q1 = _bits(W.bf16_bits_to_f32(inp.q) * np.float32(0.25))
    const = copy.copy(inp)
    const.q = q1
    const.levels = [copy.copy(lv) for lv in inp.levels]
    hkv = inp.k_suffix.shape[2]
    for lv in const.levels:
        lv.v = lv.v.copy()
        for j in range(hkv):
            lv.v[:, j, :] = _bits(float(j + 1))
    const.v_suffix = inp.v_suffix.copy()
    for j in range(hkv):
        const.v_suffix[:, :, j, :] = _bits(float(j + 1))
    out, _ = _run_tree(dev, const)
    g = inp.q.shape[1] // hkv
    want = np.broadcast_to((np.arange(inp.q.shape[1]) // g + 1.0)[None, :, None], out.shape)
    assert np.array_equal(out, want), np.abs(out - want).max()


# A prefix pass on a launch of its own with more than 128 query rows per KV head and at least 192 wide
# workgroups takes the 256-row workgroups with the long K/V rings (copies two tiles ahead): a call
# without suffixes over many prompts reaches it.
@pytest.mark.parametrize("page", [0, 16])
def test_wide_prefix_workgroups_on_their_own_launch(dev, oracle, page):
    print(f"256-row prefix workgroups, page_size {page}", flush=True)
    spec = W.small_spec(dtype="bf16", num_q_heads=32, num_kv_heads=8, head_dim=128, num_prompts=24,
                        samples_per_prompt=40, prefix_len=(100, 700), suffix_len=(0, 0), page_size=page)
    inp = W.make_attn_inputs(0, spec=spec, seed=15, poison_padding=True)
    rows = np.arange(0, spec.num_samples * spec.num_q_heads, 5, dtype=np.int64)
    check_attention(dev, oracle, inp, rows=rows)
    inp.q = _bits(W.bf16_bits_to_f32(inp.q) * np.float32(4.0))
    check_attention(dev, oracle, inp, rows=rows)


def test_large_values_within_the_stated_range(dev, oracle):
    """V scaled by 2^13 (largest magnitude about 4e4, inside the documented |v| <= 65504 of the bf16
    path, whose partial results are fp16): the output is the unscaled one times 2^13."""
    print("V scaled by 8192", flush=True)
    inp = W.make_attn_inputs(0, spec=W.small_spec(**SHAPES["fused"]), seed=16)
    ref, _ = oracle.attention_inputs(inp)
    big = copy.copy(inp)
    big.v_prefix = _bits(W.bf16_bits_to_f32(inp.v_prefix) * np.float32(8192.0))
    big.v_suffix = _bits(W.bf16_bits_to_f32(inp.v_suffix) * np.float32(8192.0))
    assert np.abs(_f(big.v_prefix)).max() > 3e4
    out, _ = _run(dev, big)
    attention_errors(out / 8192.0, ref, "bf16")
