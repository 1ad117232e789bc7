"""Pins for the fp64 attention checker: it is compared with things other than
itself: a numpy one-liner, closed forms, invariants, and the running-state algebra of
the paper's attention tasks (App., attn tasks 0-2) stated from the definition: the state
after any set of keys, on growing prefixes and under block-wise merges."""
import math

import numpy as np
import pytest

from paper_2502_02534_amd import workloads as W


def _widen(a, dtype):
    return W.bf16_bits_to_f32(a).astype(np.float64) if dtype == "bf16" else a.astype(np.float64)


def _numpy_reference(inp):
    """softmax(q K^T / sqrt(D)) V written independently with numpy (contiguous layout only)."""
    sp = inp.spec
    q = _widen(inp.q, sp.dtype)
    kp, vp = _widen(inp.k_prefix, sp.dtype), _widen(inp.v_prefix, sp.dtype)
    ks, vs = _widen(inp.k_suffix, sp.dtype), _widen(inp.v_suffix, sp.dtype)
    N, Hq, D = q.shape
    G = sp.group
    out = np.zeros((N, Hq, D))
    lse = np.full((N, Hq), -np.inf)
    for b in range(sp.num_prompts):
        p0, p1 = inp.prefix_indptr[b], inp.prefix_indptr[b + 1]
        for n in range(inp.sample_indptr[b], inp.sample_indptr[b + 1]):
            for h in range(Hq):
                j = h // G
                K = np.concatenate([kp[p0:p1, j], ks[n, : inp.suffix_lens[n], j]])
                V = np.concatenate([vp[p0:p1, j], vs[n, : inp.suffix_lens[n], j]])
                if len(K) == 0:
                    continue
                s = K @ q[n, h] / math.sqrt(D)
                w = np.exp(s - s.max())
                out[n, h] = (w / w.sum()) @ V
                lse[n, h] = s.max() + math.log(w.sum())
    return out, lse


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_brute_force_tiny_odd_shapes(oracle, dtype):
    # odd, non power-of-two sizes in the spirit of the paper's printed unit test (M=5, N=7, K=9, D=11)
    sp = W.small_spec(dtype=dtype, num_q_heads=6, num_kv_heads=3, head_dim=11, num_prompts=2,
                      samples_per_prompt=5, prefix_len=(7, 9), suffix_len=(0, 5))
    inp = W.make_attn_inputs(0, spec=sp, seed=11)
    out, lse = oracle.attention_inputs(inp)
    ref, ref_lse = _numpy_reference(inp)
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-12)
    np.testing.assert_allclose(lse, ref_lse, rtol=0, atol=1e-12)


def test_config1_against_numpy(oracle):
    inp = W.make_attn_inputs(1)
    out, lse = oracle.attention_inputs(inp)
    ref, ref_lse = _numpy_reference(inp)
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-12)
    np.testing.assert_allclose(lse, ref_lse, rtol=0, atol=1e-12)


def _plain(dtype="f32", N=2, Hq=4, Hkv=2, D=8, Lp=5, Ls=3, seed=0):
    rng = np.random.default_rng(seed)
    f = (lambda s: rng.standard_normal(s).astype(np.float32))
    d = dict(q=f((N, Hq, D)), k_prefix=f((Lp, Hkv, D)), v_prefix=f((Lp, Hkv, D)),
             prefix_lens=np.array([Lp], np.int32), prefix_indptr=np.array([0, Lp], np.int32),
             sample_indptr=np.array([0, N], np.int32), k_suffix=f((N, Ls, Hkv, D)),
             v_suffix=f((N, Ls, Hkv, D)), suffix_lens=np.full(N, Ls, np.int32), max_suffix_len=Ls)
    return d


def test_uniform_keys_give_mean_of_values(oracle):
    d = _plain(Lp=6, Ls=4)
    key = np.random.default_rng(5).standard_normal(8).astype(np.float32)
    d["k_prefix"][:] = key
    d["k_suffix"][:] = key
    d["suffix_lens"] = np.array([4, 2], np.int32)
    out, lse = oracle.attention(**d, dtype="f32")
    for n in range(2):
        for h in range(4):
            j = h // 2
            vals = np.concatenate([d["v_prefix"][:, j], d["v_suffix"][n, : d["suffix_lens"][n], j]]).astype(np.float64)
            np.testing.assert_allclose(out[n, h], vals.mean(0), atol=1e-13)
            s = float(d["q"][n, h].astype(np.float64) @ key.astype(np.float64)) / math.sqrt(8)
            assert abs(lse[n, h] - (s + math.log(len(vals)))) < 1e-12


def test_zero_query_gives_mean_of_values(oracle):
    d = _plain()
    d["q"][:] = 0
    out, lse = oracle.attention(**d, dtype="f32")
    vals = np.concatenate([d["v_prefix"][:, 1], d["v_suffix"][0, :, 1]]).astype(np.float64)
    np.testing.assert_allclose(out[0, 3], vals.mean(0), atol=1e-13)
    assert abs(lse[0, 3] - math.log(8)) < 1e-13


def test_dominant_key_selects_its_value_row(oracle):
    d = _plain(Lp=9, Ls=4, D=8)
    n, h, j = 1, 2, 1
    qv = d["q"][n, h].astype(np.float64)
    # make suffix token 2 of sample 1 score far above everything else for this query
    d["k_suffix"][n, 2, j] = (qv / np.dot(qv, qv) * 400.0).astype(np.float32)
    out, _ = oracle.attention(**d, dtype="f32")
    np.testing.assert_allclose(out[n, h], d["v_suffix"][n, 2, j].astype(np.float64), atol=1e-12)


def test_score_shift_leaves_output_and_moves_lse(oracle):
    d = _plain(Hq=2, Hkv=2, D=8)
    out0, lse0 = oracle.attention(**d, dtype="f32", scale=1.0)
    # adding c * q/|q|^2 to every key of a head adds c to every score of that head
    # (exactly representable inputs: q = e_0 * 2, shift keys' channel 0 by c/2)
    d["q"][:] = 0
    d["q"][:, :, 0] = 2.0
    d["k_prefix"][:, :, 0] = np.round(d["k_prefix"][:, :, 0] * 64) / 64      # so that +1.5 is exact in fp32
    d["k_suffix"][:, :, :, 0] = np.round(d["k_suffix"][:, :, :, 0] * 64) / 64
    base, lse_b = oracle.attention(**d, dtype="f32", scale=1.0)
    d["k_prefix"][:, :, 0] += 1.5
    d["k_suffix"][:, :, :, 0] += 1.5
    shifted, lse_s = oracle.attention(**d, dtype="f32", scale=1.0)
    np.testing.assert_allclose(shifted, base, atol=1e-12)
    np.testing.assert_allclose(lse_s, lse_b + 3.0, atol=1e-12)
    assert not np.allclose(out0, base)


def test_head_mapping_with_constant_values_per_kv_head(oracle):
    d = _plain(N=3, Hq=12, Hkv=3, D=8)
    for j in range(3):
        d["v_prefix"][:, j] = j
        d["v_suffix"][:, :, j] = j
    out, _ = oracle.attention(**d, dtype="f32")
    for h in range(12):
        np.testing.assert_allclose(out[:, h], h // 4, atol=1e-13)


def test_scale_argument(oracle):
    d = _plain()
    a, _ = oracle.attention(**d, dtype="f32")
    b, _ = oracle.attention(**d, dtype="f32", scale=1 / math.sqrt(8))
    np.testing.assert_array_equal(a, b)
    d2 = dict(d)
    d2["q"] = d["q"] * np.float32(0.5)
    c, _ = oracle.attention(**d2, dtype="f32", scale=2 / math.sqrt(8))
    np.testing.assert_allclose(a, c, atol=1e-13)


def test_empty_kv_gives_zero_and_minus_inf(oracle):
    d = _plain(Lp=0, Ls=3)
    d["suffix_lens"] = np.array([0, 2], np.int32)
    d["k_prefix"] = np.zeros((0, 2, 8), np.float32)
    d["v_prefix"] = np.zeros((0, 2, 8), np.float32)
    out, lse = oracle.attention(**d, dtype="f32")
    assert np.all(out[0] == 0) and np.all(np.isneginf(lse[0]))
    assert np.all(np.isfinite(lse[1]))


def test_paged_equals_contiguous_and_ignores_page_order(oracle):
    sp = W.small_spec(num_q_heads=4, num_kv_heads=2, head_dim=16, num_prompts=2, samples_per_prompt=3,
                      prefix_len=(5, 50), suffix_len=(0, 40), page_size=16)
    inp = W.make_attn_inputs(0, spec=sp, seed=21, poison_padding=True)
    out_p, lse_p = oracle.attention_inputs(inp)
    assert np.all(np.isfinite(out_p))
    # rebuild the same token sequences contiguously by walking the page tables in the test
    P, Hkv, D = 16, 2, 16
    B, N = 2, 6

    def seq(pool, pages, L):
        rows = [pool[pages[t // P], :, t % P, :] for t in range(L)]
        return np.stack(rows) if rows else np.zeros((0, Hkv, D), pool.dtype)

    kp = [seq(inp.k_prefix, inp.prefix_page_indices[inp.prefix_indptr[b]:], inp.prefix_lens[b]) for b in range(B)]
    vp = [seq(inp.v_prefix, inp.prefix_page_indices[inp.prefix_indptr[b]:], inp.prefix_lens[b]) for b in range(B)]
    ls_max = int(inp.suffix_lens.max())
    ks = np.zeros((N, ls_max, Hkv, D), np.uint16)
    vs = np.zeros_like(ks)
    for n in range(N):
        L = inp.suffix_lens[n]
        ks[n, :L] = seq(inp.k_suffix, inp.suffix_page_indices[inp.suffix_page_indptr[n]:], L)
        vs[n, :L] = seq(inp.v_suffix, inp.suffix_page_indices[inp.suffix_page_indptr[n]:], L)
    out_c, lse_c = oracle.attention(
        inp.q, np.concatenate(kp), np.concatenate(vp), inp.prefix_lens,
        np.concatenate([[0], np.cumsum(inp.prefix_lens)]).astype(np.int32), inp.sample_indptr,
        ks, vs, inp.suffix_lens, ls_max, dtype="bf16")
    np.testing.assert_array_equal(out_p, out_c)
    np.testing.assert_array_equal(lse_p, lse_c)
    # permuting the token order of a contiguous prefix changes nothing but rounding order
    perm = np.random.default_rng(3).permutation(int(inp.prefix_lens[0]))
    kp2, vp2 = [kp[0][perm], kp[1]], [vp[0][perm], vp[1]]
    out_q, _ = oracle.attention(
        inp.q, np.concatenate(kp2), np.concatenate(vp2), inp.prefix_lens,
        np.concatenate([[0], np.cumsum(inp.prefix_lens)]).astype(np.int32), inp.sample_indptr,
        ks, vs, inp.suffix_lens, ls_max, dtype="bf16")
    np.testing.assert_allclose(out_q, out_c, atol=1e-13)


# ---- partial softmax states and their merge, written from the definition -----------------------
# The paper's attention tasks (App., attn tasks 0-2) carry a running (maximum, sum, accumulator)
# state along the keys.  What such a state must hold after any set of keys follows from the plain
# definition alone, so it is written here as that definition (vectorised, no recurrence): the
# checker is then compared with it on growing prefixes and on block-wise merges.

def _state(scores, values):
    """(m, l, acc) of a set of keys: m = max s, l = sum exp(s - m), acc = exp(s - m) @ V.
    The empty set gives (-inf, 0, 0)."""
    if len(scores) == 0:
        return -math.inf, 0.0, np.zeros(values.shape[1])
    m = float(np.max(scores))
    w = np.exp(scores - m)
    return m, float(w.sum()), w @ values


def _merge(a, b):
    """Log-sum-exp merge of two unnormalised partial states (m, l, acc)."""
    (ma, la, oa), (mb, lb, ob) = a, b
    if la == 0:
        return b
    if lb == 0:
        return a
    m = max(ma, mb)
    fa, fb = math.exp(ma - m), math.exp(mb - m)
    return m, la * fa + lb * fb, oa * fa + ob * fb


def _scores_values(inp, n, h):
    sp = inp.spec
    j = h // sp.group
    q = _widen(inp.q, sp.dtype)[n, h]
    Lp = inp.prefix_lens[0]
    K = np.concatenate([_widen(inp.k_prefix, sp.dtype)[:Lp, j], _widen(inp.k_suffix, sp.dtype)[n, : inp.suffix_lens[n], j]])
    V = np.concatenate([_widen(inp.v_prefix, sp.dtype)[:Lp, j], _widen(inp.v_suffix, sp.dtype)[n, : inp.suffix_lens[n], j]])
    return K @ q / math.sqrt(sp.head_dim), V, Lp


def test_growing_prefixes_follow_the_state_definition(oracle):
    """After t keys the result is acc_t / l_t and the log-sum-exp m_t + ln l_t of the state over the
    first t keys, for every t: the checker run on truncated suffixes against numpy on the same
    truncation (which is what a token-by-token running state has to reproduce at every step)."""
    sp = W.small_spec(dtype="f32", num_q_heads=4, num_kv_heads=2, head_dim=11, samples_per_prompt=3,
                      prefix_len=(23, 23), suffix_len=(9, 9))
    inp = W.make_attn_inputs(0, spec=sp, seed=8)
    import copy
    for t in range(0, 10):
        cut = copy.copy(inp)
        cut.suffix_lens = np.full(3, t, np.int32)
        out, lse = oracle.attention_inputs(cut)
        for n in range(3):
            for h in range(4):
                s, V, _ = _scores_values(cut, n, h)
                m, l, acc = _state(s, V)
                np.testing.assert_allclose(acc / l, out[n, h], atol=1e-12)
                assert abs(m + math.log(l) - lse[n, h]) < 1e-12
                p = np.exp(s - s.max())
                np.testing.assert_allclose((p / p.sum()) @ V, out[n, h], atol=1e-12)


def test_cascade_merge_equals_attention_over_concatenation(oracle):
    sp = W.small_spec(dtype="bf16", num_q_heads=4, num_kv_heads=1, head_dim=16, samples_per_prompt=4,
                      prefix_len=(37, 37), suffix_len=(0, 12))
    inp = W.make_attn_inputs(0, spec=sp, seed=9)
    out, lse = oracle.attention_inputs(inp)
    empty = (-math.inf, 0.0, np.zeros(16))
    for n in range(4):
        for h in range(4):
            s, V, Lp = _scores_values(inp, n, h)
            pre = _state(s[:Lp], V[:Lp])
            suf = _state(s[Lp:], V[Lp:])
            for a, b in ((pre, suf), (suf, pre)):                      # commutative
                m, l, acc = _merge(a, b)
                np.testing.assert_allclose(acc / l, out[n, h], atol=1e-12)
                assert abs(m + math.log(l) - lse[n, h]) < 1e-12
            # any split point of the prefix, merged in any grouping (associative)
            for cut in (1, 16, 36):
                p1 = _state(s[:cut], V[:cut])
                p2 = _state(s[cut:Lp], V[cut:Lp])
                left = _merge(_merge(p1, p2), suf)
                right = _merge(p1, _merge(p2, suf))
                for m, l, acc in (left, right):
                    np.testing.assert_allclose(acc / l, out[n, h], atol=1e-12)
            # the empty state is the identity
            m, l, acc = _merge(_merge(empty, pre), _merge(suf, empty))
            np.testing.assert_allclose(acc / l, out[n, h], atol=1e-12)


def test_row_subset_matches_full(oracle):
    inp = W.make_attn_inputs(1)
    out, lse = oracle.attention_inputs(inp)
    rows = np.array([13, 0, 7], np.int64)
    o2, l2 = oracle.attention_inputs(inp, rows=rows)
    np.testing.assert_array_equal(o2, out.reshape(-1, 64)[rows])
    np.testing.assert_array_equal(l2, lse.reshape(-1)[rows])


@pytest.mark.parametrize("page_size", [0, 16])
def test_zero_keys_and_owner_coded_values_pin_the_bookkeeping(oracle, page_size):
    """Zero keys make the softmax uniform: every row is the mean of its own value rows and its
    log-sum-exp the logarithm of its token count (tests/owner_coded_inputs.py).  A wrong page, a
    wrong sample slot, a wrong KV head or a miscounted length in the checker fails here."""
    from owner_coded_inputs import ownership_problem
    spec = W.small_spec(dtype="bf16", num_q_heads=8, num_kv_heads=2, head_dim=128, num_prompts=3,
                        samples_per_prompt=4, prefix_len=(1, 100), suffix_len=(0, 50), page_size=page_size)
    inp = W.make_attn_inputs(0, spec=spec, seed=9)
    expect, expect_lse = ownership_problem(inp)
    ref, ref_lse = oracle.attention_inputs(inp)
    assert np.abs(ref.reshape(expect.shape) - expect).max() <= 1e-14
    assert np.abs(ref_lse.reshape(expect_lse.shape) - expect_lse).max() <= 1e-14


def test_owner_coded_tree_pins_the_flattened_form(oracle):
    """The tree variant of the owner-coded inputs: the checker on the flattened problem must give the
    means and token counts that follow from the levels' lengths."""
    from owner_coded_inputs import ownership_tree_problem
    inp = W.make_cascade_inputs(group_sizes=[[12], [5, 4, 3], [2, 3, 4, 3]], len_ranges=[(30, 30), (1, 40), (0, 9)],
                                suffix_len=(0, 20), seed=77)
    expect, expect_lse = ownership_tree_problem(inp)
    ref, ref_lse = oracle.attention_inputs(inp.flat)
    assert np.abs(ref.reshape(expect.shape) - expect).max() <= 1e-14
    assert np.abs(ref_lse.reshape(expect_lse.shape) - expect_lse).max() <= 1e-14
