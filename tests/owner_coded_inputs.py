"""Attention inputs whose expected result follows from the lengths alone, at any size.

All keys are zero, so every score is 0 and every token of a sequence weighs the same: the
log-sum-exp of a row is log(Lp + Ls) and its output the plain mean of the value rows it is entitled
to (the definition of attention over [prompt KV | own KV] with a uniform softmax).  The value rows
carry 0/1 codes of their owner (prompt, sample, KV head, prefix or suffix), so:
  * a channel that is 0 in all of a row's own tokens must come out exactly 0 -- one value row read
    from another sequence's page, sample slot or KV head puts a non-zero term there;
  * the log-sum-exp counts the tokens: one token dropped or taken twice moves it by 1 / (Lp + Ls).
Slots past the end of a sequence (padding, the unused part of a last page) hold NaN patterns.
Used on the CPU as a pin of the checker's bookkeeping and on the GPU for every row of the full
configurations."""
import numpy as np

_ONE, _NAN = np.uint16(0x3F80), np.uint16(0x7FC1)


def _bits(x, n):
    b = [(x >> i) & 1 for i in range(n)]
    return np.array(b + [1 - v for v in b], dtype=np.float64)   # bits, then their complements


def _code(prompt, sample, head):
    """128 channels of 0/1 for a value row of `prompt` (sample = None: a prefix token) and KV head."""
    c = np.zeros(128)
    c[0:16] = _bits(prompt, 8)
    if sample is None:
        c[48] = 1.0
    else:
        c[16:48] = _bits(sample, 16)
        c[49] = 1.0
    c[50:56] = _bits(head, 3)
    return c


def ownership_problem(inp):
    """Overwrites K and V of `inp` (bf16) as described above; returns (expected output, expected lse)."""
    sp = inp.spec
    assert sp.dtype == "bf16" and sp.head_dim == 128 and sp.num_kv_heads <= 8 and sp.num_samples < 65536
    Hkv, G, N = sp.num_kv_heads, sp.group, sp.num_samples
    as_bf16 = lambda c: np.where(c != 0, _ONE, np.uint16(0)).astype(np.uint16)
    prompt_of = np.repeat(np.arange(sp.num_prompts), np.diff(inp.sample_indptr))
    if sp.page_size:
        P = sp.page_size
        inp.k_prefix[...] = _NAN
        inp.v_prefix[...] = _NAN      # (the suffix pages live in the same pool)

        def fill(pages, length, prompt, sample):
            full, rem = divmod(int(length), P)
            for j in range(Hkv):
                code = as_bf16(_code(prompt, sample, j))
                inp.v_prefix[pages[:full], j] = code
                inp.k_prefix[pages[:full], j] = 0
                if rem:
                    inp.v_prefix[pages[full], j, :rem] = code
                    inp.k_prefix[pages[full], j, :rem] = 0

        for b in range(sp.num_prompts):
            fill(inp.prefix_page_indices[inp.prefix_indptr[b]:inp.prefix_indptr[b + 1]], inp.prefix_lens[b], b, None)
        for n in range(N):
            fill(inp.suffix_page_indices[inp.suffix_page_indptr[n]:inp.suffix_page_indptr[n + 1]], inp.suffix_lens[n],
                 int(prompt_of[n]), n)
    else:
        inp.k_prefix[...] = 0
        inp.k_suffix[...] = _NAN
        inp.v_suffix[...] = _NAN
        for b in range(sp.num_prompts):
            for j in range(Hkv):
                inp.v_prefix[inp.prefix_indptr[b]:inp.prefix_indptr[b + 1], j] = as_bf16(_code(b, None, j))
        for n in range(N):
            ls = int(inp.suffix_lens[n])
            inp.k_suffix[n, :ls] = 0
            for j in range(Hkv):
                inp.v_suffix[n, :ls, j] = as_bf16(_code(int(prompt_of[n]), n, j))
    lp = inp.prefix_lens[prompt_of].astype(np.float64)
    ls = inp.suffix_lens.astype(np.float64)
    f = ls / (lp + ls)
    expect = np.zeros((N, sp.num_q_heads, 128))
    for n in range(N):
        for j in range(Hkv):
            row = _code(int(prompt_of[n]), n, j)
            row[16:48] *= f[n]
            row[48] = 1.0 - f[n]
            row[49] = f[n]
            expect[n, j * G:(j + 1) * G] = row
    return expect, np.repeat(np.log(lp + ls)[:, None], sp.num_q_heads, axis=1)


def ownership_tree_problem(inp):
    """The same for a tree of shared prefixes (`workloads.CascadeInputs`, bf16, at most four levels
    of at most 1024 groups, fewer than 2048 samples): overwrites the levels' and the suffixes' K and V
    and rewrites the flattened form; returns (expected output, expected lse).

    Channels: level l owns 21 (10 bits of the group, their complements, one flag), the suffix 23
    (11 bits of the sample, complements, flag) from channel 84 on, the KV head 6 from channel 107."""
    from paper_2502_02534_amd import workloads as W
    q, levels = inp.q, inp.levels
    N, Hq, D = q.shape
    Hkv = levels[0].k.shape[1]
    G = Hq // Hkv
    assert q.dtype == np.uint16 and D == 128 and len(levels) <= 4 and N < 2048 and Hkv <= 8
    as_bf16 = lambda c: np.where(c != 0, _ONE, np.uint16(0)).astype(np.uint16)

    def head_part(j):
        c = np.zeros(128)
        c[107:113] = _bits(j, 3)
        return c

    def level_code(l, g, j):
        c = head_part(j)
        c[21 * l:21 * l + 20] = _bits(g, 10)
        c[21 * l + 20] = 1.0
        return c

    def suffix_code(n, j):
        c = head_part(j)
        c[84:106] = _bits(n, 11)
        c[106] = 1.0
        return c

    for l, lv in enumerate(levels):
        assert len(lv.lens) <= 1024
        lv.k[...] = 0
        for g in range(len(lv.lens)):
            for j in range(Hkv):
                lv.v[lv.indptr[g]:lv.indptr[g] + lv.lens[g], j] = as_bf16(level_code(l, g, j))
    inp.k_suffix[...] = _NAN
    inp.v_suffix[...] = _NAN
    for n in range(N):
        ls = int(inp.suffix_lens[n])
        inp.k_suffix[n, :ls] = 0
        for j in range(Hkv):
            inp.v_suffix[n, :ls, j] = as_bf16(suffix_code(n, j))
    W.flatten_cascade(inp)

    expect = np.zeros((N, Hq, 128))
    total = inp.suffix_lens.astype(np.float64).copy()
    group_of = []
    for lv in levels:
        g = np.searchsorted(lv.sample_indptr, np.arange(N), side="right") - 1
        group_of.append(g)
        total += lv.lens[g]
    for n in range(N):
        for j in range(Hkv):
            row = suffix_code(n, j) * (inp.suffix_lens[n] / total[n]) if total[n] else np.zeros(128)
            for l, lv in enumerate(levels):
                g = int(group_of[l][n])
                if total[n]:
                    row = row + level_code(l, g, j) * (lv.lens[g] / total[n])
            if total[n]:
                row[107:113] = _bits(j, 3)   # every token carries the head's bits: weights sum to 1
            expect[n, j * G:(j + 1) * G] = row
    with np.errstate(divide="ignore"):
        lse = np.log(total)
    return expect, np.repeat(lse[:, None], Hq, axis=1)
