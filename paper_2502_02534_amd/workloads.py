"""Seeded synthetic inputs for one decode step of parallel sampling.

This module only draws random numbers and lays them out in the shapes the
library consumes.  It holds none of the method's arithmetic (no softmax, no
attention, no sampling) and imports neither the HIP binding nor the checker, so
both can be fed the same bytes.

Workload shapes follow the parallel-sampling stage of the paper (Alg. 1, the
step that draws n completions from one demonstration-augmented prompt; App.
"Experiment settings": 64 samples per temperature in {0.4, 0.7, 1.0}, at most
1024 output tokens; Sec. 3.3: about 500 tokens per demonstration).  One prompt
(the shared prefix) is attended by N samples, each with a private suffix of
already generated tokens.

All arrays are host numpy arrays.  bf16 tensors are carried as uint16 bit
patterns produced by round-to-nearest-even from float32 normals.
"""
from __future__ import annotations

import concurrent.futures
import dataclasses
import os
from typing import Optional

import numpy as np

SEED_BASE = 250202534 * 10


@dataclasses.dataclass(frozen=True)
class WorkloadSpec:
    name: str
    dtype: str                # "f32" or "bf16"
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    num_prompts: int
    samples_per_prompt: int
    prefix_len: tuple         # (lo, hi) inclusive; lo == hi means fixed
    suffix_len: tuple         # (lo, hi) inclusive
    vocab: int
    logit_sigma: float
    temperature: tuple        # (lo, hi); per prompt when lo != hi
    top_p: float
    page_size: int = 0        # 0 = contiguous KV
    boosted: int = 0          # tokens per row that get +boost
    boost: float = 0.0
    layers: int = 1
    page_order: str = "shuffled"   # paged KV: "shuffled" = pages dealt out at random, "sequential" = in order of use

    @property
    def num_samples(self) -> int:
        return self.num_prompts * self.samples_per_prompt

    @property
    def group(self) -> int:
        return self.num_q_heads // self.num_kv_heads


# The five configurations.  Index = configuration id.
SPECS = {
    1: WorkloadSpec("cfg1-tiny-f32", "f32", 4, 1, 64, 1, 4, (256, 256), (32, 32),
                    1024, 2.0, (0.8, 0.8), 0.95),
    2: WorkloadSpec("cfg2-bf16-p2048-n16", "bf16", 32, 8, 128, 1, 16, (2048, 2048),
                    (256, 256), 32000, 3.0, (0.7, 0.7), 0.9),
    3: WorkloadSpec("cfg3-bf16-p8192-n64", "bf16", 32, 8, 128, 1, 64, (8192, 8192),
                    (128, 1024), 128256, 3.0, (1.0, 1.0), 0.95, boosted=50, boost=8.0),
    4: WorkloadSpec("cfg4-bf16-p16384-n32-l32", "bf16", 64, 8, 128, 1, 32,
                    (16384, 16384), (512, 512), 128256, 3.0, (0.8, 0.8), 0.9, layers=32),
    5: WorkloadSpec("cfg5-bf16-paged-b8-n1024", "bf16", 32, 8, 128, 8, 128,
                    (1024, 16384), (0, 2048), 128256, 3.0, (0.2, 1.2), 0.95, page_size=16),
}


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (nearest, ties to even); returns uint16 bit patterns."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _normal(rng: np.random.Generator, shape, dtype: str, sigma: float = 1.0) -> np.ndarray:
    """N(0, sigma^2) of the given shape.  The array is cut into slabs of 2^24 values; slab i is drawn
    from the i-th child stream of `rng`, so the result does not depend on how many threads draw."""
    n = int(np.prod(shape)) if len(shape) else 1
    out = np.empty(n, dtype=np.uint16 if dtype == "bf16" else np.float32)
    slab = 1 << 24
    starts = list(range(0, n, slab))
    streams = rng.spawn(len(starts)) if starts else []

    def fill(i):
        s = starts[i]
        e = min(n, s + slab)
        v = streams[i].standard_normal(e - s, dtype=np.float32)
        if sigma != 1.0:
            v *= np.float32(sigma)
        out[s:e] = f32_to_bf16_bits(v) if dtype == "bf16" else v

    if len(starts) > 1:
        with concurrent.futures.ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as pool:
            list(pool.map(fill, range(len(starts))))
    else:
        for i in range(len(starts)):
            fill(i)
    return out.reshape(shape)


@dataclasses.dataclass
class AttnInputs:
    """Inputs of one shared-prefix decode-attention call (one layer)."""
    spec: WorkloadSpec
    q: np.ndarray                       # [N, Hq, D]
    k_prefix: np.ndarray                # contiguous: [sum Lp, Hkv, D]; paged: pool [pages, Hkv, P, D]
    v_prefix: np.ndarray
    prefix_lens: np.ndarray             # int32 [B]
    prefix_indptr: np.ndarray           # int32 [B+1]: token offsets (contiguous) or page-list offsets (paged)
    sample_indptr: np.ndarray           # int32 [B+1]
    k_suffix: np.ndarray                # contiguous: [N, Ls_max, Hkv, D]; paged: same pool as prefix
    v_suffix: np.ndarray
    suffix_lens: np.ndarray             # int32 [N]
    max_suffix_len: int
    max_prefix_len: int
    prefix_page_indices: Optional[np.ndarray] = None   # int32, paged only
    suffix_page_indptr: Optional[np.ndarray] = None    # int32 [N+1], paged only
    suffix_page_indices: Optional[np.ndarray] = None


@dataclasses.dataclass
class SamplerInputs:
    logits: np.ndarray       # float32 [rows, V]
    temperature: np.ndarray  # float32 [rows]
    top_p: np.ndarray        # float32 [rows]
    uniforms: np.ndarray     # float32 [rows] in [0, 1)


def _lens(rng, lo_hi, n) -> np.ndarray:
    lo, hi = lo_hi
    if lo == hi:
        return np.full(n, lo, dtype=np.int32)
    return rng.integers(lo, hi + 1, size=n, dtype=np.int32)


def make_attn_inputs(cfg: int, layer: int = 0, *, spec: Optional[WorkloadSpec] = None,
                     seed: Optional[int] = None, poison_padding: bool = False) -> AttnInputs:
    """Attention inputs of configuration `cfg` (layer `layer` for the stacked one).

    `poison_padding` fills the unused tail of each padded suffix slot (and unused
    slots of partially filled pages) with NaN bit patterns so that an over-read
    shows up in the result.
    """
    sp = spec if spec is not None else SPECS[cfg]
    base = SEED_BASE + cfg if seed is None else seed
    root = np.random.default_rng([base, layer])
    r_q, r_kp, r_vp, r_ks, r_vs, r_len, r_perm = root.spawn(7)
    B, N, Hq, Hkv, D = sp.num_prompts, sp.num_samples, sp.num_q_heads, sp.num_kv_heads, sp.head_dim
    # Lengths do not depend on the layer: every layer of a model sees the same sequence.
    len_rng = np.random.default_rng([base, 0]).spawn(7)[5] if layer else r_len
    prefix_lens = _lens(len_rng, sp.prefix_len, B)
    suffix_lens = _lens(len_rng, sp.suffix_len, N)
    sample_indptr = (np.arange(B + 1, dtype=np.int64) * sp.samples_per_prompt).astype(np.int32)
    q = _normal(r_q, (N, Hq, D), sp.dtype)
    nanbits = np.uint16(0x7FC1) if sp.dtype == "bf16" else np.float32(np.nan)

    if sp.page_size == 0:
        tot = int(prefix_lens.sum())
        prefix_indptr = np.concatenate([[0], np.cumsum(prefix_lens)]).astype(np.int32)
        k_prefix = _normal(r_kp, (tot, Hkv, D), sp.dtype)
        v_prefix = _normal(r_vp, (tot, Hkv, D), sp.dtype)
        ls_max = int(sp.suffix_len[1])
        k_suffix = _normal(r_ks, (N, ls_max, Hkv, D), sp.dtype)
        v_suffix = _normal(r_vs, (N, ls_max, Hkv, D), sp.dtype)
        if poison_padding:
            for n in range(N):
                k_suffix[n, suffix_lens[n]:] = nanbits
                v_suffix[n, suffix_lens[n]:] = nanbits
        return AttnInputs(sp, q, k_prefix, v_prefix, prefix_lens, prefix_indptr, sample_indptr,
                          k_suffix, v_suffix, suffix_lens, ls_max, int(prefix_lens.max()))

    P = sp.page_size
    pp = (prefix_lens.astype(np.int64) + P - 1) // P
    spg = (suffix_lens.astype(np.int64) + P - 1) // P
    num_pages = int(pp.sum() + spg.sum())
    perm = r_perm.permutation(num_pages).astype(np.int32)
    if sp.page_order == "sequential":
        perm = np.arange(num_pages, dtype=np.int32)
    prefix_indptr = np.concatenate([[0], np.cumsum(pp)]).astype(np.int32)
    suffix_page_indptr = np.concatenate([[0], np.cumsum(spg)]).astype(np.int32)
    prefix_page_indices = perm[: int(pp.sum())].copy()
    suffix_page_indices = perm[int(pp.sum()):].copy()
    k_pool = _normal(r_kp, (num_pages, Hkv, P, D), sp.dtype)
    v_pool = _normal(r_vp, (num_pages, Hkv, P, D), sp.dtype)
    if poison_padding:
        def poison(lens, indptr, indices):
            for i, L in enumerate(lens):
                r = int(L) % P
                if L > 0 and r:
                    pg = indices[indptr[i + 1] - 1]
                    k_pool[pg, :, r:, :] = nanbits
                    v_pool[pg, :, r:, :] = nanbits
        poison(prefix_lens, prefix_indptr, prefix_page_indices)
        poison(suffix_lens, suffix_page_indptr, suffix_page_indices)
    return AttnInputs(sp, q, k_pool, v_pool, prefix_lens, prefix_indptr, sample_indptr,
                      k_pool, v_pool, suffix_lens, int(sp.suffix_len[1]), int(prefix_lens.max()),
                      prefix_page_indices, suffix_page_indptr, suffix_page_indices)


def make_sampler_inputs(cfg: int, *, spec: Optional[WorkloadSpec] = None,
                        seed: Optional[int] = None, rows: Optional[int] = None) -> SamplerInputs:
    """Logits, temperatures, nucleus mass and uniforms of configuration `cfg`."""
    sp = spec if spec is not None else SPECS[cfg]
    base = SEED_BASE + cfg if seed is None else seed
    root = np.random.default_rng([base, 1 << 20])
    r_logit, r_boost, r_t, r_u = root.spawn(4)
    n = sp.num_samples if rows is None else rows
    logits = _normal(r_logit, (n, sp.vocab), "f32", sp.logit_sigma)
    if sp.boosted:
        for r in range(n):
            idx = r_boost.choice(sp.vocab, size=sp.boosted, replace=False)
            logits[r, idx] += np.float32(sp.boost)
    lo, hi = sp.temperature
    if lo == hi:
        t = np.full(n, lo, dtype=np.float32)
    else:
        per_prompt = r_t.uniform(lo, hi, size=sp.num_prompts).astype(np.float32)
        t = np.repeat(per_prompt, sp.samples_per_prompt)[:n].copy()
        if t.shape[0] < n:
            t = np.resize(t, n)
    top_p = np.full(n, sp.top_p, dtype=np.float32)
    u = r_u.random(n, dtype=np.float32)
    return SamplerInputs(logits, t, top_p, u)


def small_spec(**kw) -> WorkloadSpec:
    """A free-form specification for tests (ragged sizes, odd shapes)."""
    d = dict(name="custom", dtype="bf16", num_q_heads=8, num_kv_heads=2, head_dim=128,
             num_prompts=1, samples_per_prompt=3, prefix_len=(100, 100), suffix_len=(0, 70),
             vocab=1000, logit_sigma=3.0, temperature=(0.7, 0.7), top_p=0.9)
    d.update(kw)
    return WorkloadSpec(**d)


@dataclasses.dataclass
class PrefixLevel:
    """One level of a tree of shared prefixes (contiguous KV)."""
    k: np.ndarray               # [sum lens, Hkv, D]
    v: np.ndarray
    lens: np.ndarray            # int32 [groups]
    indptr: np.ndarray          # int32 [groups+1] token offsets
    sample_indptr: np.ndarray   # int32 [groups+1]
    max_samples_per_group: int
    max_len: int


@dataclasses.dataclass
class CascadeInputs:
    """Inputs of one decode-attention call over several levels of shared prefixes, and the same
    problem written as a single level (`flat`): every distinct chain of groups becomes one prompt
    whose prefix is the concatenation of its groups' KV, which is what the call must equal."""
    spec: WorkloadSpec
    q: np.ndarray
    levels: list
    k_suffix: np.ndarray
    v_suffix: np.ndarray
    suffix_lens: np.ndarray
    max_suffix_len: int
    flat: AttnInputs


def make_cascade_inputs(group_sizes, len_ranges, *, dtype="bf16", num_q_heads=8, num_kv_heads=2, head_dim=128,
                        suffix_len=(0, 70), seed=0) -> CascadeInputs:
    """`group_sizes[l]` lists the number of samples in each consecutive group of level l (each list
    sums to N); `len_ranges[l]` is the (lo, hi) range of that level's group lengths."""
    N = int(sum(group_sizes[0]))
    assert all(int(sum(g)) == N for g in group_sizes)
    rng = np.random.default_rng([250202534, seed])
    r_q, r_s, r_len = rng.spawn(3)
    Hq, Hkv, D = num_q_heads, num_kv_heads, head_dim
    q = _normal(r_q, (N, Hq, D), dtype)
    levels = []
    for l, sizes in enumerate(group_sizes):
        r_k, r_v, r_l = rng.spawn(3)
        lens = _lens(r_l, len_ranges[l], len(sizes))
        indptr = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
        total = max(int(indptr[-1]), 1)
        levels.append(PrefixLevel(_normal(r_k, (total, Hkv, D), dtype), _normal(r_v, (total, Hkv, D), dtype), lens,
                                  indptr, np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32),
                                  int(max(sizes)), int(len_ranges[l][1])))
    ls_max = int(suffix_len[1])
    suffix_lens = _lens(r_len, suffix_len, N)
    r_ks, r_vs = r_s.spawn(2)
    k_suffix = _normal(r_ks, (N, max(ls_max, 1), Hkv, D), dtype)
    v_suffix = _normal(r_vs, (N, max(ls_max, 1), Hkv, D), dtype)
    inp = CascadeInputs(None, q, levels, k_suffix, v_suffix, suffix_lens, max(ls_max, 1), None)
    flatten_cascade(inp, suffix_len)
    return inp


def flatten_cascade(inp: CascadeInputs, suffix_len=None) -> None:
    """(Re)writes `inp.flat` and `inp.spec` from the levels: the same problem as one level, the samples
    cut wherever any level starts a new group.  Call it again after editing the levels' KV."""
    q, levels = inp.q, inp.levels
    _, Hq, D = q.shape
    Hkv = levels[0].k.shape[1]
    dtype = "bf16" if q.dtype == np.uint16 else "f32"
    if suffix_len is None:
        suffix_len = inp.spec.suffix_len
    cuts = sorted(set(int(c) for lv in levels for c in lv.sample_indptr))
    flat_k, flat_v, flat_lens = [], [], []
    for a in cuts[:-1]:
        ks, vs = [], []
        for lv in levels:
            g = int(np.searchsorted(lv.sample_indptr, a, side="right") - 1)
            ks.append(lv.k[lv.indptr[g]:lv.indptr[g] + lv.lens[g]])
            vs.append(lv.v[lv.indptr[g]:lv.indptr[g] + lv.lens[g]])
        flat_k.append(np.concatenate(ks))
        flat_v.append(np.concatenate(vs))
        flat_lens.append(flat_k[-1].shape[0])
    flat_lens = np.asarray(flat_lens, dtype=np.int32)
    fk = np.concatenate(flat_k) if sum(flat_lens) else np.zeros((1, Hkv, D), dtype=q.dtype)
    fv = np.concatenate(flat_v) if sum(flat_lens) else np.zeros((1, Hkv, D), dtype=q.dtype)
    sizes_flat = np.diff(np.asarray(cuts))
    spec = small_spec(dtype=dtype, num_q_heads=Hq, num_kv_heads=Hkv, head_dim=D, num_prompts=len(sizes_flat),
                      samples_per_prompt=int(sizes_flat.max()), prefix_len=(0, int(max(flat_lens.max(), 1))),
                      suffix_len=suffix_len)
    inp.spec = dataclasses.replace(spec, name="cascade")
    inp.flat = AttnInputs(inp.spec, q, fk, fv, flat_lens, np.concatenate([[0], np.cumsum(flat_lens)]).astype(np.int32),
                          np.asarray(cuts, dtype=np.int32), inp.k_suffix, inp.v_suffix, inp.suffix_lens,
                          inp.max_suffix_len, int(max(flat_lens.max(), 1)))
