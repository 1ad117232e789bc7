"""Host-side logic that needs no GPU: the seeded workload generators (shapes, determinism, paged
bookkeeping, the flattened form of a prefix tree) and the benchmark's refusal of more than one GPU."""
import os
import subprocess
import sys

import numpy as np
import pytest

from paper_2502_02534_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.parametrize("cfg", [1, 2])
def test_generator_is_seeded_and_shaped(cfg):
    a, b = W.make_attn_inputs(cfg), W.make_attn_inputs(cfg)
    sp = W.SPECS[cfg]
    n = sp.num_prompts * sp.samples_per_prompt
    assert a.q.shape == (n, sp.num_q_heads, sp.head_dim)
    assert a.q.dtype == (np.uint16 if sp.dtype == "bf16" else np.float32)
    for x, y in ((a.q, b.q), (a.k_prefix, b.k_prefix), (a.v_suffix, b.v_suffix), (a.suffix_lens, b.suffix_lens)):
        assert np.array_equal(x, y)
    assert a.prefix_lens.min() >= sp.prefix_len[0] and a.prefix_lens.max() <= sp.prefix_len[1]
    assert a.sample_indptr[0] == 0 and a.sample_indptr[-1] == n
    s1, s2 = W.make_sampler_inputs(cfg), W.make_sampler_inputs(cfg)
    assert s1.logits.shape == (n, sp.vocab) and np.array_equal(s1.logits, s2.logits)
    assert np.all((s1.uniforms >= 0) & (s1.uniforms < 1))
    other = W.make_attn_inputs(cfg, layer=1)
    assert not np.array_equal(other.q, a.q)          # layers draw from their own streams


def test_bf16_round_trip_is_round_to_nearest_even():
    x = np.float32([1.0, 1.00390625, 1.005859375, -2.5, 3.0e38, 1e-40, 0.0])
    bits = W.f32_to_bf16_bits(x)
    back = W.bf16_bits_to_f32(bits)
    assert back[0] == 1.0 and back[3] == -2.5 and back[6] == 0.0
    assert back[1] == 1.0                               # 1 + 2^-8 is a tie: rounds to the even mantissa
    assert back[2] == np.float32(1.0078125)             # 1 + 1.5 * 2^-8 rounds up to 1 + 2^-7
    assert np.all(np.abs(back[:4] - x[:4]) <= np.abs(x[:4]) * 2.0 ** -8)


def test_paged_layout_bookkeeping():
    spec = W.small_spec(dtype="bf16", num_q_heads=8, num_kv_heads=2, head_dim=128, num_prompts=3,
                        samples_per_prompt=4, prefix_len=(1, 100), suffix_len=(0, 50), page_size=16)
    inp = W.make_attn_inputs(0, spec=spec, seed=9)
    pages_p = np.diff(inp.prefix_indptr)
    assert np.array_equal(pages_p, (inp.prefix_lens + 15) // 16)
    pages_s = np.diff(inp.suffix_page_indptr)
    assert np.array_equal(pages_s, (inp.suffix_lens + 15) // 16)
    used = np.concatenate([inp.prefix_page_indices, inp.suffix_page_indices])
    assert len(set(used.tolist())) == len(used)         # no page is handed out twice
    assert used.max() < inp.k_prefix.shape[0]


def test_pages_in_order_of_use_differ_from_the_shuffled_table_only_in_the_table():
    import dataclasses
    spec = W.small_spec(dtype="bf16", num_q_heads=8, num_kv_heads=2, head_dim=128, num_prompts=3,
                        samples_per_prompt=4, prefix_len=(1, 100), suffix_len=(0, 50), page_size=16)
    a = W.make_attn_inputs(0, spec=spec, seed=9)
    b = W.make_attn_inputs(0, spec=dataclasses.replace(spec, page_order="sequential"), seed=9)
    used = np.concatenate([b.prefix_page_indices, b.suffix_page_indices])
    assert np.array_equal(used, np.arange(len(used)))   # handed out in order of use
    assert not np.array_equal(a.prefix_page_indices, b.prefix_page_indices)
    for x, y in ((a.q, b.q), (a.k_prefix, b.k_prefix), (a.prefix_lens, b.prefix_lens), (a.suffix_lens, b.suffix_lens),
                 (a.prefix_indptr, b.prefix_indptr), (a.suffix_page_indptr, b.suffix_page_indptr)):
        assert np.array_equal(x, y)


def test_prefix_tree_and_its_flattened_form_agree():
    c = W.make_cascade_inputs([[6], [2, 4], [1, 1, 2, 2]], [(5, 5), (0, 7), (1, 3)], suffix_len=(0, 4), seed=3)
    flat = c.flat
    assert flat.sample_indptr.tolist() == [0, 1, 2, 4, 6]
    for g in range(4):                                   # every flat prompt is root | mid | leaf of its chain
        a = int(flat.sample_indptr[g])
        want = []
        for lv in c.levels:
            grp = int(np.searchsorted(lv.sample_indptr, a, side="right") - 1)
            want.append(lv.k[lv.indptr[grp]:lv.indptr[grp] + lv.lens[grp]])
        got = flat.k_prefix[flat.prefix_indptr[g]:flat.prefix_indptr[g] + flat.prefix_lens[g]]
        assert np.array_equal(got, np.concatenate(want))
    assert flat.prefix_lens.sum() == sum(int(lv.lens[np.searchsorted(lv.sample_indptr, a, side="right") - 1])
                                         for a in flat.sample_indptr[:-1] for lv in c.levels)


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr


def test_hand_scheduled_attention_kernels_do_not_spill():
    """The prefix body issues its LDS reads by hand, several fragments ahead of the MFMA that uses
    them, and orders them with explicit waits; that is sound as long as the compiler neither copies
    nor spills a fragment register between the read and the wait.  A kernel that has to spill could
    do so, so the build must keep these kernels free of scratch memory."""
    import concurrent.futures
    import re
    import shutil
    import subprocess
    import tempfile
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc")
    csrc = os.path.join(ROOT, "paper_2502_02534_amd", "csrc")

    def usage(src):
        with tempfile.TemporaryDirectory() as tmp:
            out = subprocess.run(
                [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden", "-munsafe-fp-atomics",
                 "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Rpass-analysis=kernel-resource-usage",
                 "-c", os.path.join(csrc, src), "-o", os.path.join(tmp, "o.o")],
                capture_output=True, text=True, check=True).stderr
        names = re.findall(r"Function Name: (\S+)", out)
        scratch = [int(v) for v in re.findall(r"ScratchSize \[bytes/lane\]: (\d+)", out)]
        assert names and len(names) == len(scratch), out[-2000:]
        return list(zip(names, scratch))

    with concurrent.futures.ThreadPoolExecutor(2) as pool:
        for kernels in pool.map(usage, ["attn_prefix_mfma.hip", "attn_fused.hip"]):
            for name, scratch in kernels:
                assert scratch == 0, (name, scratch)
