"""The C-ABI library loads and exports every symbol include/spdecode.h declares;
host-side argument checks answer with status codes (no GPU needed, no compute calls)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "spdecode.h")


@pytest.fixture(scope="module")
def lib():
    from paper_2502_02534_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    return binding.load()


def declared_symbols():
    text = open(HEADER).read()
    return sorted(set(re.findall(r"SPD_API\s+[\w\s\*]+?\b(\w+)\s*\(", text)))


def test_header_declares_the_two_entry_points():
    names = declared_symbols()
    assert "shared_prefix_decode_attn" in names and "sample_tokens" in names
    assert len(names) >= 6


def test_every_declared_symbol_is_exported(lib):
    for name in declared_symbols():
        assert hasattr(lib, name), name


def test_status_strings(lib):
    from paper_2502_02534_amd import binding as B
    assert B.status_string(0) == "ok"
    assert "workspace" in B.status_string(3)


def test_plan_and_workspace_size_are_host_arithmetic(lib):
    from paper_2502_02534_amd import binding as B
    d = B.make_desc(dtype=B.SPD_BF16, num_q_heads=32, num_kv_heads=8, head_dim=128, num_prompts=1, num_samples=64)
    pst, nps, sct, nsc = B.spd_attn_plan(d, 8192, 1024)
    assert pst * nps >= 8192 and pst * (nps - 1) < 8192
    assert sct * nsc >= 1024 and sct * (nsc - 1) < 1024
    ws = B.shared_prefix_decode_attn_workspace_size(d, 8192, 1024)
    assert ws >= (nps + nsc) * 64 * 32 * (128 + 2) * 4
    assert B.sample_tokens_workspace_size(64, 128256) > 0
    assert B.sample_tokens_workspace_size(0, 10) == 0


def test_invalid_descriptions_are_rejected_on_the_host(lib):
    from paper_2502_02534_amd import binding as B
    bad = B.make_desc(dtype=B.SPD_BF16, num_q_heads=30, num_kv_heads=8, head_dim=128, num_prompts=1, num_samples=4)
    assert B.shared_prefix_decode_attn_workspace_size(bad, 128, 128) == 0
    with pytest.raises(B.SpdError) as e:
        B.spd_attn_plan(bad, 128, 128)
    assert e.value.status == 1
    unsupported = B.make_desc(dtype=7, num_q_heads=8, num_kv_heads=8, head_dim=128, num_prompts=1, num_samples=4)
    with pytest.raises(B.SpdError) as e:
        B.spd_attn_plan(unsupported, 128, 128)
    assert e.value.status == 2
    paged = B.make_desc(dtype=B.SPD_BF16, num_q_heads=8, num_kv_heads=8, head_dim=128, num_prompts=1, num_samples=4, page_size=32)
    with pytest.raises(B.SpdError):
        B.spd_attn_plan(paged, 128, 128)


def test_null_pointers_are_rejected_before_any_launch(lib):
    from paper_2502_02534_amd import binding as B
    d = B.make_desc(dtype=B.SPD_BF16, num_q_heads=8, num_kv_heads=2, head_dim=128, num_prompts=1, num_samples=4)
    z = ctypes.c_void_p(0)
    rc = lib.shared_prefix_decode_attn(ctypes.byref(d), *([z] * 12), 128, 128, z, z, z, 0, z)
    assert rc == 1
    rc = lib.sample_tokens(z, 0, 4, 100, 100, z, z, z, z, z, 0, z)
    assert rc == 1
    one = ctypes.c_void_p(256)   # never dereferenced: the checks below fail first
    assert lib.sample_tokens(one, 1, 4, 100, 100, one, one, one, one, one, 256, z) == 2     # bf16 logits
    assert lib.sample_tokens(one, 0, 4, 100, 50, one, one, one, one, one, 256, z) == 1      # stride < vocab
    assert lib.sample_tokens(one, 0, 4, 100, 100, one, one, one, one, z, 0, z) == 3         # no workspace
    rc = lib.shared_prefix_decode_attn(ctypes.byref(d), *([one] * 12), 128, 128, one, z, one, 16, z)
    assert rc == 3                                                                            # workspace too small


@pytest.mark.parametrize("samples,hq,hkv,max_prefix,max_suffix", [
    (1, 8, 8, 1, 0), (4, 4, 1, 256, 32), (16, 32, 8, 2048, 256), (64, 32, 8, 8192, 1024),
    (32, 64, 8, 16384, 512), (1024, 32, 8, 16384, 2048), (2, 32, 8, 1 << 20, 1 << 17), (8, 16, 16, 100, 7),
])
def test_plan_invariants(lib, samples, hq, hkv, max_prefix, max_suffix):
    """The launch plan is host arithmetic: parts cover the lengths, are whole tiles, and stay
    within what the merge kernel can take (64 prefix splits + 64 suffix chunks)."""
    from paper_2502_02534_amd import binding as B
    desc = B.make_desc(dtype=B.SPD_BF16, num_q_heads=hq, num_kv_heads=hkv, head_dim=128, num_prompts=1,
                       num_samples=samples, max_samples_per_prompt=samples, page_size=0)
    split, nsplit, chunk, nchunk = B.spd_attn_plan(desc, max_prefix, max_suffix)
    assert split % 64 == 0 and split > 0 and 1 <= nsplit <= 64
    assert split * nsplit >= max_prefix > split * (nsplit - 1)
    assert chunk % 32 == 0 and chunk > 0 and nchunk <= 64
    assert chunk * nchunk >= max_suffix
    if max_suffix > 0:
        assert max_suffix > chunk * (nchunk - 1)
    ws = B.shared_prefix_decode_attn_workspace_size(desc, max_prefix, max_suffix)
    assert ws >= (nsplit + nchunk) * samples * hq * (128 * 2 + 8)


def _levels(B, specs):
    arr = (B.PrefixLevel * len(specs))()
    for i, (groups, spg, max_len, ptr) in enumerate(specs):
        arr[i] = B.PrefixLevel(ptr, ptr, ptr, ptr, 0, ptr, groups, spg, max_len)
    return arr


def test_levels_and_append_entry_points_check_their_arguments(lib):
    from paper_2502_02534_amd import binding as B
    d = B.make_desc(dtype=B.SPD_BF16, num_q_heads=32, num_kv_heads=8, head_dim=128, num_prompts=1, num_samples=64)
    z = ctypes.c_void_p(0)
    one = 256   # never dereferenced: the checks below fail first
    lv = _levels(B, [(1, 64, 4096, one), (4, 16, 700, one)])
    ws = B.shared_prefix_decode_attn_levels_workspace_size(d, lv, 512)
    single = B.shared_prefix_decode_attn_workspace_size(d, 4096, 512)
    assert ws > 0 and single > 0
    # more levels than supported, a level without groups, and stage masks are rejected
    too_many = _levels(B, [(1, 64, 64, one)] * 5)
    assert B.shared_prefix_decode_attn_levels_workspace_size(d, too_many, 512) == 0
    assert B.shared_prefix_decode_attn_levels_workspace_size(d, _levels(B, [(0, 0, 64, one)]), 512) == 0
    o = ctypes.c_void_p(one)
    rc = lib.shared_prefix_decode_attn_levels(ctypes.byref(d), o, 2, lv, o, o, o, z, z, 512, o, z, z, 0, z)
    assert rc == 3                                        # no workspace
    rc = lib.shared_prefix_decode_attn_levels(ctypes.byref(d), z, 2, lv, o, o, o, z, z, 512, o, z, o, ws, z)
    assert rc == 1                                        # no queries
    staged = B.make_desc(dtype=B.SPD_BF16, num_q_heads=32, num_kv_heads=8, head_dim=128, num_prompts=1,
                         num_samples=64, stages=B.STAGE_PREFIX)
    rc = lib.shared_prefix_decode_attn_levels(ctypes.byref(staged), o, 2, lv, o, o, o, z, z, 512, o, z, o, ws, z)
    assert rc == 1
    # append: null tensors and a paged description without page tables
    assert lib.append_suffix_kv(ctypes.byref(d), z, z, z, z, z, z, z, 512, z, -1, z, z) == 1
    paged = B.make_desc(dtype=B.SPD_BF16, num_q_heads=32, num_kv_heads=8, head_dim=128, num_prompts=1,
                        num_samples=64, page_size=16)
    assert lib.append_suffix_kv(ctypes.byref(paged), o, o, o, o, o, z, z, 512, z, -1, z, z) == 1


def test_step_calls_check_their_arguments(lib):
    from paper_2502_02534_amd import binding as B
    z = ctypes.c_void_p(0)
    st = ctypes.c_void_p(256)   # never dereferenced: the checks below fail first
    ok = (B.RowCopy * 1)(B.RowCopy(256, 512, 64))
    for fn in (lib.decode_step_select, lib.decode_step_record):
        assert fn(z, 4, 1, ok, z) == 1                          # no step counter
        assert fn(ctypes.c_void_p(260), 4, 1, ok, z) == 1       # counter not 8-byte aligned
        assert fn(st, 0, 1, ok, z) == 1                         # no steps
        assert fn(st, 4, 0, ok, z) == 1                         # no copies
        assert fn(st, 4, 9, ok, z) == 1                         # more copies than SPD_MAX_STEP_COPIES
        assert fn(st, 4, 1, None, z) == 1
        for bad in (B.RowCopy(0, 512, 64), B.RowCopy(256, 0, 64), B.RowCopy(256, 512, 0),
                    B.RowCopy(256, 512, 6), B.RowCopy(258, 512, 64), B.RowCopy(256, 514, 64)):
            assert fn(st, 4, 1, (B.RowCopy * 1)(bad), z) == 1
    # the one-launch form: the same checks on both lists, then those of append_suffix_kv
    desc = B.make_desc(dtype=B.SPD_BF16, num_q_heads=8, num_kv_heads=2, head_dim=128, num_prompts=1, num_samples=4)
    p = ctypes.c_void_p(4096)

    def adv(state=st, steps=4, nrec=1, rec=ok, nsel=1, sel=ok, d=desc, k=p, v=p, ks=p, vs=p, lens=p, cap=64):
        return lib.decode_step_advance(state, steps, nrec, rec, nsel, sel, ctypes.byref(d) if d is not None else None,
                                       k, v, ks, vs, lens, z, z, cap, z, -1, z, z, z)

    assert adv(state=z) == 1 and adv(state=ctypes.c_void_p(260)) == 1 and adv(steps=0) == 1
    assert adv(nrec=9) == 1 and adv(nsel=9) == 1 and adv(nrec=-1) == 1
    assert adv(nrec=1, rec=None) == 1 and adv(nsel=1, sel=None) == 1
    assert adv(rec=(B.RowCopy * 1)(B.RowCopy(256, 512, 6))) == 1 and adv(sel=(B.RowCopy * 1)(B.RowCopy(0, 512, 64))) == 1
    assert adv(d=None) == 1 and adv(k=z) == 1 and adv(v=z) == 1 and adv(ks=z) == 1 and adv(vs=z) == 1 and adv(lens=z) == 1
    assert adv(k=ctypes.c_void_p(4100)) == 1 and adv(cap=-1) == 1
    paged = B.make_desc(dtype=B.SPD_BF16, num_q_heads=8, num_kv_heads=2, head_dim=128, num_prompts=1, num_samples=4,
                        page_size=16)
    assert adv(d=paged) == 1                                     # paged KV without a page table
    bad_dim = B.make_desc(dtype=B.SPD_BF16, num_q_heads=8, num_kv_heads=2, head_dim=264, num_prompts=1, num_samples=4)
    assert adv(d=bad_dim) == 2
