"""Attention over a tree of shared prefixes (`shared_prefix_decode_attn_levels`): the paper's prompts
nest (base prompt shared by all tasks, demonstrations by an iteration's tasks, task text by its
samples); the result must equal plain attention over each sample's concatenated chain of prefixes,
which is what the CPU checker computes on the flattened problem."""
import numpy as np
import pytest

from gpu_checks import attention_errors, lse_errors
from paper_2502_02534_amd import workloads as W

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

CASES = [
    # two levels: one root shared by all 12 samples, three leaf groups
    dict(group_sizes=[[12], [5, 4, 3]], len_ranges=[(300, 300), (1, 200)], suffix_len=(0, 60)),
    # three levels, bf16, enough rows per KV head at every level for the tiled and the fused kernels
    dict(group_sizes=[[72], [40, 32], [20, 20, 16, 16]], len_ranges=[(1500, 1500), (100, 700), (0, 300)],
         num_q_heads=32, num_kv_heads=8, suffix_len=(0, 200)),
    # groups that do not nest (any consecutive grouping is allowed), an empty level, no suffix at all
    dict(group_sizes=[[7, 9], [4, 8, 4], [16]], len_ranges=[(10, 90), (0, 130), (0, 0)], suffix_len=(0, 0)),
    # fp32 path, four levels
    dict(group_sizes=[[6], [3, 3], [2, 2, 2], [1] * 6], len_ranges=[(70, 70), (1, 40), (0, 33), (0, 9)],
         dtype="f32", num_q_heads=4, num_kv_heads=2, head_dim=64, suffix_len=(0, 20)),
]


@pytest.fixture(scope="module")
def dev():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    from paper_2502_02534_amd import binding, device
    binding.load()
    return device


@pytest.mark.parametrize("i", range(len(CASES)))
def test_cascade_equals_attention_over_concatenated_prefixes(dev, oracle, i):
    print(f"cascade case {i}: {CASES[i]}", flush=True)
    inp = W.make_cascade_inputs(seed=900 + i, **CASES[i])
    d = dev.DeviceCascade(inp)
    d.out.fill_(float("nan"))
    d.run()
    torch.cuda.synchronize()
    out = d.out.float().cpu().numpy().astype(np.float64)
    lse = d.lse.cpu().numpy().astype(np.float64)
    ref_out, ref_lse = oracle.attention_inputs(inp.flat)
    err = attention_errors(out, ref_out, inp.spec.dtype)
    lse_errors(lse, ref_lse, inp.spec.dtype)
    print(f"  max abs err {err:.3e}")


def test_paper_shaped_tree_every_row(dev):
    """The tree the paper's prompts form, at its own size (base prompt shared by all 26 tasks' 64
    samples each, demonstrations by all of them, task text by a task's samples; 1664 samples), on
    inputs whose result follows from the lengths alone (tests/owner_coded_inputs.py): zero keys,
    value rows that carry 0/1 codes of level, group, sample and KV head.  Every row of the multi-level
    call and of the same problem flattened to one level."""
    from owner_coded_inputs import ownership_tree_problem
    tasks, per_task = 26, 64
    n = tasks * per_task
    print(f"paper-shaped tree: {tasks} tasks x {per_task} samples, levels 4096 / 8192 / 512 tokens", flush=True)
    inp = W.make_cascade_inputs([[n], [n], [per_task] * tasks], [(4096, 4096), (8192, 8192), (300, 512)],
                                num_q_heads=32, num_kv_heads=8, suffix_len=(0, 1024), seed=5)
    expect, expect_lse = ownership_tree_problem(inp)
    zero = expect == 0
    for name, d in (("levels", dev.DeviceCascade(inp)), ("flattened", dev.upload_attn(inp.flat))):
        d.out.fill_(float("nan"))
        d.lse.fill_(float("nan"))
        d.run()
        torch.cuda.synchronize()
        got = d.out.float().cpu().numpy().astype(np.float64)
        lse = d.lse.cpu().numpy().astype(np.float64)
        del d
        torch.cuda.empty_cache()
        assert np.all(np.isfinite(got)) and np.all(np.isfinite(lse))
        assert np.all(got[zero] == 0), f"{name}: {int((got[zero] != 0).sum())} channels hold a foreign value row"
        # half a unit in the last place of the bf16 result and of the fp16 partial states
        rel = np.abs(got[~zero] - expect[~zero]) / expect[~zero]
        assert rel.max() <= 2.0 ** -8 + 2.0 ** -10, (name, rel.max())
        assert np.abs(lse - expect_lse).max() <= 2e-5, (name, np.abs(lse - expect_lse).max())
        print(f"  {name}: rows {got.shape[0] * got.shape[1]}, max rel err {rel.max():.2e}, "
              f"max lse err {np.abs(lse - expect_lse).max():.2e}", flush=True)
