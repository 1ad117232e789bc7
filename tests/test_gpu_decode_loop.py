"""Loop of decode steps with KV append on the device (`append_suffix_kv` + attention + sampler),
checked step by step against the CPU checker run on the same growing KV; then the same loop
replayed from a captured graph must reproduce the eager results bit for bit."""
import copy

import numpy as np
import pytest

from gpu_checks import attention_errors, compare_tokens
from paper_2502_02534_amd import workloads as W

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

STEPS = 9
VOCAB = 4099
CASES = [
    dict(dtype="bf16", num_q_heads=8, num_kv_heads=2, head_dim=128, num_prompts=2, samples_per_prompt=6,
         prefix_len=(40, 300), suffix_len=(0, 60)),
    dict(dtype="bf16", num_q_heads=32, num_kv_heads=8, head_dim=128, num_prompts=1, samples_per_prompt=24,
         prefix_len=(700, 700), suffix_len=(0, 90)),
    dict(dtype="bf16", num_q_heads=16, num_kv_heads=4, head_dim=128, num_prompts=2, samples_per_prompt=20,
         prefix_len=(100, 500), suffix_len=(0, 70), page_size=16),
    dict(dtype="f32", num_q_heads=4, num_kv_heads=2, head_dim=64, num_prompts=1, samples_per_prompt=5,
         prefix_len=(33, 33), suffix_len=(0, 20)),
]


@pytest.fixture(scope="module")
def dev():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    from paper_2502_02534_amd import binding, device
    binding.load()
    return device


def _step_inputs(inp, seed):
    sp = inp.spec
    rng = np.random.default_rng(seed)
    n = inp.q.shape[0]
    def draw(shape):
        x = rng.standard_normal(shape).astype(np.float32)
        return W.f32_to_bf16_bits(x) if sp.dtype == "bf16" else x
    q = draw((STEPS, n, sp.num_q_heads, sp.head_dim))
    k = draw((STEPS, n, sp.num_kv_heads, sp.head_dim))
    v = draw((STEPS, n, sp.num_kv_heads, sp.head_dim))
    u = rng.random((STEPS, n), dtype=np.float32)
    logits = (rng.standard_normal((n, VOCAB)) * 3).astype(np.float32)
    return q, k, v, u, logits


def _capacity(inp):
    n = inp.q.shape[0]
    if inp.spec.page_size == 0:
        return np.full(n, inp.max_suffix_len, dtype=np.int64)
    pages = np.diff(inp.suffix_page_indptr).astype(np.int64)
    return np.minimum(pages * inp.spec.page_size, inp.max_suffix_len)


def _host_append(inp, n, pos, krow, vrow):
    if inp.spec.page_size == 0:
        inp.k_suffix[n, pos] = krow
        inp.v_suffix[n, pos] = vrow
    else:
        P = inp.spec.page_size
        pg = inp.suffix_page_indices[inp.suffix_page_indptr[n] + pos // P]
        inp.k_suffix[pg, :, pos % P, :] = krow
        inp.v_suffix[pg, :, pos % P, :] = vrow


@pytest.mark.parametrize("one_launch", [False, True], ids=["three_launches", "one_launch"])
@pytest.mark.parametrize("i", range(len(CASES)))
def test_decode_loop_matches_checker_and_graph_replay(dev, oracle, i, one_launch):
    """`one_launch`: select, append and record as one decode_step_advance call per step (the results
    of a step are recorded by the next step's call, those of the last by a final record call);
    otherwise as three calls."""
    print(f"decode loop case {i}: {CASES[i]}, one_launch={one_launch}", flush=True)
    inp = W.make_attn_inputs(0, spec=W.small_spec(**CASES[i]), seed=700 + i)
    # leave every sample room for the steps inside its own slot / page list where it had any
    inp.suffix_lens = np.maximum(inp.suffix_lens - STEPS + 2, 0).astype(np.int32)
    q, k, v, u, logits = _step_inputs(inp, 800 + i)
    n = inp.q.shape[0]
    temp = np.full(n, 0.8, np.float32)
    top_p = np.full(n, 0.9, np.float32)
    bf16 = inp.spec.dtype == "bf16"

    # ---- checker: the same loop on the host ----
    tokens_ref = [oracle.sample_tokens(logits, temp, top_p, u[t]) for t in range(STEPS)]
    end_token = int(np.bincount(tokens_ref[1]["token"]).argmax())  # some samples finish after step 1
    host = copy.deepcopy(inp)
    cap = _capacity(host)
    finished = np.zeros(n, dtype=bool)
    ref_out, ref_lens = [], []
    for t in range(STEPS):
        if t > 0:
            finished |= tokens_ref[t - 1]["token"] == end_token
        for s in range(n):
            pos = int(host.suffix_lens[s])
            if not finished[s] and pos < cap[s]:
                _host_append(host, s, pos, k[t, s], v[t, s])
                host.suffix_lens[s] = pos + 1
        host.q = q[t]
        out, _ = oracle.attention_inputs(host)
        ref_out.append(out)
        ref_lens.append(host.suffix_lens.copy())
    assert finished.any() and not finished.all()

    # ---- device: eager loop ----
    def fresh_loop():
        a = dev.upload_attn(inp)
        s = dev.upload_sampler(W.SamplerInputs(logits, temp, top_p, u[0].copy()))
        to = lambda x: torch.from_numpy(x).cuda()
        as_el = (lambda x: to(x).view(torch.int16).view(torch.bfloat16)) if bf16 else to
        return dev.DecodeLoop(a, s, as_el(q), as_el(k), as_el(v), to(u), end_token, one_launch=one_launch)

    loop = fresh_loop()
    for t in range(STEPS):
        loop.one_step()
    loop.flush()
    torch.cuda.synchronize()
    assert loop.step.tolist() == [STEPS, STEPS, 0]
    lens = loop.lens_steps.cpu().numpy()
    toks = loop.tokens_steps.cpu().numpy()
    outs = loop.out_steps.float().cpu().numpy().astype(np.float64)
    for t in range(STEPS):
        assert np.array_equal(lens[t], ref_lens[t]), (t, lens[t], ref_lens[t])
        attention_errors(outs[t], ref_out[t], inp.spec.dtype)
        compare_tokens(toks[t], tokens_ref[t], u[t], VOCAB, label=f"step {t} ")

    # ---- device: one step captured as a graph, replayed STEPS times ----
    g_loop = fresh_loop()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        g_loop.one_step()          # warm-up outside the capture (same stream rules as a capture)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    # restore the state the warm-up step changed
    fresh = fresh_loop()
    g_loop.attn.k_suffix.copy_(fresh.attn.k_suffix)
    g_loop.attn.v_suffix.copy_(fresh.attn.v_suffix)
    g_loop.attn.suffix_lens.copy_(fresh.attn.suffix_lens)
    g_loop.finished.zero_()
    g_loop.step.zero_()
    g_loop.sampler.tokens.fill_(-1)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        g_loop.one_step()
    # the capture itself executes nothing; replay the step STEPS times with eager work in between
    for t in range(STEPS):
        graph.replay()
        _ = (g_loop.attn.out.float().sum() + t).item()   # eager kernel + host synchronisation between replays
    g_loop.flush()
    torch.cuda.synchronize()
    assert torch.equal(g_loop.lens_steps, loop.lens_steps)
    assert torch.equal(g_loop.tokens_steps, loop.tokens_steps)
    assert torch.equal(g_loop.out_steps.view(torch.uint8), loop.out_steps.view(torch.uint8))


def test_step_select_and_record_follow_the_device_counter(dev):
    """Rows chosen by the device-side counter: wide (16-byte) and narrow (4-byte) copies, rows
    longer than one workgroup's share, the last row repeated by select past the end, nothing
    recorded past the end, and the counter pair after every call."""
    from paper_2502_02534_amd import binding as B
    steps = 5
    g = torch.Generator(device="cpu").manual_seed(3)
    big = torch.randint(-2**31, 2**31 - 1, (steps, 40000), dtype=torch.int32, generator=g).cuda()   # 160000 B rows
    odd = torch.randint(-2**31, 2**31 - 1, (steps, 7), dtype=torch.int32, generator=g).cuda()       # 28 B rows
    shifted = torch.randint(-2**31, 2**31 - 1, (steps * 12 + 1,), dtype=torch.int32, generator=g).cuda()[1:].view(steps, 12)
    big_now, odd_now, sh_now = torch.zeros(40000, dtype=torch.int32).cuda(), torch.zeros(7, dtype=torch.int32).cuda(), \
        torch.zeros(12, dtype=torch.int32).cuda()
    rec_big, rec_odd = torch.full_like(big, -1), torch.full_like(odd, -1)
    state = torch.zeros(2, dtype=torch.int64).cuda()
    sel = B.make_row_copies([(big, big_now, 160000), (odd, odd_now, 28), (shifted, sh_now, 48)])
    rec = B.make_row_copies([(big_now, rec_big, 160000), (odd_now, rec_odd, 28)])
    for t in range(steps + 2):
        B.decode_step_select(state, steps, sel)
        torch.cuda.synchronize()
        row = min(t, steps - 1)
        assert state.tolist() == [t, t + 1]
        assert torch.equal(big_now, big[row]) and torch.equal(odd_now, odd[row]) and torch.equal(sh_now, shifted[row])
        B.decode_step_record(state, steps, rec)
        torch.cuda.synchronize()
        assert state.tolist() == [t + 1, t + 1]
    assert torch.equal(rec_big, big) and torch.equal(rec_odd, odd)


def test_step_advance_records_selects_and_appends_in_one_launch(dev):
    """decode_step_advance alone, against plain tensor arithmetic: the counter triple after every
    call, rows selected (the last one repeated past the end), results recorded one call later
    (nothing past the end), the new K/V rows in the suffix slots, lengths recorded before the
    append, full slots and finished samples left alone."""
    from paper_2502_02534_amd import binding as B
    steps, n, hkv, d, cap = 4, 3, 2, 64, 5
    g = torch.Generator(device="cpu").manual_seed(11)
    rnd = lambda *shape: torch.randn(*shape, generator=g).cuda()
    k_steps, v_steps = rnd(steps, n, hkv, d), rnd(steps, n, hkv, d)
    x_steps = torch.randint(-2**31, 2**31 - 1, (steps, 50), dtype=torch.int32, generator=g).cuda()   # 200 B rows
    x_now = torch.zeros(50, dtype=torch.int32).cuda()
    result = torch.zeros(7, dtype=torch.int32).cuda()                                               # 28 B rows
    result_steps = torch.full((steps, 7), -1, dtype=torch.int32).cuda()
    k_suffix, v_suffix = torch.zeros(n, cap, hkv, d).cuda(), torch.zeros(n, cap, hkv, d).cuda()
    lens0 = [0, 3, 5]                                             # sample 2 starts with a full slot
    lens = torch.tensor(lens0, dtype=torch.int32).cuda()
    lens_steps = torch.full((steps, n), -1, dtype=torch.int32).cuda()
    tokens = torch.tensor([7, 7, 7], dtype=torch.int32).cuda()    # nobody's last token is the end token (9) yet
    finished = torch.zeros(n, dtype=torch.int32).cuda()
    desc = B.make_desc(dtype=B.SPD_F32, num_q_heads=hkv, num_kv_heads=hkv, head_dim=d, num_prompts=1, num_samples=n)
    state = torch.zeros(3, dtype=torch.int64).cuda()
    rec = B.make_row_copies([(result, result_steps, 28)])
    sel = B.make_row_copies([(x_steps, x_now, 200)])
    want_len = list(lens0)
    want_k = torch.zeros_like(k_suffix)
    done = [False] * n
    for t in range(steps + 2):
        if t == 2:
            tokens[0] = 9                                          # sample 0 draws the end token in step 1
        B.decode_step_advance(state, steps, rec, sel, desc, k_steps, v_steps, k_suffix, v_suffix, lens, None, None, cap,
                              tokens, 9, finished, lens_steps)
        torch.cuda.synchronize()
        row = min(t, steps - 1)
        assert state.tolist() == [t + 1, t + 1, 0]
        assert torch.equal(x_now, x_steps[row])
        if 1 <= t <= steps:
            assert lens_steps[t - 1].tolist() == want_len          # the lengths the step before left
            assert torch.equal(result_steps[t - 1], torch.full((7,), 100 + t - 1, dtype=torch.int32).cuda())
        for s in range(n):
            done[s] = done[s] or int(tokens[s]) == 9
            if not done[s] and want_len[s] < cap:
                want_k[s, want_len[s]] = k_steps[row, s]
                want_len[s] += 1
        assert lens.tolist() == want_len and finished.tolist() == [int(x) for x in done]
        assert torch.equal(k_suffix, want_k)
        result.fill_(100 + t)                                      # "the step's result"
    assert (result_steps >= 100).all() and (lens_steps >= 0).all()
    assert want_len == [2, 5, 5]
