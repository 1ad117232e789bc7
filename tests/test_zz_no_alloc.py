"""`sample_tokens_static` (the entry point that allocates nothing: its scratch memory is an array
inside the library) against `sample_tokens` with a caller's workspace, through the C ABI: the same
tokens on two calls in a row, the second on a smaller input; sizes beyond the array are refused."""
import numpy as np
import pytest

from paper_2502_02534_amd import workloads as W

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _case(rows, vocab, seed, T, top_p):
    rng = np.random.default_rng(seed)
    x = (rng.standard_normal((rows, vocab)) * 3).astype(np.float32)
    return W.SamplerInputs(x, np.full(rows, T, np.float32), np.full(rows, top_p, np.float32),
                           rng.random(rows, dtype=np.float32))


def test_static_scratch_entry_point_matches_workspace_entry_point(oracle):
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2502_02534_amd import binding as B
    from paper_2502_02534_amd import device
    B.load()
    from gpu_checks import compare_tokens
    for rows, vocab, seed, T, top_p in ((48, 128256, 1, 1.0, 0.95), (5, 20011, 2, 0.7, 0.9), (64, 32000, 3, 0.8, 1.0)):
        print(f"static scratch: rows {rows} vocab {vocab}", flush=True)
        sin = _case(rows, vocab, seed, T, top_p)
        ds = device.upload_sampler(sin)
        ds.tokens.fill_(-7)
        ds.run()                                   # sample_tokens with a caller's workspace
        torch.cuda.synchronize()
        want = ds.tokens.cpu().numpy().copy()
        got = torch.full((rows,), -9, dtype=torch.int32, device="cuda")
        B.sample_tokens_static(ds.logits, B.SPD_F32, rows, vocab, ds.logits.stride(0), ds.temperature, ds.top_p,
                               ds.uniforms, got)
        torch.cuda.synchronize()
        assert np.array_equal(got.cpu().numpy(), want)
        compare_tokens(want, oracle.sample_tokens(sin.logits, sin.temperature, sin.top_p, sin.uniforms),
                       sin.uniforms, vocab)
    # beyond the library's array: refused, nothing launched
    big = torch.zeros((200, 128256), dtype=torch.float32, device="cuda")
    t = torch.ones(200, device="cuda")
    tok = torch.full((200,), -9, dtype=torch.int32, device="cuda")
    with pytest.raises(B.SpdError) as e:
        B.sample_tokens_static(big, B.SPD_F32, 200, 128256, 128256, t, t, t, tok)
    assert e.value.status == 3
    torch.cuda.synchronize()
    assert int((tok != -9).sum()) == 0
