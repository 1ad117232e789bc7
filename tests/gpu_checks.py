"""Comparison rules shared by the GPU parity tests (HIP library through its C ABI against the fp64
checker on the same seeded inputs).

Attention
  bf16 output : contractual bound |gpu - ref| <= 2e-2 elementwise wherever |ref| <= 2 (above 2 the
                bf16 grid of the output itself is coarser: half a unit in the last place is 7.8e-3
                in [2, 4) and 1.6e-2 in [4, 8)), and beside it, for every element, a regression bound
                |gpu - ref| <= 2e-3 + 2^-7 * (largest |ref| of the output row): the result is rounded
                to bf16 once (up to 2^-8 relative), the probabilities once more on their way into the
                second product (2^-9 relative on terms as large as the row's values), the stored
                partial states to fp16.  Averaged outputs of magnitude 0.03 are observed at
                3e-4 .. 1.2e-3, peaked ones (|o| of 1 to 5) at 0.5 .. 0.9 of the regression bound.
  fp32 output : |gpu - ref| <= 1e-5 |ref| + 1e-6 elementwise
  log-sum-exp : |gpu - ref| <= 1e-4 (fp32) / 2.1e-3 (bf16 inputs), -inf exactly where the checker has it
Tokens
  identical to the checker's.  A row may differ only if its uniform lies within 1e-6 of a boundary of
  the checker's CDF, or a threshold (nucleus cut, min-p, top-k) lies within 1e-6 (relative) of a
  value that fp32 and fp64 may order differently; such rows are counted, and the number of them
  that actually differ is bounded by `allow_exempt_mismatch` (0 unless a case states otherwise).
"""
import numpy as np
import torch

BF16_ABS = 2e-2


def attention_errors(got, ref, dtype):
    """Asserts the elementwise bounds; returns the largest absolute error."""
    assert np.all(np.isfinite(got)), "non-finite output"
    err = np.abs(got - ref)
    if dtype == "f32":
        assert np.all(err <= 1e-5 * np.abs(ref) + 1e-6), f"max err {err.max():.3e}"
    else:
        small = np.abs(ref) <= 2.0
        assert np.all(err[small] <= BF16_ABS), f"max err {err[small].max():.3e} beyond the contractual bound"
        reg = np.broadcast_to(2e-3 + 2.0 ** -7 * np.abs(ref).max(axis=-1, keepdims=True), err.shape)
        worst = int(np.argmax(err - reg))
        assert np.all(err <= reg), (f"regression bound: err {err.flat[worst]:.3e} at |ref| "
                                    f"{abs(ref.flat[worst]):.3e} (max err {err.max():.3e})")
    return float(err.max()) if err.size else 0.0


def lse_errors(lse, ref_lse, dtype):
    fin = np.isfinite(ref_lse)
    assert np.array_equal(np.isneginf(lse), np.isneginf(ref_lse))
    tol = 1e-4 + (0 if dtype == "f32" else 2e-3)
    assert np.all(np.abs(lse[fin] - ref_lse[fin]) <= tol), np.abs(lse[fin] - ref_lse[fin]).max()


def check_attention(dev, oracle, inp, rows=None, stages=0, poison_workspace=True):
    """Runs the attention call on `inp` and compares with the checker (all rows, or the flat
    (sample, head) rows listed in `rows`)."""
    d = dev.upload_attn(inp)
    d.out.fill_(float("nan"))
    d.lse.fill_(float("nan"))
    if poison_workspace:
        d.workspace.view(torch.float32)[: d.workspace.numel() // 4].fill_(float("nan"))
    d.run(stages)
    torch.cuda.synchronize()
    got = d.out.float().cpu().numpy().astype(np.float64)
    lse = d.lse.cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(got)), "non-finite output somewhere in the full result"
    D = inp.spec.head_dim
    if rows is None:
        ref, ref_lse = oracle.attention_inputs(inp)
    else:
        ref, ref_lse = oracle.attention_inputs(inp, rows=rows)
        got = got.reshape(-1, D)[rows]
        lse = lse.reshape(-1)[rows]
    err = attention_errors(got, ref, inp.spec.dtype)
    lse_errors(lse, ref_lse, inp.spec.dtype)
    del d
    return err


def compare_tokens(tok, o, uniforms, vocab, allow_exempt_mismatch=0, extra_exempt=None, label=""):
    """`o` is the checker's record.  Returns (exempt near a CDF boundary, exempt near a threshold,
    differing)."""
    u = np.asarray(uniforms).astype(np.float64)
    near_cdf = np.minimum(np.abs(u - o["cdf_lo"]), np.abs(u - o["cdf_hi"])) < 1e-6
    near_cut = o["cut_margin"] < 1e-6
    if "filter_margin" in o:
        near_cut = near_cut | (o["filter_margin"] < 1e-6)
    if extra_exempt is not None:
        near_cut = near_cut | extra_exempt
    mism = tok != o["token"]
    hard = mism & ~near_cdf & ~near_cut
    print(f"  {label}rows {len(tok)}: exempt near-CDF {int(near_cdf.sum())}, near a threshold "
          f"{int(near_cut.sum())}, differing tokens {int(mism.sum())}", flush=True)
    assert not hard.any(), (np.nonzero(hard)[0][:8], tok[hard][:8], o["token"][hard][:8])
    assert int(mism.sum()) <= allow_exempt_mismatch, \
        (f"{int(mism.sum())} exempt rows differ (allowed {allow_exempt_mismatch})",
         np.nonzero(mism)[0][:8], tok[mism][:8], o["token"][mism][:8])
    assert np.all((tok >= 0) & (tok < vocab))
    return int(near_cdf.sum()), int(near_cut.sum()), int(mism.sum())


def check_tokens(dev, oracle, sin, row_stride=None, allow_exempt_mismatch=0):
    ds = dev.upload_sampler(sin, row_stride=row_stride, pad_value=1e30)
    ds.tokens.fill_(-7)
    ds.run()
    torch.cuda.synchronize()
    tok = ds.tokens.cpu().numpy()
    o = oracle.sample_tokens(sin.logits, sin.temperature, sin.top_p, sin.uniforms)
    del ds
    return compare_tokens(tok, o, sin.uniforms, sin.logits.shape[1], allow_exempt_mismatch)
