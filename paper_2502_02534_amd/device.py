"""Device-memory plumbing around the binding: moves a generated workload to the
GPU, allocates outputs and workspace with torch, and issues the library calls.
No arithmetic of the method happens here."""
from __future__ import annotations

import dataclasses
from typing import Optional

import numpy as np
import torch

from . import binding as B


def _dev(a: Optional[np.ndarray], device, bf16: bool = False):
    if a is None:
        return None
    t = torch.from_numpy(np.ascontiguousarray(a))
    if bf16:
        t = t.view(torch.int16).view(torch.bfloat16)
    return t.to(device)


@dataclasses.dataclass
class DeviceAttn:
    desc: B.AttnDesc
    q: torch.Tensor
    k_prefix: torch.Tensor
    v_prefix: torch.Tensor
    prefix_lens: torch.Tensor
    prefix_indptr: torch.Tensor
    prefix_page_indices: Optional[torch.Tensor]
    sample_indptr: torch.Tensor
    k_suffix: torch.Tensor
    v_suffix: torch.Tensor
    suffix_lens: torch.Tensor
    suffix_page_indptr: Optional[torch.Tensor]
    suffix_page_indices: Optional[torch.Tensor]
    max_prefix_len: int
    max_suffix_len: int
    out: torch.Tensor
    lse: torch.Tensor
    workspace: torch.Tensor

    def run(self, stages: int = 0, stream=None) -> None:
        self.desc.stages = stages
        B.shared_prefix_decode_attn(
            self.desc, self.q, self.k_prefix, self.v_prefix, self.prefix_lens, self.prefix_indptr,
            self.prefix_page_indices, self.sample_indptr, self.k_suffix, self.v_suffix,
            self.suffix_lens, self.suffix_page_indptr, self.suffix_page_indices,
            self.max_prefix_len, self.max_suffix_len, self.out, self.lse, self.workspace, stream)


def upload_attn(inp, device="cuda:0", workspace: Optional[torch.Tensor] = None) -> DeviceAttn:
    """Copy an AttnInputs record to the GPU and allocate output + workspace."""
    sp = inp.spec
    bf16 = sp.dtype == "bf16"
    paged = sp.page_size != 0
    desc = B.make_desc(dtype=B.SPD_BF16 if bf16 else B.SPD_F32, num_q_heads=sp.num_q_heads,
                       num_kv_heads=sp.num_kv_heads, head_dim=sp.head_dim,
                       num_prompts=sp.num_prompts, num_samples=sp.num_samples,
                       max_samples_per_prompt=sp.samples_per_prompt, page_size=sp.page_size)
    kp, vp = _dev(inp.k_prefix, device, bf16), _dev(inp.v_prefix, device, bf16)
    if paged and inp.k_suffix is inp.k_prefix:
        ks, vs = kp, vp
    else:
        ks, vs = _dev(inp.k_suffix, device, bf16), _dev(inp.v_suffix, device, bf16)
    N, Hq, D = inp.q.shape
    out = torch.empty((N, Hq, D), dtype=torch.bfloat16 if bf16 else torch.float32, device=device)
    lse = torch.empty((N, Hq), dtype=torch.float32, device=device)
    if workspace is None:
        nbytes = B.shared_prefix_decode_attn_workspace_size(desc, inp.max_prefix_len, inp.max_suffix_len)
        workspace = torch.empty(nbytes, dtype=torch.uint8, device=device)
    return DeviceAttn(desc, _dev(inp.q, device, bf16), kp, vp, _dev(inp.prefix_lens, device),
                      _dev(inp.prefix_indptr, device), _dev(inp.prefix_page_indices, device),
                      _dev(inp.sample_indptr, device), ks, vs, _dev(inp.suffix_lens, device),
                      _dev(inp.suffix_page_indptr, device), _dev(inp.suffix_page_indices, device),
                      inp.max_prefix_len, inp.max_suffix_len, out, lse, workspace)


@dataclasses.dataclass
class DeviceSampler:
    logits: torch.Tensor
    temperature: torch.Tensor
    top_p: torch.Tensor
    uniforms: torch.Tensor
    tokens: torch.Tensor
    workspace: torch.Tensor

    def run(self, stream=None) -> None:
        rows, vocab = self.logits.shape
        B.sample_tokens(self.logits, B.SPD_F32, rows, vocab, self.logits.stride(0), self.temperature,
                        self.top_p, self.uniforms, self.tokens, self.workspace, stream)


def upload_sampler(inp, device="cuda:0", row_stride=None, pad_value=float("nan")) -> DeviceSampler:
    """Uploads sampler inputs.  With `row_stride` > vocab the logits sit in a wider matrix whose
    extra columns hold `pad_value` (the kernels must never read them as logits)."""
    rows, vocab = inp.logits.shape
    ws = torch.empty(max(256, B.sample_tokens_workspace_size(rows, vocab)), dtype=torch.uint8, device=device)
    if row_stride is not None and row_stride != vocab:
        wide = torch.full((rows, row_stride), pad_value, dtype=torch.float32, device=device)
        wide[:, :vocab] = _dev(inp.logits, device)
        logits = wide[:, :vocab]  # a view: stride(0) == row_stride
    else:
        logits = _dev(inp.logits, device)
    return DeviceSampler(logits, _dev(inp.temperature, device), _dev(inp.top_p, device),
                         _dev(inp.uniforms, device), torch.empty(rows, dtype=torch.int32, device=device), ws)


class DecodeLoop:
    """A loop of decode steps on the device: append the step's K/V (synthetic: there are no
    weights), attention, sampling; lengths, finished flags and the step counter live on the
    device, so the steps can be replayed from a captured graph without host synchronisation.
    Every kernel of a step is one of the library's own launches.

    Per-step inputs are rows of tensors indexed by the device-side step counter:
      q_steps [steps, N, Hq, D], k_steps / v_steps [steps, N, Hkv, D], u_steps [steps, rows].
    The logits are the same every step (only the uniforms change); `tokens_steps`, `out_steps`
    and `lens_steps` record every step's results for checking."""

    def __init__(self, attn: DeviceAttn, sampler: DeviceSampler, q_steps, k_steps, v_steps, u_steps,
                 end_token: int = -1, one_launch: bool = True):
        self.attn, self.sampler = attn, sampler
        self.one_launch = one_launch
        self.q_steps, self.k_steps, self.v_steps, self.u_steps = q_steps, k_steps, v_steps, u_steps
        self.steps = q_steps.shape[0]
        dev = q_steps.device
        n = attn.q.shape[0]
        self.step = torch.zeros(3, dtype=torch.int64, device=dev)  # {current, next, arrivals}
        self.finished = torch.zeros(n, dtype=torch.int32, device=dev)
        self.end_token = end_token
        sampler.tokens.fill_(-1)  # "no token yet": never equal to an end token (>= 0)
        self.k_cur = torch.empty_like(k_steps[0])
        self.v_cur = torch.empty_like(v_steps[0])
        self.tokens_steps = torch.full((self.steps, sampler.tokens.shape[0]), -1, dtype=torch.int32, device=dev)
        self.out_steps = torch.zeros((self.steps,) + tuple(attn.out.shape), dtype=attn.out.dtype, device=dev)
        self.lens_steps = torch.zeros((self.steps, n), dtype=torch.int32, device=dev)
        nbytes = lambda t: t.numel() * t.element_size()
        self._select = B.make_row_copies([(q_steps, attn.q, nbytes(attn.q)), (k_steps, self.k_cur, nbytes(self.k_cur)),
                                          (v_steps, self.v_cur, nbytes(self.v_cur)),
                                          (u_steps, sampler.uniforms, nbytes(sampler.uniforms))])
        self._record = B.make_row_copies([(sampler.tokens, self.tokens_steps, nbytes(sampler.tokens)),
                                          (attn.out, self.out_steps, nbytes(attn.out)),
                                          (attn.suffix_lens, self.lens_steps, nbytes(attn.suffix_lens))])
        # one launch per step: the lengths are recorded by the append itself, K and V rows are read
        # straight from the step tensors
        self._select_qu = B.make_row_copies([(q_steps, attn.q, nbytes(attn.q)),
                                             (u_steps, sampler.uniforms, nbytes(sampler.uniforms))])
        self._record_to = B.make_row_copies([(sampler.tokens, self.tokens_steps, nbytes(sampler.tokens)),
                                             (attn.out, self.out_steps, nbytes(attn.out))])

    def one_step(self) -> None:
        """Enqueues one decode step on the current stream (capturable: kernel launches only).  With
        `one_launch` the results of a step are recorded by the next step's advance call, those of
        the last step by `flush`."""
        a, s = self.attn, self.sampler
        if self.one_launch:
            B.decode_step_advance(self.step, self.steps, self._record_to, self._select_qu, a.desc, self.k_steps,
                                  self.v_steps, a.k_suffix, a.v_suffix, a.suffix_lens, a.suffix_page_indptr,
                                  a.suffix_page_indices, a.max_suffix_len, s.tokens, self.end_token, self.finished,
                                  self.lens_steps)
            a.run()
            s.run()
            return
        B.decode_step_select(self.step, self.steps, self._select)
        B.append_suffix_kv(a.desc, self.k_cur, self.v_cur, a.k_suffix, a.v_suffix, a.suffix_lens,
                           a.suffix_page_indptr, a.suffix_page_indices, a.max_suffix_len,
                           s.tokens, self.end_token, self.finished)
        a.run()
        s.run()
        B.decode_step_record(self.step, self.steps, self._record)

    def flush(self) -> None:
        """After the last step of a `one_launch` loop: records that step's results."""
        if self.one_launch:
            B.decode_step_record(self.step, self.steps, self._record)


@dataclasses.dataclass
class DeviceLevel:
    k: torch.Tensor
    v: torch.Tensor
    lens: torch.Tensor
    indptr: torch.Tensor
    sample_indptr: torch.Tensor
    max_samples_per_group: int
    max_len: int


class DeviceCascade:
    """A CascadeInputs record on the GPU and the multi-level attention call on it."""

    def __init__(self, inp, device="cuda:0"):
        sp = inp.spec
        bf16 = sp.dtype == "bf16"
        n, hq, d = inp.q.shape
        self.desc = B.make_desc(dtype=B.SPD_BF16 if bf16 else B.SPD_F32, num_q_heads=hq,
                                num_kv_heads=sp.num_kv_heads, head_dim=d, num_prompts=1, num_samples=n)
        self.q = _dev(inp.q, device, bf16)
        self.levels = [DeviceLevel(_dev(lv.k, device, bf16), _dev(lv.v, device, bf16), _dev(lv.lens, device),
                                   _dev(lv.indptr, device), _dev(lv.sample_indptr, device),
                                   lv.max_samples_per_group, lv.max_len) for lv in inp.levels]
        self.level_array = B.make_levels(self.levels)
        self.k_suffix, self.v_suffix = _dev(inp.k_suffix, device, bf16), _dev(inp.v_suffix, device, bf16)
        self.suffix_lens = _dev(inp.suffix_lens, device)
        self.max_suffix_len = inp.max_suffix_len
        self.out = torch.empty((n, hq, d), dtype=torch.bfloat16 if bf16 else torch.float32, device=device)
        self.lse = torch.empty((n, hq), dtype=torch.float32, device=device)
        nbytes = B.shared_prefix_decode_attn_levels_workspace_size(self.desc, self.level_array, self.max_suffix_len)
        self.workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)

    def run(self, stream=None) -> None:
        B.shared_prefix_decode_attn_levels(self.desc, self.q, self.level_array, self.k_suffix, self.v_suffix,
                                           self.suffix_lens, None, None, self.max_suffix_len, self.out, self.lse,
                                           self.workspace, stream)
