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
