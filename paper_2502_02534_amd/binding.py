"""ctypes binding of libspdecode.so: argument marshalling only.

Every function here has the name and argument order of the C entry point it
calls (see include/spdecode.h).  Tensors are torch tensors on the GPU; the
binding passes their device pointers and the current torch stream.  There is no
fallback: if the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libspdecode.so")

SPD_OK = 0
SPD_F32, SPD_BF16 = 0, 1
STAGE_PREFIX, STAGE_SUFFIX, STAGE_MERGE = 1, 2, 4

_lib = None


class SpdError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


class AttnDesc(ctypes.Structure):
    _fields_ = [("dtype", ctypes.c_int32), ("num_q_heads", ctypes.c_int32),
                ("num_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("num_prompts", ctypes.c_int32), ("num_samples", ctypes.c_int32),
                ("max_samples_per_prompt", ctypes.c_int32), ("page_size", ctypes.c_int32),
                ("sm_scale", ctypes.c_float), ("stages", ctypes.c_uint32)]


class PrefixLevel(ctypes.Structure):
    _fields_ = [("k", ctypes.c_void_p), ("v", ctypes.c_void_p), ("lens", ctypes.c_void_p),
                ("indptr", ctypes.c_void_p), ("page_indices", ctypes.c_void_p),
                ("sample_indptr", ctypes.c_void_p), ("num_groups", ctypes.c_int32),
                ("max_samples_per_group", ctypes.c_int32), ("max_len", ctypes.c_int64)]


class RowCopy(ctypes.Structure):
    _fields_ = [("src", ctypes.c_void_p), ("dst", ctypes.c_void_p), ("row_bytes", ctypes.c_int64)]


def load() -> ctypes.CDLL:
    """Load the HIP library.  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it first (paper_2502_02534_amd/csrc/build.sh "
                           "or __graft_entry__.build()); there is no fallback path")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i64, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_size_t
    dp = ctypes.POINTER(AttnDesc)
    lib.spd_status_string.restype = ctypes.c_char_p
    lib.spd_status_string.argtypes = [ctypes.c_int]
    lib.spd_attn_plan.restype = ctypes.c_int
    lib.spd_attn_plan.argtypes = [dp, i64, i64] + [ctypes.POINTER(ctypes.c_int32)] * 4
    lib.shared_prefix_decode_attn_workspace_size.restype = sz
    lib.shared_prefix_decode_attn_workspace_size.argtypes = [dp, i64, i64]
    lib.shared_prefix_decode_attn.restype = ctypes.c_int
    lib.shared_prefix_decode_attn.argtypes = [dp] + [vp] * 12 + [i64, i64, vp, vp, vp, sz, vp]
    lib.sample_tokens_workspace_size.restype = sz
    lib.sample_tokens_workspace_size.argtypes = [i64, i64]
    lib.sample_tokens.restype = ctypes.c_int
    lib.sample_tokens.argtypes = [vp, ctypes.c_int32, i64, i64, i64, vp, vp, vp, vp, vp, sz, vp]
    lib.sample_tokens_static.restype = ctypes.c_int
    lib.sample_tokens_static.argtypes = [vp, ctypes.c_int32, i64, i64, i64, vp, vp, vp, vp, vp]
    lib.sample_tokens_filtered.restype = ctypes.c_int
    lib.sample_tokens_filtered.argtypes = [vp, ctypes.c_int32, i64, i64, i64, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lp = ctypes.POINTER(PrefixLevel)
    lib.shared_prefix_decode_attn_levels_workspace_size.restype = sz
    lib.shared_prefix_decode_attn_levels_workspace_size.argtypes = [dp, ctypes.c_int32, lp, i64]
    lib.shared_prefix_decode_attn_levels.restype = ctypes.c_int
    lib.shared_prefix_decode_attn_levels.argtypes = [dp, vp, ctypes.c_int32, lp] + [vp] * 5 + [i64, vp, vp, vp, sz, vp]
    lib.append_suffix_kv.restype = ctypes.c_int
    lib.append_suffix_kv.argtypes = [dp] + [vp] * 7 + [i64, vp, ctypes.c_int32, vp, vp]
    for fn in (lib.decode_step_select, lib.decode_step_record):
        fn.restype = ctypes.c_int
        fn.argtypes = [vp, i64, ctypes.c_int32, ctypes.POINTER(RowCopy), vp]
    lib.decode_step_advance.restype = ctypes.c_int
    lib.decode_step_advance.argtypes = ([vp, i64, ctypes.c_int32, ctypes.POINTER(RowCopy), ctypes.c_int32,
                                         ctypes.POINTER(RowCopy), dp] + [vp] * 7 +
                                        [i64, vp, ctypes.c_int32, vp, vp, vp])
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load().spd_status_string(status).decode()


def _ptr(t: Optional[torch.Tensor]):
    return ctypes.c_void_p(0 if t is None else t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def make_desc(*, dtype: int, num_q_heads: int, num_kv_heads: int, head_dim: int, num_prompts: int,
              num_samples: int, max_samples_per_prompt: int = 0, page_size: int = 0,
              sm_scale: float = 0.0, stages: int = 0) -> AttnDesc:
    return AttnDesc(dtype, num_q_heads, num_kv_heads, head_dim, num_prompts, num_samples,
                    max_samples_per_prompt, page_size, sm_scale, stages)


def spd_attn_plan(desc: AttnDesc, max_prefix_len: int, max_suffix_len: int):
    vals = [ctypes.c_int32() for _ in range(4)]
    rc = load().spd_attn_plan(ctypes.byref(desc), max_prefix_len, max_suffix_len,
                              *[ctypes.byref(v) for v in vals])
    if rc != SPD_OK:
        raise SpdError(rc, "spd_attn_plan")
    return tuple(v.value for v in vals)


def shared_prefix_decode_attn_workspace_size(desc: AttnDesc, max_prefix_len: int, max_suffix_len: int) -> int:
    return int(load().shared_prefix_decode_attn_workspace_size(ctypes.byref(desc), max_prefix_len, max_suffix_len))


def shared_prefix_decode_attn(desc: AttnDesc, q, k_prefix, v_prefix, prefix_lens, prefix_indptr,
                              prefix_page_indices, sample_indptr, k_suffix, v_suffix, suffix_lens,
                              suffix_page_indptr, suffix_page_indices, max_prefix_len: int,
                              max_suffix_len: int, out, lse_out, workspace, stream=None) -> None:
    rc = load().shared_prefix_decode_attn(
        ctypes.byref(desc), _ptr(q), _ptr(k_prefix), _ptr(v_prefix), _ptr(prefix_lens),
        _ptr(prefix_indptr), _ptr(prefix_page_indices), _ptr(sample_indptr), _ptr(k_suffix),
        _ptr(v_suffix), _ptr(suffix_lens), _ptr(suffix_page_indptr), _ptr(suffix_page_indices),
        int(max_prefix_len), int(max_suffix_len), _ptr(out), _ptr(lse_out), _ptr(workspace),
        0 if workspace is None else workspace.numel() * workspace.element_size(), _stream(stream))
    if rc != SPD_OK:
        raise SpdError(rc, "shared_prefix_decode_attn")


def sample_tokens_workspace_size(rows: int, vocab: int) -> int:
    return int(load().sample_tokens_workspace_size(rows, vocab))


def sample_tokens(logits, logits_dtype: int, rows: int, vocab: int, row_stride: int, temperature,
                  top_p, uniforms, tokens_out, workspace, stream=None) -> None:
    rc = load().sample_tokens(
        _ptr(logits), logits_dtype, int(rows), int(vocab), int(row_stride), _ptr(temperature),
        _ptr(top_p), _ptr(uniforms), _ptr(tokens_out), _ptr(workspace),
        0 if workspace is None else workspace.numel() * workspace.element_size(), _stream(stream))
    if rc != SPD_OK:
        raise SpdError(rc, "sample_tokens")


def sample_tokens_static(logits, logits_dtype: int, rows: int, vocab: int, row_stride: int, temperature,
                         top_p, uniforms, tokens_out, stream=None) -> None:
    rc = load().sample_tokens_static(
        _ptr(logits), logits_dtype, int(rows), int(vocab), int(row_stride), _ptr(temperature),
        _ptr(top_p), _ptr(uniforms), _ptr(tokens_out), _stream(stream))
    if rc != SPD_OK:
        raise SpdError(rc, "sample_tokens_static")


def append_suffix_kv(desc: AttnDesc, k_new, v_new, k_suffix, v_suffix, suffix_lens, suffix_page_indptr,
                     suffix_page_indices, max_suffix_len: int, last_tokens=None, end_token: int = -1,
                     finished=None, stream=None) -> None:
    rc = load().append_suffix_kv(
        ctypes.byref(desc), _ptr(k_new), _ptr(v_new), _ptr(k_suffix), _ptr(v_suffix), _ptr(suffix_lens),
        _ptr(suffix_page_indptr), _ptr(suffix_page_indices), int(max_suffix_len), _ptr(last_tokens),
        int(end_token), _ptr(finished), _stream(stream))
    if rc != SPD_OK:
        raise SpdError(rc, "append_suffix_kv")


def make_row_copies(pairs):
    """ctypes array of RowCopy from (src tensor, dst tensor, bytes per row) triples."""
    arr = (RowCopy * len(pairs))()
    for i, (src, dst, row_bytes) in enumerate(pairs):
        arr[i] = RowCopy(src.data_ptr(), dst.data_ptr(), int(row_bytes))
    return arr


def decode_step_select(step_state, num_steps: int, copies, stream=None) -> None:
    rc = load().decode_step_select(_ptr(step_state), int(num_steps), len(copies), copies, _stream(stream))
    if rc != SPD_OK:
        raise SpdError(rc, "decode_step_select")


def decode_step_record(step_state, num_steps: int, copies, stream=None) -> None:
    rc = load().decode_step_record(_ptr(step_state), int(num_steps), len(copies), copies, _stream(stream))
    if rc != SPD_OK:
        raise SpdError(rc, "decode_step_record")


def decode_step_advance(step_state, num_steps: int, record, select, desc: AttnDesc, k_steps, v_steps, k_suffix,
                        v_suffix, suffix_lens, suffix_page_indptr, suffix_page_indices, max_suffix_len: int,
                        last_tokens=None, end_token: int = -1, finished=None, lens_record=None, stream=None) -> None:
    """`record` / `select`: ctypes arrays from make_row_copies, or None for no copies of that kind."""
    rc = load().decode_step_advance(
        _ptr(step_state), int(num_steps), 0 if record is None else len(record), record,
        0 if select is None else len(select), select, ctypes.byref(desc), _ptr(k_steps), _ptr(v_steps),
        _ptr(k_suffix), _ptr(v_suffix), _ptr(suffix_lens), _ptr(suffix_page_indptr), _ptr(suffix_page_indices),
        int(max_suffix_len), _ptr(last_tokens), int(end_token), _ptr(finished), _ptr(lens_record), _stream(stream))
    if rc != SPD_OK:
        raise SpdError(rc, "decode_step_advance")


def make_levels(levels):
    """ctypes array of PrefixLevel from records with tensor fields k, v, lens, indptr, sample_indptr
    (and optionally page_indices) plus max_samples_per_group and max_len."""
    arr = (PrefixLevel * len(levels))()
    for i, lv in enumerate(levels):
        pages = getattr(lv, "page_indices", None)
        arr[i] = PrefixLevel(lv.k.data_ptr(), lv.v.data_ptr(), lv.lens.data_ptr(), lv.indptr.data_ptr(),
                             0 if pages is None else pages.data_ptr(), lv.sample_indptr.data_ptr(),
                             int(lv.lens.numel()), int(lv.max_samples_per_group), int(lv.max_len))
    return arr


def shared_prefix_decode_attn_levels_workspace_size(desc: AttnDesc, levels, max_suffix_len: int) -> int:
    return int(load().shared_prefix_decode_attn_levels_workspace_size(ctypes.byref(desc), len(levels), levels,
                                                                      int(max_suffix_len)))


def shared_prefix_decode_attn_levels(desc: AttnDesc, q, levels, k_suffix, v_suffix, suffix_lens,
                                     suffix_page_indptr, suffix_page_indices, max_suffix_len: int, out, lse_out,
                                     workspace, stream=None) -> None:
    rc = load().shared_prefix_decode_attn_levels(
        ctypes.byref(desc), _ptr(q), len(levels), levels, _ptr(k_suffix), _ptr(v_suffix), _ptr(suffix_lens),
        _ptr(suffix_page_indptr), _ptr(suffix_page_indices), int(max_suffix_len), _ptr(out), _ptr(lse_out),
        _ptr(workspace), 0 if workspace is None else workspace.numel() * workspace.element_size(),
        _stream(stream))
    if rc != SPD_OK:
        raise SpdError(rc, "shared_prefix_decode_attn_levels")


def sample_tokens_filtered(logits, logits_dtype: int, rows: int, vocab: int, row_stride: int, temperature,
                           top_p, top_k, min_p, uniforms, tokens_out, workspace, stream=None) -> None:
    rc = load().sample_tokens_filtered(
        _ptr(logits), logits_dtype, int(rows), int(vocab), int(row_stride), _ptr(temperature), _ptr(top_p),
        _ptr(top_k), _ptr(min_p), _ptr(uniforms), _ptr(tokens_out), _ptr(workspace),
        0 if workspace is None else workspace.numel() * workspace.element_size(), _stream(stream))
    if rc != SPD_OK:
        raise SpdError(rc, "sample_tokens_filtered")
