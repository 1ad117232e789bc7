"""fp64 CPU checker for the decode-step library.  TEST INFRASTRUCTURE ONLY.

Nothing under the product package may import this.  The arithmetic is in the
C files next to this one (plain loops, fp64); this module compiles them with
gcc and hands numpy arrays to them through ctypes.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "liboracle.so")
_SRCS = [os.path.join(_HERE, f) for f in ("attention_oracle.c", "sampler_oracle.c", "sampler_filtered_oracle.c")]
_lib = None


def build(force: bool = False) -> str:
    """Compile the checker (gcc -O2 -fopenmp).  Returns the library path."""
    stale = force or not os.path.exists(_SO) or any(
        os.path.getmtime(s) > os.path.getmtime(_SO) for s in _SRCS)
    if stale:
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fno-fast-math", "-shared", "-fPIC",
                               "-o", _SO] + _SRCS + ["-lm"])
    return _SO


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_attention.restype = ctypes.c_int
        _lib.oracle_sample_tokens.restype = ctypes.c_int
        _lib.oracle_sample_tokens_filtered.restype = ctypes.c_int
    return _lib


def _p(a: Optional[np.ndarray]):
    if a is None:
        return ctypes.c_void_p(0)
    assert a.flags["C_CONTIGUOUS"]
    return ctypes.c_void_p(a.ctypes.data)


def _i32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.int32)


def attention(q, k_prefix, v_prefix, prefix_lens, prefix_indptr, sample_indptr,
              k_suffix, v_suffix, suffix_lens, max_suffix_len, *, dtype: str,
              page_size: int = 0, prefix_page_indices=None, suffix_page_indptr=None,
              suffix_page_indices=None, scale: Optional[float] = None, rows=None):
    """softmax(q K^T * scale) V over [prefix | suffix] per (sample, query head), in fp64.

    Arrays are as laid out by the workload generator (bf16 carried as uint16).
    `rows` optionally selects flat (n * Hq + h) rows.  Returns (out, lse) with
    out float64 [rows, D] (or [N, Hq, D]) and lse float64 [rows] (or [N, Hq]).
    """
    lib = _load()
    N, Hq, D = q.shape
    Hkv = k_prefix.shape[1]
    B = len(prefix_lens)
    code = {"f32": 0, "bf16": 1}[dtype]
    want = np.float32 if code == 0 else np.uint16
    for a in (q, k_prefix, v_prefix, k_suffix, v_suffix):
        assert a.dtype == want, (a.dtype, want)
    sc = float(scale) if scale is not None else 1.0 / np.sqrt(float(D))
    rows_arr = None if rows is None else np.ascontiguousarray(rows, dtype=np.int64)
    nrows = N * Hq if rows_arr is None else len(rows_arr)
    out = np.empty((nrows, D), dtype=np.float64)
    lse = np.empty(nrows, dtype=np.float64)
    keep = [_i32(prefix_lens), _i32(prefix_indptr), _i32(prefix_page_indices), _i32(sample_indptr),
            _i32(suffix_lens), _i32(suffix_page_indptr), _i32(suffix_page_indices)]
    rc = lib.oracle_attention(
        ctypes.c_int(code), ctypes.c_int(N), ctypes.c_int(Hq), ctypes.c_int(Hkv), ctypes.c_int(D),
        ctypes.c_int(B), ctypes.c_int(page_size), ctypes.c_double(sc),
        _p(np.ascontiguousarray(q)), _p(np.ascontiguousarray(k_prefix)),
        _p(np.ascontiguousarray(v_prefix)), _p(keep[0]), _p(keep[1]), _p(keep[2]), _p(keep[3]),
        _p(np.ascontiguousarray(k_suffix)), _p(np.ascontiguousarray(v_suffix)), _p(keep[4]),
        ctypes.c_int64(int(max_suffix_len)), _p(keep[5]), _p(keep[6]),
        _p(rows_arr), ctypes.c_int64(nrows), _p(out), _p(lse))
    if rc != 0:
        raise ValueError("oracle_attention: inconsistent arguments")
    if rows is None:
        return out.reshape(N, Hq, D), lse.reshape(N, Hq)
    return out, lse


def attention_inputs(inp, rows=None):
    """`attention` on a workload-generator AttnInputs record."""
    sp = inp.spec
    return attention(inp.q, inp.k_prefix, inp.v_prefix, inp.prefix_lens, inp.prefix_indptr,
                     inp.sample_indptr, inp.k_suffix, inp.v_suffix, inp.suffix_lens,
                     inp.max_suffix_len, dtype=sp.dtype, page_size=sp.page_size,
                     prefix_page_indices=inp.prefix_page_indices,
                     suffix_page_indptr=inp.suffix_page_indptr,
                     suffix_page_indices=inp.suffix_page_indices, rows=rows)


def sample_tokens(logits, temperature, top_p, uniforms):
    """Serial temperature / nucleus / inverse-CDF sampling per row, in fp64.

    Returns a dict: token int32 [rows]; cdf_lo, cdf_hi float64 [rows] (the
    normalised running kept mass before and after the returned token);
    cut_margin float64 [rows] (relative distance of the nucleus cut from
    top_p * S, inf when nothing is cut); kept int32 [rows].
    """
    lib = _load()
    logits = np.ascontiguousarray(logits, dtype=np.float32)
    rows, vocab = logits.shape
    t = np.ascontiguousarray(temperature, dtype=np.float32)
    tp = np.ascontiguousarray(top_p, dtype=np.float32)
    u = np.ascontiguousarray(uniforms, dtype=np.float32)
    assert t.shape == (rows,) and tp.shape == (rows,) and u.shape == (rows,)
    tok = np.empty(rows, dtype=np.int32)
    lo = np.empty(rows, dtype=np.float64)
    hi = np.empty(rows, dtype=np.float64)
    mg = np.empty(rows, dtype=np.float64)
    kept = np.empty(rows, dtype=np.int32)
    rc = lib.oracle_sample_tokens(_p(logits), ctypes.c_int64(rows), ctypes.c_int64(vocab),
                                  ctypes.c_int64(vocab), _p(t), _p(tp), _p(u),
                                  _p(tok), _p(lo), _p(hi), _p(mg), _p(kept))
    if rc != 0:
        raise ValueError("oracle_sample_tokens: inconsistent arguments")
    return {"token": tok, "cdf_lo": lo, "cdf_hi": hi, "cut_margin": mg, "kept": kept}


def sample_tokens_filtered(logits, temperature, top_p, uniforms, top_k=None, min_p=None):
    """Sampling with min-p, top-k and top-p filters applied in that order, per row, in fp64.

    `top_k` int32 [rows] (0 = off) and `min_p` float32 [rows] (0 = off) may be None.  Returns
    the dict of `sample_tokens` plus filter_margin float64 [rows] (relative distance between a
    filter threshold and the nearest probability not exactly on it; inf when no filter acts).
    """
    lib = _load()
    logits = np.ascontiguousarray(logits, dtype=np.float32)
    rows, vocab = logits.shape
    t = np.ascontiguousarray(temperature, dtype=np.float32)
    tp = np.ascontiguousarray(top_p, dtype=np.float32)
    u = np.ascontiguousarray(uniforms, dtype=np.float32)
    tk = None if top_k is None else np.ascontiguousarray(top_k, dtype=np.int32)
    mp = None if min_p is None else np.ascontiguousarray(min_p, dtype=np.float32)
    assert t.shape == (rows,) and tp.shape == (rows,) and u.shape == (rows,)
    tok = np.empty(rows, dtype=np.int32)
    lo = np.empty(rows, dtype=np.float64)
    hi = np.empty(rows, dtype=np.float64)
    mg = np.empty(rows, dtype=np.float64)
    fm = np.empty(rows, dtype=np.float64)
    kept = np.empty(rows, dtype=np.int32)
    rc = lib.oracle_sample_tokens_filtered(_p(logits), ctypes.c_int64(rows), ctypes.c_int64(vocab),
                                           ctypes.c_int64(vocab), _p(t), _p(tp), _p(tk), _p(mp), _p(u),
                                           _p(tok), _p(lo), _p(hi), _p(mg), _p(fm), _p(kept))
    if rc != 0:
        raise ValueError("oracle_sample_tokens_filtered: inconsistent arguments")
    return {"token": tok, "cdf_lo": lo, "cdf_hi": hi, "cut_margin": mg, "filter_margin": fm, "kept": kept}
