"""ctypes front end of the fp64 CPU oracle (paged_attention_oracle.cpp).

TEST INFRASTRUCTURE ONLY: reached from tests/, the smoke check and the
benchmark's CPU-baseline leg, never from the product path.  Shares nothing
with the GPU library; it only marshals arrays into the C++ routine, which is
the scaled-dot-product definition the paper cites in section 2 ("Phases of LLM
inference") evaluated over a block-structured KV cache (section 5.2).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "paged_attention_oracle.cpp")
_LIB = os.path.join(_HERE, "liboserve_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with g++ (single-threaded, strict IEEE: no -ffast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["g++", "-O2", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off",
                               "-o", _LIB, _SRC])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i64, i32, vp = ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p
        lib.oserve_oracle_paged_decode_attn.restype = ctypes.c_int
        lib.oserve_oracle_paged_decode_attn.argtypes = [
            vp, i64, i64, vp, vp, i64, i64, i64, i64, vp, i64, vp,
            i32, i32, i32, i32, i32, ctypes.c_float, vp, vp]
        lib.oserve_oracle_one_head.restype = ctypes.c_int
        lib.oserve_oracle_one_head.argtypes = [
            vp, i64, i64, vp, vp, i64, i64, i64, i64, vp, i64, vp,
            i32, i32, i32, i32, ctypes.c_float, i32, i32, vp, vp]
        lib.oserve_oracle_paged_prefill_attn.restype = ctypes.c_int
        lib.oserve_oracle_paged_prefill_attn.argtypes = [
            vp, i64, i64, vp, vp, i64, i64, i64, i64, vp, i64, vp, vp,
            i32, i32, i32, i32, i32, ctypes.c_float, vp]
        _lib = lib
    return _lib


def _bits(x) -> np.ndarray:
    """bf16 payload as a uint16 numpy array (no copy when possible).

    Accepts a numpy uint16 array (already bit patterns) or a torch CPU bf16
    tensor.
    """
    if isinstance(x, np.ndarray):
        if x.dtype != np.uint16:
            raise TypeError("numpy input must hold bf16 bit patterns as uint16")
        return x
    import torch
    if x.dtype != torch.bfloat16 or x.device.type != "cpu":
        raise TypeError("expected a CPU bf16 tensor")
    return x.view(torch.int16).numpy().view(np.uint16)


def _i32(x) -> np.ndarray:
    if not isinstance(x, np.ndarray):
        x = x.numpy()
    if x.dtype != np.int32:
        raise TypeError("expected int32")
    return x


def _elem_strides(a: np.ndarray):
    return [s // a.itemsize for s in a.strides]


def _check_kv(k: np.ndarray, v: np.ndarray):
    if k.ndim != 4 or k.shape != v.shape or k.strides != v.strides:
        raise ValueError("k_pages / v_pages must be 4-D [pages, kv_heads, page, dim] with equal strides")
    if _elem_strides(k)[3] != 1:
        raise ValueError("head_dim must be the unit-stride axis")


def paged_decode_attn(q, k_pages, v_pages, block_table, context_lens, scale: float,
                      return_lse: bool = False):
    """Oracle output, double [B, Hq, D] (and lse double [B, Hq] if asked)."""
    lib = _load()
    qb, kb, vb = _bits(q), _bits(k_pages), _bits(v_pages)
    bt, cl = _i32(block_table), _i32(context_lens)
    _check_kv(kb, vb)
    B, Hq, D = qb.shape
    P, Hkv, page, Dk = kb.shape
    if Dk != D or _elem_strides(qb)[2] != 1 or bt.ndim != 2 or bt.shape[0] != B or cl.shape != (B,):
        raise ValueError("shape mismatch")
    if not cl.flags.c_contiguous or _elem_strides(bt)[1] != 1:
        raise ValueError("context_lens / block_table rows must be contiguous")
    if B and int(cl.max()) > bt.shape[1] * page:
        raise ValueError("context length exceeds block table width")
    out = np.empty((B, Hq, D), dtype=np.float64)
    lse = np.empty((B, Hq), dtype=np.float64) if return_lse else None
    qs, ks = _elem_strides(qb), _elem_strides(kb)
    rc = lib.oserve_oracle_paged_decode_attn(
        qb.ctypes.data, qs[0], qs[1], kb.ctypes.data, vb.ctypes.data, P, ks[0], ks[1], ks[2],
        bt.ctypes.data, _elem_strides(bt)[0], cl.ctypes.data, B, Hq, Hkv, D, page,
        ctypes.c_float(scale), out.ctypes.data, lse.ctypes.data if return_lse else None)
    if rc != 0:
        raise ValueError(f"oracle rejected its input (code {rc})")
    return (out, lse) if return_lse else out


def one_head(q, k_pages, v_pages, block_table, context_lens, scale: float, b: int, h: int):
    """Oracle output row for one (request, query head): double [D]."""
    lib = _load()
    qb, kb, vb = _bits(q), _bits(k_pages), _bits(v_pages)
    bt, cl = _i32(block_table), _i32(context_lens)
    _check_kv(kb, vb)
    B, Hq, D = qb.shape
    P, Hkv, page, _ = kb.shape
    out = np.empty((D,), dtype=np.float64)
    qs, ks = _elem_strides(qb), _elem_strides(kb)
    rc = lib.oserve_oracle_one_head(
        qb.ctypes.data, qs[0], qs[1], kb.ctypes.data, vb.ctypes.data, P, ks[0], ks[1], ks[2],
        bt.ctypes.data, _elem_strides(bt)[0], cl.ctypes.data, Hq, Hkv, D, page,
        ctypes.c_float(scale), b, h, out.ctypes.data, None)
    if rc != 0:
        raise ValueError(f"oracle rejected its input (code {rc})")
    return out


def paged_prefill_attn(q, k_pages, v_pages, block_table, context_lens, q_lens, scale: float):
    """Causal chunked-prefill oracle: q is [sum(q_lens), Hq, D] (requests packed), output double of that shape."""
    lib = _load()
    qb, kb, vb = _bits(q), _bits(k_pages), _bits(v_pages)
    bt, cl, ql = _i32(block_table), _i32(context_lens), _i32(q_lens)
    _check_kv(kb, vb)
    T, Hq, D = qb.shape
    P, Hkv, page, Dk = kb.shape
    B = cl.shape[0]
    if Dk != D or _elem_strides(qb)[2] != 1 or bt.ndim != 2 or bt.shape[0] != B or ql.shape != (B,):
        raise ValueError("shape mismatch")
    if int(ql.sum()) != T:
        raise ValueError("q_lens must add up to the number of query rows")
    if not cl.flags.c_contiguous or not ql.flags.c_contiguous or _elem_strides(bt)[1] != 1:
        raise ValueError("context_lens / q_lens / block_table rows must be contiguous")
    if B and int(cl.max()) > bt.shape[1] * page:
        raise ValueError("context length exceeds block table width")
    out = np.empty((T, Hq, D), dtype=np.float64)
    qs, ks = _elem_strides(qb), _elem_strides(kb)
    rc = lib.oserve_oracle_paged_prefill_attn(
        qb.ctypes.data, qs[0], qs[1], kb.ctypes.data, vb.ctypes.data, P, ks[0], ks[1], ks[2],
        bt.ctypes.data, _elem_strides(bt)[0], cl.ctypes.data, ql.ctypes.data, B, Hq, Hkv, D, page,
        ctypes.c_float(scale), out.ctypes.data)
    if rc != 0:
        raise ValueError(f"oracle rejected its input (code {rc})")
    return out
