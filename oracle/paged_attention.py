"""ctypes front of ``paged_attn_oracle.c`` (fp64 paged decode attention).

TEST INFRASTRUCTURE ONLY; see the header of the C file for what is computed
(paper Section 3.1: block-table gather, Q.K^T, softmax, logits.V).

Arrays are numpy; 16-bit floating inputs travel as raw ``uint16`` bit patterns
plus a dtype name ("f16" or "bf16") so no conversion happens outside the C file.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "paged_attn_oracle.c")
_LIB = os.path.join(_HERE, "libpaged_attn_oracle.so")
_lock = threading.Lock()
_lib = None

_DTYPES = {"f16": 0, "bf16": 1}


def build_oracle(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP over (b, h) pairs)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


def _load():
    global _lib
    with _lock:
        if _lib is None:
            lib = ctypes.CDLL(build_oracle())
            u16p = ctypes.POINTER(ctypes.c_uint16)
            i32p = ctypes.POINTER(ctypes.c_int32)
            f64p = ctypes.POINTER(ctypes.c_double)
            lib.oracle_paged_attention.restype = ctypes.c_int
            lib.oracle_paged_attention.argtypes = [
                u16p, u16p, u16p, i32p, i32p, f64p,
                ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                ctypes.c_int64, ctypes.c_int, ctypes.c_double, i32p, ctypes.c_int,
            ]
            lib.oracle_paged_attention_probs.restype = ctypes.c_int
            lib.oracle_paged_attention_probs.argtypes = [
                u16p, u16p, u16p, i32p, i32p, f64p, f64p,
                ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                ctypes.c_int, ctypes.c_int64, ctypes.c_int, ctypes.c_double,
            ]
            lib.oracle_f16_to_f64.restype = ctypes.c_double
            lib.oracle_f16_to_f64.argtypes = [ctypes.c_uint16]
            lib.oracle_bf16_to_f64.restype = ctypes.c_double
            lib.oracle_bf16_to_f64.argtypes = [ctypes.c_uint16]
            lib.oracle_num_threads.restype = ctypes.c_int
            u8p = ctypes.POINTER(ctypes.c_uint8)
            lib.oracle_fp8e4m3_to_f64.restype = ctypes.c_double
            lib.oracle_fp8e4m3_to_f64.argtypes = [ctypes.c_uint8]
            lib.oracle_paged_attention_kv8.restype = ctypes.c_int
            lib.oracle_paged_attention_kv8.argtypes = [
                u16p, u8p, u8p, i32p, i32p, f64p,
                ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                ctypes.c_int64, ctypes.c_int, ctypes.c_double, ctypes.c_double, ctypes.c_double, i32p, ctypes.c_int,
            ]
            _lib = lib
    return _lib


def oracle_threads() -> int:
    """Threads the OpenMP loop over (b, h) pairs will use."""
    return int(_load().oracle_num_threads())


def bits_of(t) -> np.ndarray:
    """Raw uint16 bit patterns of a 16-bit torch tensor (or pass a uint16 array through)."""
    if isinstance(t, np.ndarray):
        assert t.dtype == np.uint16
        return np.ascontiguousarray(t)
    import torch  # local: numpy callers do not need torch

    assert t.dtype in (torch.float16, torch.bfloat16)
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def widen_bits(bits: np.ndarray, dtype: str) -> np.ndarray:
    """fp64 values of raw 16-bit patterns, through the C oracle's own converters."""
    lib = _load()
    fn = lib.oracle_f16_to_f64 if dtype == "f16" else lib.oracle_bf16_to_f64
    flat = np.ascontiguousarray(bits, dtype=np.uint16).ravel()
    return np.array([fn(int(x)) for x in flat], dtype=np.float64).reshape(bits.shape)


def _ptr(a, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def _check_shapes(q, k_cache, v_cache, block_tables, context_lens):
    assert q.ndim == 3 and k_cache.ndim == 4 and v_cache.shape == k_cache.shape
    B, Hq, d = q.shape
    NBLK, Hkv, bs, d2 = k_cache.shape
    assert d2 == d and Hq % Hkv == 0
    assert block_tables.ndim == 2 and block_tables.shape[0] == B
    assert context_lens.shape == (B,)
    return B, Hq, d, NBLK, Hkv, bs, block_tables.shape[1]


def paged_attention(q, k_cache, v_cache, block_tables, context_lens, scale, dtype, pairs=None):
    """fp64 attention output.

    q [B,Hq,d], k_cache/v_cache [NBLK,Hkv,bs,d] as uint16 bits, block_tables [B,MB] int32,
    context_lens [B] int32.  Returns [B,Hq,d] float64, or [len(pairs),d] for a list of
    (b, h) pairs.
    """
    q = np.ascontiguousarray(q, dtype=np.uint16)
    k_cache = np.ascontiguousarray(k_cache, dtype=np.uint16)
    v_cache = np.ascontiguousarray(v_cache, dtype=np.uint16)
    block_tables = np.ascontiguousarray(block_tables, dtype=np.int32)
    context_lens = np.ascontiguousarray(context_lens, dtype=np.int32)
    B, Hq, d, NBLK, Hkv, bs, MB = _check_shapes(q, k_cache, v_cache, block_tables, context_lens)
    lib = _load()
    if pairs is None:
        out = np.empty((B, Hq, d), dtype=np.float64)
        pp, npairs = None, 0
    else:
        pairs = np.ascontiguousarray(pairs, dtype=np.int32).reshape(-1, 2)
        assert ((pairs[:, 0] >= 0) & (pairs[:, 0] < B) & (pairs[:, 1] >= 0) & (pairs[:, 1] < Hq)).all()
        out = np.empty((pairs.shape[0], d), dtype=np.float64)
        pp, npairs = _ptr(pairs, ctypes.c_int32), pairs.shape[0]
    rc = lib.oracle_paged_attention(
        _ptr(q, ctypes.c_uint16), _ptr(k_cache, ctypes.c_uint16), _ptr(v_cache, ctypes.c_uint16),
        _ptr(block_tables, ctypes.c_int32), _ptr(context_lens, ctypes.c_int32),
        _ptr(out, ctypes.c_double), B, Hq, Hkv, d, bs, MB, NBLK, _DTYPES[dtype], float(scale),
        pp, npairs,
    )
    if rc != 0:
        raise RuntimeError(f"oracle_paged_attention failed with status {rc}")
    return out


def paged_attention_probs(q, k_cache, v_cache, block_tables, context_lens, scale, dtype, b, h):
    """(out_row [d], probs [n_b]) of one (b, h): exposes the softmax row for the tests."""
    q = np.ascontiguousarray(q, dtype=np.uint16)
    k_cache = np.ascontiguousarray(k_cache, dtype=np.uint16)
    v_cache = np.ascontiguousarray(v_cache, dtype=np.uint16)
    block_tables = np.ascontiguousarray(block_tables, dtype=np.int32)
    context_lens = np.ascontiguousarray(context_lens, dtype=np.int32)
    B, Hq, d, NBLK, Hkv, bs, MB = _check_shapes(q, k_cache, v_cache, block_tables, context_lens)
    n = max(int(context_lens[b]), 0)
    out_row = np.empty(d, dtype=np.float64)
    probs = np.empty(max(n, 1), dtype=np.float64)
    rc = _load().oracle_paged_attention_probs(
        _ptr(q, ctypes.c_uint16), _ptr(k_cache, ctypes.c_uint16), _ptr(v_cache, ctypes.c_uint16),
        _ptr(block_tables, ctypes.c_int32), _ptr(context_lens, ctypes.c_int32),
        _ptr(out_row, ctypes.c_double), _ptr(probs, ctypes.c_double),
        int(b), int(h), Hq, Hkv, d, bs, MB, NBLK, _DTYPES[dtype], float(scale),
    )
    if rc != 0:
        raise RuntimeError(f"oracle_paged_attention_probs failed with status {rc}")
    return out_row, probs[:n]


def fp8e4m3_to_f64(codes) -> np.ndarray:
    """OCP FP8 E4M3 codes (uint8) -> float64, through the C decoder."""
    lib = _load()
    flat = np.ascontiguousarray(codes, dtype=np.uint8).ravel()
    return np.array([lib.oracle_fp8e4m3_to_f64(int(c)) for c in flat], dtype=np.float64).reshape(np.shape(codes))


def paged_attention_kv8(q, k_cache, v_cache, block_tables, context_lens, scale, qdtype, k_scale=1.0,
                        v_scale=1.0, pairs=None):
    """fp64 attention output over an FP8 E4M3 cache.

    q [B,Hq,d] as uint16 bits of ``qdtype``; k_cache/v_cache [NBLK,Hkv,bs,d] uint8 codes; the real K is
    ``k_scale * decode(code)``, V likewise.  Returns like :func:`paged_attention`.
    """
    q = np.ascontiguousarray(q, dtype=np.uint16)
    k_cache = np.ascontiguousarray(k_cache, dtype=np.uint8)
    v_cache = np.ascontiguousarray(v_cache, dtype=np.uint8)
    block_tables = np.ascontiguousarray(block_tables, dtype=np.int32)
    context_lens = np.ascontiguousarray(context_lens, dtype=np.int32)
    B, Hq, d, NBLK, Hkv, bs, MB = _check_shapes(q, k_cache, v_cache, block_tables, context_lens)
    lib = _load()
    if pairs is None:
        out = np.empty((B, Hq, d), dtype=np.float64)
        pp, npairs = None, 0
    else:
        pairs = np.ascontiguousarray(pairs, dtype=np.int32).reshape(-1, 2)
        assert ((pairs[:, 0] >= 0) & (pairs[:, 0] < B) & (pairs[:, 1] >= 0) & (pairs[:, 1] < Hq)).all()
        out = np.empty((pairs.shape[0], d), dtype=np.float64)
        pp, npairs = _ptr(pairs, ctypes.c_int32), pairs.shape[0]
    rc = lib.oracle_paged_attention_kv8(
        _ptr(q, ctypes.c_uint16), _ptr(k_cache, ctypes.c_uint8), _ptr(v_cache, ctypes.c_uint8),
        _ptr(block_tables, ctypes.c_int32), _ptr(context_lens, ctypes.c_int32),
        _ptr(out, ctypes.c_double), B, Hq, Hkv, d, bs, MB, NBLK, _DTYPES[qdtype], float(scale),
        float(k_scale), float(v_scale), pp, npairs,
    )
    if rc != 0:
        raise RuntimeError(f"oracle_paged_attention_kv8 failed with status {rc}")
    return out
