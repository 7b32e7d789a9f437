"""ctypes loader for the fp64 CPU oracle (``mla_oracle.c``).  TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the ``cpu_baseline`` leg of the benchmark may
import this module; the product path never does.  It shares nothing with the HIP
path: inputs arrive as numpy ``uint16`` arrays holding bf16 bit patterns and
results leave as numpy ``float64`` arrays.

The arithmetic lives in ``mla_oracle.c`` (Section 3.1 definition of
S = Q K^T, P = softmax(S), O = P V; equations (1)-(4) for the transposed form;
L = m + log(l) from the last step of Algorithm 1).  This file only marshals
arguments.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mla_oracle.c")
_LIB = os.path.join(_HERE, "libmla_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile ``mla_oracle.c`` with gcc into ``libmla_oracle.so`` (beside the source)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
             _SRC, "-o", tmp, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        u16p = ctypes.POINTER(ctypes.c_uint16)
        i32p = ctypes.POINTER(ctypes.c_int32)
        f64p = ctypes.POINTER(ctypes.c_double)
        ci, cd, i64 = ctypes.c_int, ctypes.c_double, ctypes.c_int64
        lib.mla_oracle_decode.argtypes = [u16p, u16p, i64, i32p, ci, ci, ci, ci, cd, f64p, f64p, ci]
        lib.mla_oracle_decode.restype = ci
        lib.mla_oracle_decode_general.argtypes = [u16p, u16p, i64, i32p, ci, ci, ci, ci, ci, ci, cd, f64p, f64p, ci]
        lib.mla_oracle_decode_general.restype = ci
        lib.mla_oracle_decode_range.argtypes = [u16p, u16p, i64, i32p, ci, ci, ci, ci, ci, ci, cd, f64p, f64p]
        lib.mla_oracle_decode_range.restype = ci
        lib.mla_oracle_decode_transposed.argtypes = [u16p, u16p, i64, i32p, ci, ci, ci, ci, cd, f64p, f64p]
        lib.mla_oracle_decode_transposed.restype = ci
        lib.mla_oracle_merge.argtypes = [f64p, f64p, ci, ci, f64p, f64p]
        lib.mla_oracle_merge.restype = ci
        lib.mla_oracle_probs.argtypes = [u16p, u16p, i64, i32p, ci, ci, ci, ci, cd, f64p]
        lib.mla_oracle_probs.restype = ci
        lib.mla_oracle_threads.argtypes = []
        lib.mla_oracle_threads.restype = ci
        _lib = lib
    return _lib


def _u16(a):
    a = np.ascontiguousarray(a)
    if a.dtype != np.uint16:
        raise TypeError("bf16 bit patterns must be uint16, got %s" % a.dtype)
    return a


def _ptr(a, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def _shapes(q_bits, kv_bits, seqlens):
    q_bits, kv_bits = _u16(q_bits), _u16(kv_bits)
    if q_bits.ndim == 4:  # [batch, 1, heads, d_qk]
        if q_bits.shape[1] != 1:
            raise ValueError("q_len must be 1")
        q_bits = q_bits.reshape(q_bits.shape[0], q_bits.shape[2], q_bits.shape[3])
    batch, heads, d_qk = q_bits.shape
    if kv_bits.ndim != 3 or kv_bits.shape[0] != batch or kv_bits.shape[2] != d_qk:
        raise ValueError("kv must be [batch, max_seqlen, d_qk]")
    seqlens = np.ascontiguousarray(seqlens, dtype=np.int32)
    if seqlens.shape != (batch,) or (seqlens < 0).any() or (seqlens > kv_bits.shape[1]).any():
        raise ValueError("seqlens must be [batch] with 0 <= len <= max_seqlen")
    return q_bits, kv_bits, seqlens, batch, heads, d_qk


def threads() -> int:
    """Threads the batched oracle runs with (OpenMP's current maximum)."""
    return int(_load().mla_oracle_threads())


def decode(q_bits, kv_bits, seqlens, scale, d_v, nthreads=0):
    """Direct formulation.  Returns (out [batch, heads, d_v] f64, lse [batch, heads] f64)."""
    lib = _load()
    q_bits, kv_bits, seqlens, batch, heads, d_qk = _shapes(q_bits, kv_bits, seqlens)
    out = np.empty((batch, heads, d_v), dtype=np.float64)
    lse = np.empty((batch, heads), dtype=np.float64)
    rc = lib.mla_oracle_decode(_ptr(q_bits, ctypes.c_uint16), _ptr(kv_bits, ctypes.c_uint16),
                               kv_bits.shape[1] * d_qk, _ptr(seqlens, ctypes.c_int32),
                               batch, heads, d_qk, d_v, float(scale),
                               _ptr(out, ctypes.c_double), _ptr(lse, ctypes.c_double), int(nthreads))
    if rc != 0:
        raise RuntimeError("mla_oracle_decode failed")
    return out, lse


BF16, F16 = 0, 1


def decode_general(q_bits, kv_bits, seqlens, scale, d_v, dtype=BF16, nthreads=0):
    """q_len query tokens per sequence (causal among themselves) and bf16 or fp16 bit patterns.

    q_bits [batch, q_len, heads, d_qk] uint16, kv_bits [batch, max_seqlen, d_qk] uint16;
    seqlens count the KV rows including the q_len new tokens.
    Returns (out [batch, q_len, heads, d_v] f64, lse [batch, q_len, heads] f64).
    """
    lib = _load()
    q_bits, kv_bits = _u16(q_bits), _u16(kv_bits)
    if q_bits.ndim != 4:
        raise ValueError("q must be [batch, q_len, heads, d_qk]")
    batch, q_len, heads, d_qk = q_bits.shape
    if kv_bits.ndim != 3 or kv_bits.shape[0] != batch or kv_bits.shape[2] != d_qk:
        raise ValueError("kv must be [batch, max_seqlen, d_qk]")
    seqlens = np.ascontiguousarray(seqlens, dtype=np.int32)
    if seqlens.shape != (batch,) or (seqlens < 0).any() or (seqlens > kv_bits.shape[1]).any():
        raise ValueError("seqlens must be [batch] with 0 <= len <= max_seqlen")
    out = np.empty((batch, q_len, heads, d_v), dtype=np.float64)
    lse = np.empty((batch, q_len, heads), dtype=np.float64)
    rc = lib.mla_oracle_decode_general(_ptr(q_bits, ctypes.c_uint16), _ptr(kv_bits, ctypes.c_uint16),
                                       kv_bits.shape[1] * d_qk, _ptr(seqlens, ctypes.c_int32),
                                       batch, q_len, heads, d_qk, d_v, int(dtype), float(scale),
                                       _ptr(out, ctypes.c_double), _ptr(lse, ctypes.c_double), int(nthreads))
    if rc != 0:
        raise RuntimeError("mla_oracle_decode_general failed")
    return out, lse


def decode_transposed(q_bits, kv_bits, seqlens, scale, d_v):
    """Transposed formulation, equations (1)-(4).  Same return as :func:`decode`."""
    lib = _load()
    q_bits, kv_bits, seqlens, batch, heads, d_qk = _shapes(q_bits, kv_bits, seqlens)
    out = np.empty((batch, heads, d_v), dtype=np.float64)
    lse = np.empty((batch, heads), dtype=np.float64)
    rc = lib.mla_oracle_decode_transposed(_ptr(q_bits, ctypes.c_uint16), _ptr(kv_bits, ctypes.c_uint16),
                                          kv_bits.shape[1] * d_qk, _ptr(seqlens, ctypes.c_int32),
                                          batch, heads, d_qk, d_v, float(scale),
                                          _ptr(out, ctypes.c_double), _ptr(lse, ctypes.c_double))
    if rc != 0:
        raise RuntimeError("mla_oracle_decode_transposed failed")
    return out, lse


def decode_range(q_bits, kv_bits, seqlens, scale, d_v, t0, t1):
    """Attention over tokens [t0, t1) only (clipped to each sequence's length)."""
    lib = _load()
    q_bits, kv_bits, seqlens, batch, heads, d_qk = _shapes(q_bits, kv_bits, seqlens)
    out = np.empty((batch, heads, d_v), dtype=np.float64)
    lse = np.empty((batch, heads), dtype=np.float64)
    rc = lib.mla_oracle_decode_range(_ptr(q_bits, ctypes.c_uint16), _ptr(kv_bits, ctypes.c_uint16),
                                     kv_bits.shape[1] * d_qk, _ptr(seqlens, ctypes.c_int32),
                                     batch, heads, d_qk, d_v, int(t0), int(t1), float(scale),
                                     _ptr(out, ctypes.c_double), _ptr(lse, ctypes.c_double))
    if rc != 0:
        raise RuntimeError("mla_oracle_decode_range failed")
    return out, lse


def merge(part_out, part_lse):
    """LSE merge of the parts of one (b, h) pair.  part_out [n, d_v], part_lse [n]."""
    lib = _load()
    part_out = np.ascontiguousarray(part_out, dtype=np.float64)
    part_lse = np.ascontiguousarray(part_lse, dtype=np.float64)
    n, d_v = part_out.shape
    out = np.empty((d_v,), dtype=np.float64)
    lse = np.empty((1,), dtype=np.float64)
    rc = lib.mla_oracle_merge(_ptr(part_out, ctypes.c_double), _ptr(part_lse, ctypes.c_double), n, d_v,
                              _ptr(out, ctypes.c_double), _ptr(lse, ctypes.c_double))
    if rc != 0:
        raise RuntimeError("mla_oracle_merge failed")
    return out, float(lse[0])


def probs(q_bits, kv_bits, seqlens, scale, b, h):
    """Softmax probabilities p[t], t < N_b, of one (b, h) pair."""
    lib = _load()
    q_bits, kv_bits, seqlens, batch, heads, d_qk = _shapes(q_bits, kv_bits, seqlens)
    p = np.empty((max(int(seqlens[b]), 1),), dtype=np.float64)
    rc = lib.mla_oracle_probs(_ptr(q_bits, ctypes.c_uint16), _ptr(kv_bits, ctypes.c_uint16),
                              kv_bits.shape[1] * d_qk, _ptr(seqlens, ctypes.c_int32),
                              heads, d_qk, int(b), int(h), float(scale), _ptr(p, ctypes.c_double))
    if rc != 0:
        raise RuntimeError("mla_oracle_probs failed")
    return p[: int(seqlens[b])]
