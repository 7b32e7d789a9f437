"""Thin Python binding of the C ABI in ``include/mla_decode.h`` (argument marshalling only).

Every step of the computation runs inside ``libmla_decode.so``; torch is used for device
memory and the current stream, nothing else.  There is no fallback: if the library is
not built it is built (hipcc), and if that or the load fails, callers get an error.
"""
from __future__ import annotations

import ctypes
import os

import torch

NUM_HEADS = 16
D_QK = 576
D_V = 512

MLA_OK = 0
MLA_ERR_INVALID_ARG = 1
MLA_ERR_UNSUPPORTED_SHAPE = 2
MLA_ERR_WORKSPACE_TOO_SMALL = 3
MLA_ERR_HIP = 4
MLA_ERR_STATIC_LIMIT = 5

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libmla_decode.so")
_lib = None


class MlaError(RuntimeError):
    def __init__(self, status, where):
        self.status = int(status)
        msg = lib().mla_status_string(self.status).decode()
        super().__init__("%s: %s (status %d)" % (where, msg, self.status))


def lib():
    """Load ``libmla_decode.so``.  What is built is loaded as it is; only when nothing is built is
    the build step (``paper_2506_01969_amd.build``, hipcc) run first.  Any failure raises: there is
    no other implementation to fall back to."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            from . import build as _build
            _build.build_library()
        L = ctypes.CDLL(LIB_PATH)
        vp, ci, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
        szp, cip = ctypes.POINTER(ctypes.c_size_t), ctypes.POINTER(ctypes.c_int)
        L.mla_decode_workspace_size.argtypes = [ci, ci, ci, ci, szp, cip]
        L.mla_decode_workspace_size.restype = ci
        L.mla_decode_workspace_size_for.argtypes = [ci, ci, ci, ci, szp, cip]
        L.mla_decode_workspace_size_for.restype = ci
        L.mla_decode.argtypes = [vp, vp, ctypes.c_int64, vp, ci, ci, ci, ctypes.c_float, vp, vp, vp, sz, vp]
        L.mla_decode.restype = ci
        L.mla_decode_ex.argtypes = [vp, vp, ctypes.c_int64, vp, ci, ci, ci, ctypes.c_float, vp, vp,
                                    vp, sz, ci, ci, vp]
        L.mla_decode_ex.restype = ci
        L.mla_decode_typed.argtypes = [vp, vp, ctypes.c_int64, vp, ci, ci, ci, ci, ci, ctypes.c_float, vp, vp,
                                       vp, sz, ci, ci, vp]
        L.mla_decode_typed.restype = ci
        L.mla_decode_static.argtypes = [vp, vp, ctypes.c_int64, vp, ci, ci, ci, ci, ci, ctypes.c_float, vp, vp, vp]
        L.mla_decode_static.restype = ci
        L.mla_decode_plan_table.argtypes = [vp, ci, ci, ci, ci, ci, vp, cip, cip, vp]
        L.mla_decode_plan_table.restype = ci
        L.mla_decode_planned_workgroups.argtypes = [ci, ci, ci, cip]
        L.mla_decode_planned_workgroups.restype = ci
        L.mla_status_string.argtypes = [ci]
        L.mla_status_string.restype = ctypes.c_char_p
        _lib = L
    return _lib


def mla_decode_workspace_size(batch, num_heads, max_seqlen_kv, num_workgroups=0):
    """-> (bytes, num_workgroups_used).  num_workgroups=0 is the automatic plan (asks the device)."""
    nbytes, used = ctypes.c_size_t(0), ctypes.c_int(0)
    st = lib().mla_decode_workspace_size(batch, num_heads, max_seqlen_kv, num_workgroups,
                                         ctypes.byref(nbytes), ctypes.byref(used))
    if st != MLA_OK:
        raise MlaError(st, "mla_decode_workspace_size")
    return nbytes.value, used.value


def mla_decode_workspace_size_for(batch, num_heads, max_seqlen_kv, num_compute_units):
    """-> (bytes, num_workgroups_used) of the automatic plan on a device of that many compute units (host only)."""
    nbytes, used = ctypes.c_size_t(0), ctypes.c_int(0)
    st = lib().mla_decode_workspace_size_for(batch, num_heads, max_seqlen_kv, num_compute_units,
                                             ctypes.byref(nbytes), ctypes.byref(used))
    if st != MLA_OK:
        raise MlaError(st, "mla_decode_workspace_size_for")
    return nbytes.value, used.value


def mla_decode_planned_workgroups(batch, q_len, max_seqlen_kv):
    """Workgroups the automatic plan launches on the current device for this shape."""
    n = ctypes.c_int(0)
    st = lib().mla_decode_planned_workgroups(batch, q_len, max_seqlen_kv, ctypes.byref(n))
    if st != MLA_OK:
        raise MlaError(st, "mla_decode_planned_workgroups")
    return n.value


def _check_tensors(q, kv_cache, cache_seqlens):
    if q.dtype not in (torch.bfloat16, torch.float16) or kv_cache.dtype != q.dtype:
        raise TypeError("q and kv_cache must both be bf16 or both be fp16")
    if cache_seqlens.dtype != torch.int32:
        raise TypeError("cache_seqlens must be int32")
    if not (q.is_cuda and kv_cache.is_cuda and cache_seqlens.is_cuda):
        raise ValueError("q, kv_cache and cache_seqlens must be device tensors")
    if q.dim() != 4 or q.shape[1] < 1 or q.shape[3] != D_QK or not q.is_contiguous():
        raise ValueError("q must be contiguous [batch, q_len, heads, 576]")
    if kv_cache.dim() != 3 or kv_cache.shape[0] != q.shape[0] or kv_cache.shape[2] != D_QK:
        raise ValueError("kv_cache must be [batch, max_seqlen_kv, 576]")
    if kv_cache.stride(2) != 1 or kv_cache.stride(1) != D_QK:
        raise ValueError("kv_cache rows must be contiguous (row stride 576)")
    if cache_seqlens.shape != (q.shape[0],) or not cache_seqlens.is_contiguous():
        raise ValueError("cache_seqlens must be contiguous [batch]")


PHASE_SPLIT = 1
PHASE_COMBINE = 2
ORIENT_DIRECT = 8
UNIT_FINE = 16
UNIT_COARSE = 32
DTYPE_BF16 = 0
DTYPE_F16 = 1


def mla_decode(q, kv_cache, cache_seqlens, scale, out=None, lse=None, workspace=None, num_workgroups=None,
               phases=None):
    """out [batch, q_len, heads, 512] fp32, lse [batch, heads] fp32 ([batch, q_len, heads] when
    q_len > 1) on the current stream (asynchronous).

    q [batch, q_len, 16, 576] and kv_cache [batch, max_seqlen_kv, 576] (batch stride free), both
    bf16 or both fp16; cache_seqlens [batch] int32 (counting the q_len new tokens, which attend
    causally among themselves); all on the current device.  ``out``, ``lse`` and ``workspace`` (a
    uint8 tensor) are allocated with torch when not given.  ``num_workgroups`` forces the split
    plan; ``phases`` is the ``flags`` argument of ``mla_decode_ex`` (PHASE_SPLIT, PHASE_COMBINE,
    ORIENT_DIRECT).  fp16 or q_len > 1 go through ``mla_decode_typed``.
    """
    _check_tensors(q, kv_cache, cache_seqlens)
    batch, q_len, heads, _ = q.shape
    max_seqlen = kv_cache.shape[1]
    dev = q.device
    need, _ = mla_decode_workspace_size(batch * q_len, heads, max_seqlen, int(num_workgroups or 0))
    if out is None:
        out = torch.empty((batch, q_len, heads, D_V), dtype=torch.float32, device=dev)
    if lse is None:
        lse = torch.empty((batch, heads) if q_len == 1 else (batch, q_len, heads), dtype=torch.float32, device=dev)
    if workspace is None:
        workspace = torch.empty((need,), dtype=torch.uint8, device=dev)
    stream = ctypes.c_void_p(torch.cuda.current_stream(dev).cuda_stream)
    head = [ctypes.c_void_p(q.data_ptr()), ctypes.c_void_p(kv_cache.data_ptr()), kv_cache.stride(0),
            ctypes.c_void_p(cache_seqlens.data_ptr()), batch]
    shape = [heads, max_seqlen]
    tail = [float(scale), ctypes.c_void_p(out.data_ptr()), ctypes.c_void_p(lse.data_ptr()),
            ctypes.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size()]
    args = head + shape + tail
    if q.dtype == torch.float16 or q_len != 1:
        st = lib().mla_decode_typed(*head, q_len, *shape, DTYPE_F16 if q.dtype == torch.float16 else DTYPE_BF16,
                                    *tail, int(num_workgroups or 0),
                                    int(PHASE_SPLIT | PHASE_COMBINE if phases is None else phases), stream)
        where = "mla_decode_typed"
    elif num_workgroups is None and phases is None:
        st = lib().mla_decode(*args, stream)
        where = "mla_decode"
    else:
        st = lib().mla_decode_ex(*args, int(num_workgroups or 0),
                                 int(PHASE_SPLIT | PHASE_COMBINE if phases is None else phases), stream)
        where = "mla_decode_ex"
    if st != MLA_OK:
        raise MlaError(st, where)
    return out, lse


def mla_decode_static(q, kv_cache, cache_seqlens, scale, out, lse):
    """``mla_decode_static`` of the C ABI: the automatic plan with the library's own static workspace,
    for callers that cannot allocate.  ``out`` and ``lse`` are the caller's; nothing is allocated here."""
    _check_tensors(q, kv_cache, cache_seqlens)
    batch, q_len, heads, _ = q.shape
    if out.dtype != torch.float32 or lse.dtype != torch.float32 or not (out.is_contiguous() and lse.is_contiguous()):
        raise TypeError("out and lse must be contiguous fp32 tensors")
    if out.numel() != batch * q_len * heads * D_V or lse.numel() != batch * q_len * heads:
        raise ValueError("out must hold [batch, q_len, heads, 512] and lse [batch, q_len, heads]")
    stream = ctypes.c_void_p(torch.cuda.current_stream(q.device).cuda_stream)
    st = lib().mla_decode_static(ctypes.c_void_p(q.data_ptr()), ctypes.c_void_p(kv_cache.data_ptr()), kv_cache.stride(0),
                                 ctypes.c_void_p(cache_seqlens.data_ptr()), batch, q_len, heads, kv_cache.shape[1],
                                 DTYPE_F16 if q.dtype == torch.float16 else DTYPE_BF16, float(scale),
                                 ctypes.c_void_p(out.data_ptr()), ctypes.c_void_p(lse.data_ptr()), stream)
    if st != MLA_OK:
        raise MlaError(st, "mla_decode_static")
    return out, lse


def mla_decode_plan_table(cache_seqlens, q_len, max_seqlen_kv, num_workgroups=0, flags=0):
    """``mla_decode_plan_table`` of the C ABI -> (table [teams + batch, 8] int32 on the device, teams,
    unit_tokens): the partition as the kernels derive it on the device (tests, diagnosis)."""
    if cache_seqlens.dtype != torch.int32 or not cache_seqlens.is_cuda or not cache_seqlens.is_contiguous():
        raise TypeError("cache_seqlens must be a contiguous int32 device tensor")
    batch = cache_seqlens.numel()
    rows = int(num_workgroups) or mla_decode_planned_workgroups(batch, q_len, max_seqlen_kv)
    table = torch.full((rows + batch, 8), -7, dtype=torch.int32, device=cache_seqlens.device)
    teams, unit = ctypes.c_int(0), ctypes.c_int(0)
    stream = ctypes.c_void_p(torch.cuda.current_stream(cache_seqlens.device).cuda_stream)
    st = lib().mla_decode_plan_table(ctypes.c_void_p(cache_seqlens.data_ptr()), batch, q_len, max_seqlen_kv,
                                     int(num_workgroups), int(flags), ctypes.c_void_p(table.data_ptr()),
                                     ctypes.byref(teams), ctypes.byref(unit), stream)
    if st != MLA_OK:
        raise MlaError(st, "mla_decode_plan_table")
    return table[:teams.value + batch], teams.value, unit.value
