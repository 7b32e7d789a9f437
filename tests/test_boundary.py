"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, the split plan is sane, and every host-detectable error is reported before any
device work (fake but well-aligned pointers are never dereferenced on these paths)."""
import ctypes
import os
import re

import pytest

from paper_2506_01969_amd import mla

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "mla_decode.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mla_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_functions()
    assert {"mla_decode", "mla_decode_ex", "mla_decode_typed", "mla_decode_static", "mla_decode_workspace_size",
            "mla_decode_workspace_size_for", "mla_decode_planned_workgroups", "mla_decode_plan_table",
            "mla_status_string"} <= set(names)
    lib = mla.lib()
    for n in names:
        assert hasattr(lib, n), n


def test_status_strings():
    lib = mla.lib()
    seen = {lib.mla_status_string(i) for i in range(6)}
    assert len(seen) == 6 and all(seen)
    assert lib.mla_status_string(99)


@pytest.mark.parametrize("batch,num_wg", [(1, 256), (16, 256), (32, 304), (3, 1), (1024, 64)])
def test_workspace_size_is_two_slots_per_workgroup_one_per_sequence_plus_eight(batch, num_wg):
    nbytes, used = mla.mla_decode_workspace_size(batch, 16, 65536, num_workgroups=num_wg)
    assert used == num_wg
    slot = 16 * 512 * 4 + 16 * 4
    # a workgroup writes one partial result per query token it works for: at most two
    assert (2 * num_wg + batch + 8) * slot <= nbytes <= (2 * num_wg + batch + 8) * slot + 16
    # independent of the KV length: the lengths live on the device
    assert mla.mla_decode_workspace_size(batch, 16, 7, num_workgroups=num_wg) == (nbytes, used)


def test_workspace_size_of_the_automatic_plan_without_a_device():
    # the automatic plan for a device of 256 compute units: 208 workgroups for a long stream, 256 for a short
    # one; the size covers 256 workgroups with two query tokens each, whatever the plan launches
    slot = 16 * 512 * 4 + 16 * 4
    for batch, seqlen, want_wg in ((16, 65536, 208), (16, 4096, 256), (1, 512, 256), (128, 65536, 208)):
        nbytes, used = mla.mla_decode_workspace_size_for(batch, 16, seqlen, 256)
        assert used == want_wg
        assert nbytes == mla.mla_decode_workspace_size(batch, 16, seqlen, num_workgroups=256)[0]
        assert (2 * 256 + batch + 8) * slot <= nbytes <= (2 * 256 + batch + 8) * slot + 16
    assert mla.mla_decode_workspace_size_for(3, 16, 100, 1) == (mla.mla_decode_workspace_size(3, 16, 100, num_workgroups=1)[0], 1)
    lib = mla.lib()
    n = ctypes.c_size_t(0)
    assert lib.mla_decode_workspace_size_for(16, 16, 4096, 0, ctypes.byref(n), None) == mla.MLA_ERR_INVALID_ARG
    assert lib.mla_decode_workspace_size_for(16, 8, 4096, 256, ctypes.byref(n), None) == mla.MLA_ERR_UNSUPPORTED_SHAPE
    assert lib.mla_decode_workspace_size_for(16, 16, 4096, 256, None, None) == mla.MLA_ERR_INVALID_ARG


def test_workspace_size_errors():
    lib = mla.lib()
    n = ctypes.c_size_t(0)
    assert lib.mla_decode_workspace_size(16, 8, 4096, 256, ctypes.byref(n), None) == mla.MLA_ERR_UNSUPPORTED_SHAPE
    assert lib.mla_decode_workspace_size(0, 16, 4096, 256, ctypes.byref(n), None) == mla.MLA_ERR_INVALID_ARG
    assert lib.mla_decode_workspace_size(16, 16, 0, 256, ctypes.byref(n), None) == mla.MLA_ERR_INVALID_ARG
    assert lib.mla_decode_workspace_size(16, 16, 4096, -1, ctypes.byref(n), None) == mla.MLA_ERR_INVALID_ARG
    assert lib.mla_decode_workspace_size(16, 16, 4096, 1 << 20, ctypes.byref(n), None) == mla.MLA_ERR_INVALID_ARG
    assert lib.mla_decode_workspace_size(16, 16, 4096, 256, None, None) == mla.MLA_ERR_INVALID_ARG


def _call(q=0x1000, kv=0x2000, stride=4096 * 576, lens=0x3000, batch=2, heads=16, seqlen=4096, scale=0.1,
          out=0x4000, lse=0x5000, ws=0x6000, ws_bytes=1 << 30, num_wg=256, phases=3):
    vp = ctypes.c_void_p
    return mla.lib().mla_decode_ex(vp(q), vp(kv), stride, vp(lens), batch, heads, seqlen, scale, vp(out), vp(lse),
                                   vp(ws), ws_bytes, num_wg, phases, None)


def test_planned_workgroups_argument_errors():
    lib = mla.lib()
    n = ctypes.c_int(0)
    assert lib.mla_decode_planned_workgroups(16, 1, 4096, None) == mla.MLA_ERR_INVALID_ARG
    assert lib.mla_decode_planned_workgroups(0, 1, 4096, ctypes.byref(n)) == mla.MLA_ERR_INVALID_ARG
    assert lib.mla_decode_planned_workgroups(16, 1, 0, ctypes.byref(n)) == mla.MLA_ERR_INVALID_ARG
    assert lib.mla_decode_planned_workgroups(16, 0, 4096, ctypes.byref(n)) == mla.MLA_ERR_UNSUPPORTED_SHAPE
    assert lib.mla_decode_planned_workgroups(16, 9, 4096, ctypes.byref(n)) == mla.MLA_ERR_UNSUPPORTED_SHAPE


def test_decode_argument_errors_come_before_any_device_work():
    E = mla
    assert _call(q=0) == E.MLA_ERR_INVALID_ARG
    assert _call(kv=0) == E.MLA_ERR_INVALID_ARG
    assert _call(lens=0) == E.MLA_ERR_INVALID_ARG
    assert _call(out=0) == E.MLA_ERR_INVALID_ARG
    assert _call(lse=0) == E.MLA_ERR_INVALID_ARG
    assert _call(ws=0) == E.MLA_ERR_INVALID_ARG
    assert _call(q=0x1008) == E.MLA_ERR_INVALID_ARG          # misaligned
    assert _call(kv=0x2004) == E.MLA_ERR_INVALID_ARG
    assert _call(out=0x4002) == E.MLA_ERR_INVALID_ARG
    assert _call(lse=0x5001) == E.MLA_ERR_INVALID_ARG
    assert _call(heads=8) == E.MLA_ERR_UNSUPPORTED_SHAPE
    assert _call(heads=128) == E.MLA_ERR_UNSUPPORTED_SHAPE
    assert _call(batch=0) == E.MLA_ERR_INVALID_ARG
    assert _call(seqlen=-5) == E.MLA_ERR_INVALID_ARG
    assert _call(stride=4095 * 576) == E.MLA_ERR_INVALID_ARG   # rows of one sequence would overlap the next
    assert _call(stride=4096 * 576 + 4) == E.MLA_ERR_INVALID_ARG  # breaks 16-byte alignment of rows
    assert _call(scale=float("nan")) == E.MLA_ERR_INVALID_ARG
    assert _call(scale=float("inf")) == E.MLA_ERR_INVALID_ARG
    assert _call(scale=2.0e6) == E.MLA_ERR_INVALID_ARG and _call(scale=-2.0e6) == E.MLA_ERR_INVALID_ARG    # beyond MLA_MAX_ABS_SCALE
    assert _call(num_wg=-1) == E.MLA_ERR_INVALID_ARG
    assert _call(num_wg=1 << 20) == E.MLA_ERR_INVALID_ARG
    assert _call(phases=0) == E.MLA_ERR_INVALID_ARG
    assert _call(phases=4) == E.MLA_ERR_INVALID_ARG     # no phase selected
    assert _call(phases=8) == E.MLA_ERR_INVALID_ARG
    need, _ = mla.mla_decode_workspace_size(2, 16, 4096, 256)
    assert _call(ws_bytes=need - 1) == E.MLA_ERR_WORKSPACE_TOO_SMALL


def test_typed_entry_argument_errors():
    vp = ctypes.c_void_p

    def call(dtype=0, q_len=1, batch=2):
        return mla.lib().mla_decode_typed(vp(0x1000), vp(0x2000), 4096 * 576, vp(0x3000), batch, q_len, 16, 4096, dtype,
                                          0.1, vp(0x4000), vp(0x5000), vp(0x6000), 1 << 30, 256, 3, None)
    assert call(dtype=2) == mla.MLA_ERR_INVALID_ARG
    assert call(dtype=-1) == mla.MLA_ERR_INVALID_ARG
    assert call(q_len=0) == mla.MLA_ERR_UNSUPPORTED_SHAPE
    assert call(q_len=9) == mla.MLA_ERR_UNSUPPORTED_SHAPE
    assert call(batch=0) == mla.MLA_ERR_INVALID_ARG


def test_binding_rejects_host_tensors():
    import torch
    q = torch.zeros((1, 1, 16, 576), dtype=torch.bfloat16)
    kv = torch.zeros((1, 8, 576), dtype=torch.bfloat16)
    lens = torch.zeros((1,), dtype=torch.int32)
    with pytest.raises(ValueError):
        mla.mla_decode(q, kv, lens, 0.1)
    with pytest.raises(TypeError):
        mla.mla_decode(q.float(), kv, lens, 0.1)


def test_algorithmic_bytes_and_flops_of_the_headline_shape():
    """The figures the roofline fraction is computed from: 1152 B per KV row read once for all 16 heads,
    plus q (18,432 B), out (32,768 B), lse (64 B) and the length (4 B) per sequence; 2 (576 + 512) flop per
    head and KV row."""
    from paper_2506_01969_amd import inputs
    lens = [65536] * 16
    assert inputs.algorithmic_bytes(lens) == 1152 * 16 * 65536 + 51268 * 16 == 1208779840
    assert inputs.algorithmic_flops(lens) == 2 * (576 + 512) * 16 * 16 * 65536 == 36507222016
    assert inputs.algorithmic_bytes([1, 0, 7]) == 1152 * 8 + 51268 * 3
