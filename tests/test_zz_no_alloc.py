"""The entry point for callers that cannot allocate (`mla_decode_static`: partial results in a
file-scope device array of the library) against `mla_decode_typed` with a caller's workspace, through
the C ABI.  The same kernels run with the same plan, so the results must agree bit for bit; they are
also held to the oracle.  Two calls in a row share the array, the second with a smaller input."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2506_01969_amd import inputs, mla

pytestmark = pytest.mark.gpu


def _typed(qd, kvd, ld, q_len, dtype_code):
    """mla_decode_typed through ctypes: automatic plan, both phases, a torch workspace."""
    batch = qd.shape[0]
    need, _ = mla.mla_decode_workspace_size(batch * q_len, 16, kvd.shape[1], 0)
    ws = torch.full((need,), 0xFF, dtype=torch.uint8, device=qd.device)
    out = torch.full((batch, q_len, 16, 512), float("nan"), dtype=torch.float32, device=qd.device)
    lse = torch.full((batch, q_len, 16), float("nan"), dtype=torch.float32, device=qd.device)
    vp = ctypes.c_void_p
    st = mla.lib().mla_decode_typed(vp(qd.data_ptr()), vp(kvd.data_ptr()), kvd.stride(0), vp(ld.data_ptr()), batch, q_len,
                                    16, kvd.shape[1], dtype_code, inputs.SCALE, vp(out.data_ptr()), vp(lse.data_ptr()),
                                    vp(ws.data_ptr()), need, 0, mla.PHASE_SPLIT | mla.PHASE_COMBINE,
                                    vp(torch.cuda.current_stream().cuda_stream))
    assert st == mla.MLA_OK
    torch.cuda.synchronize()
    return out, lse


def _static(qd, kvd, ld, q_len, dtype_code):
    batch = qd.shape[0]
    out = torch.full((batch, q_len, 16, 512), float("nan"), dtype=torch.float32, device=qd.device)
    lse = torch.full((batch, q_len, 16), float("nan"), dtype=torch.float32, device=qd.device)
    vp = ctypes.c_void_p
    st = mla.lib().mla_decode_static(vp(qd.data_ptr()), vp(kvd.data_ptr()), kvd.stride(0), vp(ld.data_ptr()), batch, q_len,
                                     16, kvd.shape[1], dtype_code, inputs.SCALE, vp(out.data_ptr()), vp(lse.data_ptr()),
                                     vp(torch.cuda.current_stream().cuda_stream))
    assert st == mla.MLA_OK, mla.lib().mla_status_string(st)
    torch.cuda.synchronize()
    return out, lse


def test_static_workspace_call_equals_the_call_with_a_workspace_twice_in_a_row(oracle):
    assert torch.cuda.is_available()
    dev = torch.device("cuda:0")
    # first call: 12 ragged sequences, two query tokens, many workgroups per sequence;
    # second call: smaller in every way (fewer sequences, shorter, one token), so it finds the
    # first call's partial results in every slot it does not write itself
    cases = [([9000, 1, 4097, 128, 0, 6000, 33, 2500, 7777, 640, 8191, 5], 9000, 2),
             ([700, 0, 129, 2048], 2048, 1)]
    for lens, max_len, q_len in cases:
        q, kv, l = inputs.make_inputs(len(lens), max_len, lens, seed=900 + q_len, poison_tail=True, q_len=q_len)
        qd, kvd, ld = q.to(dev), kv.to(dev), l.to(dev)
        print("case static batch %d q_len %d" % (len(lens), q_len), flush=True)
        got_o, got_l = _static(qd, kvd, ld, q_len, mla.DTYPE_BF16)
        want_o, want_l = _typed(qd, kvd, ld, q_len, mla.DTYPE_BF16)
        assert torch.equal(got_o, want_o) and torch.equal(got_l, want_l)
        ref_o, ref_l = oracle.decode_general(inputs.bits16(q), inputs.bits16(kv), l.numpy(), inputs.SCALE, inputs.D_V,
                                             dtype=oracle.BF16)
        o = got_o.cpu().numpy().astype(np.float64).reshape(ref_o.shape)
        s = got_l.cpu().numpy().astype(np.float64).reshape(ref_l.shape)
        fin = np.isfinite(ref_l)
        assert np.abs(o - ref_o).max() <= 5e-5 and np.isneginf(s[~fin]).all() and np.abs(s[fin] - ref_l[fin]).max() <= 2e-5


def test_static_workspace_call_rejects_what_does_not_fit():
    dev = torch.device("cuda:0")
    q, kv, l = inputs.make_inputs(65, 64, None, seed=3)
    qd, kvd, ld = q.to(dev), kv.to(dev), l.to(dev)
    out = torch.full((65, 1, 16, 512), 7.0, dtype=torch.float32, device=dev)
    lse = torch.full((65, 1, 16), 7.0, dtype=torch.float32, device=dev)
    with pytest.raises(mla.MlaError) as e:
        mla.mla_decode_static(qd, kvd, ld, inputs.SCALE, out, lse)
    assert e.value.status == mla.MLA_ERR_STATIC_LIMIT
    torch.cuda.synchronize()
    assert (out == 7.0).all() and (lse == 7.0).all()
