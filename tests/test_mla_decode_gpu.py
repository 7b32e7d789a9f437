"""Parity of the HIP path (through the C ABI) against the fp64 CPU oracle, on a real MI355X.

Tolerances (fp32 output, bf16 inputs, fp32 accumulation), over all `out` elements of a case:
    max |out - ref| <= 2e-3,  RMSE <= 1e-4,  max |lse - ref| <= 1e-4      (the stated bar)
The kernel feeds P to the second product as a two-term bf16 split, so its own error budget is
fp32 accumulation over <= 64K terms of magnitude <= |v|*p: about 1e-5 absolute.  The tests also
hold it to that tighter derived bound (TIGHT_*), which a dropped low term or a wrong tile would
break while still passing the stated bar at long KV.
"""
import math

import numpy as np
import pytest
import torch

from paper_2506_01969_amd import inputs, mla

pytestmark = pytest.mark.gpu

MAX_ABS, RMSE, LSE_ABS = 2e-3, 1e-4, 1e-4
TIGHT_MAX_ABS, TIGHT_RMSE, TIGHT_LSE = 5e-5, 5e-6, 2e-5


def _dev():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return torch.device("cuda:0")


def _run(q, kv, lens, scale=inputs.SCALE, num_wg=None, kv_dev=None):
    dev = _dev()
    qd = q.to(dev)
    kvd = kv.to(dev) if kv_dev is None else kv_dev
    ld = lens.to(dev)
    out, lse = mla.mla_decode(qd, kvd, ld, scale, num_workgroups=num_wg)
    torch.cuda.synchronize()
    return out.cpu().numpy().reshape(q.shape[0], q.shape[2], inputs.D_V).astype(np.float64), lse.cpu().numpy().astype(np.float64)


def _check(out, lse, ref_o, ref_l, tight=True, label=""):
    assert np.isfinite(out).all(), label
    err = np.abs(out - ref_o)
    rmse = math.sqrt(float((err ** 2).mean()))
    fin = np.isfinite(ref_l)
    assert (np.isneginf(lse[~fin])).all(), label
    lerr = float(np.abs(lse[fin] - ref_l[fin]).max()) if fin.any() else 0.0
    print("%s max_abs %.3e rmse %.3e lse_err %.3e" % (label, err.max(), rmse, lerr), flush=True)
    assert err.max() <= MAX_ABS and rmse <= RMSE and lerr <= LSE_ABS, label
    if tight:
        assert err.max() <= TIGHT_MAX_ABS and rmse <= TIGHT_RMSE and lerr <= TIGHT_LSE, label


def _oracle(oracle, q, kv, lens, scale=inputs.SCALE):
    return oracle.decode(inputs.bf16_bits(q), inputs.bf16_bits(kv), lens.numpy(), scale, inputs.D_V)


# ---- small cases: several tiles, ragged tails, every split count ---------------------------------

@pytest.mark.parametrize("num_wg", [None, 1, 2, 7, 40, 1000])
def test_small_ragged_elementwise(oracle, num_wg):
    lens = [1, 31, 32, 33, 127, 128, 129, 700, 1000, 95, 513, 640]
    q, kv, l = inputs.make_inputs(len(lens), 1000, lens, seed=101, poison_tail=True)
    ref_o, ref_l = _oracle(oracle, q, kv, l)
    print("case small_ragged num_wg", num_wg, flush=True)
    out, lse = _run(q, kv, l, num_wg=num_wg)
    _check(out, lse, ref_o, ref_l, label="small_ragged num_wg=%s" % num_wg)


@pytest.mark.parametrize("num_wg", [None, 7, 300])
def test_many_short_sequences(oracle, num_wg):
    """More sequences than one wavefront scans at once (64), many per workgroup, empty ones between."""
    g = torch.Generator().manual_seed(1234)
    lens = torch.randint(0, 401, (300,), generator=g).tolist()
    lens[5] = lens[6] = lens[64] = lens[128] = lens[299] = 0
    q, kv, l = inputs.make_inputs(300, 400, lens, seed=110, poison_tail=True)
    ref_o, ref_l = _oracle(oracle, q, kv, l)
    print("case many_short num_wg", num_wg, flush=True)
    out, lse = _run(q, kv, l, num_wg=num_wg)
    _check(out, lse, ref_o, ref_l, label="many_short num_wg=%s" % num_wg)


@pytest.mark.parametrize("num_wg", [None, 1000])
def test_thousands_of_sequences(oracle, num_wg):
    """Three thousand sequences of 0 ... 48 rows (47 chunks of 64 lengths for the wavefront-wide scans, a
    dozen sequences per workgroup, empty ones throughout, a last chunk that is not full)."""
    g = torch.Generator().manual_seed(99)
    lens = torch.randint(0, 49, (3000,), generator=g).tolist()
    for i in range(0, 3000, 7):
        lens[i] = 0
    q, kv, l = inputs.make_inputs(3000, 48, lens, seed=113, poison_tail=True)
    ref_o, ref_l = _oracle(oracle, q, kv, l)
    print("case thousands num_wg", num_wg, flush=True)
    out, lse = _run(q, kv, l, num_wg=num_wg)
    _check(out, lse, ref_o, ref_l, label="thousands num_wg=%s" % num_wg)


def test_largest_number_of_workgroups(oracle):
    """num_workgroups at its maximum (65536: a 4.3 GB workspace, a grid far larger than the unit stream,
    so almost every workgroup finds no unit and leaves at once), with 32-row and with 128-row units."""
    lens = [700, 0, 33, 1000, 129]
    q, kv, l = inputs.make_inputs(len(lens), 1000, lens, seed=114, poison_tail=True)
    ref_o, ref_l = _oracle(oracle, q, kv, l)
    dev = _dev()
    need, used = mla.mla_decode_workspace_size(len(lens), 16, 1000, 65536)
    assert used == 65536
    ws = torch.empty((need,), dtype=torch.uint8, device=dev)
    for flags in (mla.UNIT_FINE, mla.UNIT_COARSE):
        print("case largest grid flags", flags, flush=True)
        out, lse = mla.mla_decode(q.to(dev), kv.to(dev), l.to(dev), inputs.SCALE, workspace=ws, num_workgroups=65536,
                                  phases=mla.PHASE_SPLIT | mla.PHASE_COMBINE | flags)
        torch.cuda.synchronize()
        _check(out.cpu().numpy().reshape(len(lens), 16, 512).astype(np.float64), lse.cpu().numpy().astype(np.float64),
               ref_o, ref_l, label="largest grid flags=%d" % flags)
    del ws


def test_one_very_long_sequence(oracle):
    """A single sequence of 300,001 rows shared by every workgroup (176 pieces for the combine
    kernel to merge: more than one batch of its loads), next to a one-row sequence."""
    q, kv, l = inputs.make_inputs(2, 300001, [300001, 1], seed=111, poison_tail=True)
    ref_o, ref_l = _oracle(oracle, q, kv, l)
    for nwg in (None, 1000):
        print("case very_long num_wg", nwg, flush=True)
        out, lse = _run(q, kv, l, num_wg=nwg)
        _check(out, lse, ref_o, ref_l, label="very_long num_wg=%s" % nwg)


def test_empty_and_full_sequences(oracle):
    lens = [0, 384, 0, 1]
    q, kv, l = inputs.make_inputs(4, 384, lens, seed=102, poison_tail=True)
    ref_o, ref_l = _oracle(oracle, q, kv, l)
    for nwg in (None, 1, 3, 5):
        print("case empty_and_full num_wg", nwg, flush=True)
        out, lse = _run(q, kv, l, num_wg=nwg)
        _check(out, lse, ref_o, ref_l, label="empty/full num_wg=%s" % nwg)
        assert (out[0] == 0).all() and (out[2] == 0).all()
        assert np.isneginf(lse[0]).all() and np.isneginf(lse[2]).all()


def test_lengths_are_clamped_on_the_device(oracle):
    q, kv, l = inputs.make_inputs(2, 256, [256, 200], seed=103)
    ref_o, ref_l = _oracle(oracle, q, kv, l)
    wild = torch.tensor([100000, 200], dtype=torch.int32)    # first entry beyond max_seqlen_kv
    print("case clamp", flush=True)
    out, lse = _run(q, kv, wild)
    _check(out, lse, ref_o, ref_l, label="clamp")


@pytest.mark.parametrize("scale", [0.0, -0.05, 0.5])
def test_unusual_scales(oracle, scale):
    """scale 0 gives the plain mean of V and lse = ln N; a negative scale prefers the smallest
    scores; a large one makes the softmax nearly one-hot (scores of standard deviation 12)."""
    q, kv, l = inputs.make_inputs(3, 700, [700, 129, 5], seed=112, poison_tail=True)
    ref_o, ref_l = _oracle(oracle, q, kv, l, scale=scale)
    print("case scale", scale, flush=True)
    out, lse = _run(q, kv, l, scale=scale)
    _check(out, lse, ref_o, ref_l, tight=(scale != 0.5), label="scale=%g" % scale)
    if scale == 0.0:
        assert abs(lse[0, 0] - math.log(700)) < 1e-5


def test_batch_stride_larger_than_sequence(oracle):
    dev = _dev()
    q, kv, l = inputs.make_inputs(3, 300, [300, 17, 222], seed=104)
    ref_o, ref_l = _oracle(oracle, q, kv, l)
    big = torch.full((3, 300 + 52, inputs.D_QK), float("nan"), dtype=torch.bfloat16, device=dev)
    big[:, :300] = kv.to(dev)
    view = big[:, :300]                                       # batch stride 352*576, rows contiguous
    assert view.stride(0) == 352 * inputs.D_QK
    print("case batch_stride", flush=True)
    out, lse = _run(q, kv, l, kv_dev=view)
    _check(out, lse, ref_o, ref_l, label="batch_stride")


def test_growing_scores_exercise_the_rescale_path(oracle):
    # keys grow along the sequence so the running maximum keeps jumping by more than the lazy
    # threshold: the accumulator rescale (R of Algorithm 1) must run many times and stay exact.
    n = 2048
    q, kv, l = inputs.make_inputs(2, n, [n, n - 77], seed=105)
    ramp = torch.linspace(0.05, 6.0, n).view(1, n, 1)
    kv = (kv.float() * ramp).to(torch.bfloat16)
    ref_o, ref_l = _oracle(oracle, q, kv, l)
    assert ref_l.min() > 20                  # maxima climb by far more than the lazy threshold
    for nwg in (None, 1, 2):
        print("case growing_scores num_wg", nwg, flush=True)
        out, lse = _run(q, kv, l, num_wg=nwg)
        # |v| grows to ~20, so the absolute bounds scale with it
        err = np.abs(out - ref_o)
        rel = err.max() / np.abs(ref_o).max()
        print("growing max_abs %.3e rel %.3e lse %.3e" % (err.max(), rel, np.abs(lse - ref_l).max()), flush=True)
        assert rel < 2e-5
        assert np.abs(lse - ref_l).max() < 5e-5   # lse ~ 30: a few fp32 ulps


def test_split_choice_does_not_change_the_result_beyond_rounding():
    q, kv, l = inputs.make_inputs(4, 4096, [4096, 3000, 129, 2048], seed=106)
    print("case split_choice", flush=True)
    base_o, base_l = _run(q, kv, l, num_wg=1)
    for nwg in (2, 3, 16, 75, 256):
        o, s = _run(q, kv, l, num_wg=nwg)
        assert np.abs(o - base_o).max() < 1e-5
        assert np.abs(s - base_l).max() < 1e-5


def test_repeat_is_bit_identical_and_workspace_contents_do_not_matter(oracle):
    dev = _dev()
    q, kv, l = inputs.make_inputs(5, 3000, [3000, 2999, 1, 1500, 640], seed=107, poison_tail=True)
    qd, kvd, ld = q.to(dev), kv.to(dev), l.to(dev)
    need, nwg = mla.mla_decode_workspace_size(5, 16, 3000, 0)
    print("case repeat num_wg", nwg, flush=True)
    ws = torch.empty((need,), dtype=torch.uint8, device=dev)
    outs = []
    for fill in (0x00, 0xFF, 0x7F):          # 0xFF.. and 0x7F7F.. are NaN / huge as fp32
        ws.fill_(fill)
        out = torch.full((5, 1, 16, 512), float("nan"), dtype=torch.float32, device=dev)
        lse = torch.full((5, 16), float("nan"), dtype=torch.float32, device=dev)
        mla.mla_decode(qd, kvd, ld, inputs.SCALE, out=out, lse=lse, workspace=ws)
        torch.cuda.synchronize()
        outs.append((out.cpu(), lse.cpu()))
    for o, s in outs[1:]:
        assert torch.equal(o, outs[0][0]) and torch.equal(s, outs[0][1])
    ref_o, ref_l = _oracle(oracle, q, kv, l)
    _check(outs[0][0].numpy().reshape(5, 16, 512).astype(np.float64), outs[0][1].numpy().astype(np.float64),
           ref_o, ref_l, label="repeat")


def test_phases_split_then_combine_equals_one_call():
    dev = _dev()
    q, kv, l = inputs.make_inputs(2, 1024, [1024, 600], seed=108)
    qd, kvd, ld = q.to(dev), kv.to(dev), l.to(dev)
    need, _ = mla.mla_decode_workspace_size(2, 16, 1024, 5)
    ws = torch.zeros((need,), dtype=torch.uint8, device=dev)
    print("case phases", flush=True)
    o1, s1 = mla.mla_decode(qd, kvd, ld, inputs.SCALE, workspace=ws, num_workgroups=5)
    torch.cuda.synchronize()
    o2 = torch.zeros_like(o1); s2 = torch.zeros_like(s1)
    mla.mla_decode(qd, kvd, ld, inputs.SCALE, out=o2, lse=s2, workspace=ws, num_workgroups=5, phases=mla.PHASE_SPLIT)
    mla.mla_decode(qd, kvd, ld, inputs.SCALE, out=o2, lse=s2, workspace=ws, num_workgroups=5, phases=mla.PHASE_COMBINE)
    torch.cuda.synchronize()
    assert torch.equal(o1, o2) and torch.equal(s1, s2)


def test_call_can_be_captured_in_a_graph_and_replayed(oracle):
    """The library allocates nothing and never synchronises, so a call can be recorded into a HIP
    graph.  Every replay, with eager work and synchronisation in between, must reproduce the eager
    result bit for bit (the tile assignment is static)."""
    dev = _dev()
    q, kv, l = inputs.make_inputs(4, 3000, [3000, 1, 1500, 640], seed=120, poison_tail=True)
    ref_o, ref_l = _oracle(oracle, q, kv, l)
    qd, kvd, ld = q.to(dev), kv.to(dev), l.to(dev)
    need, _ = mla.mla_decode_workspace_size(4, 16, 3000, 0)
    ws = torch.empty((need,), dtype=torch.uint8, device=dev)
    out = torch.empty((4, 1, 16, 512), dtype=torch.float32, device=dev)
    lse = torch.empty((4, 16), dtype=torch.float32, device=dev)
    print("case graph", flush=True)
    mla.mla_decode(qd, kvd, ld, inputs.SCALE, out=out, lse=lse, workspace=ws)      # eager; also the one-time set-up
    torch.cuda.synchronize()
    eager_o, eager_l = out.clone(), lse.clone()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream(device=dev)
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            mla.mla_decode(qd, kvd, ld, inputs.SCALE, out=out, lse=lse, workspace=ws)
    torch.cuda.synchronize()
    for rep_ in range(4):
        out.fill_(float("nan")); lse.fill_(float("nan")); ws.fill_(0xFF)     # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager_o) and torch.equal(lse, eager_l), "replay %d" % rep_
    _check(out.cpu().numpy().reshape(4, 16, 512).astype(np.float64), lse.cpu().numpy().astype(np.float64),
           ref_o, ref_l, label="graph replay")


def test_runtime_errors_leave_outputs_untouched():
    dev = _dev()
    q, kv, l = inputs.make_inputs(2, 512, None, seed=109)
    qd, kvd, ld = q.to(dev), kv.to(dev), l.to(dev)
    out = torch.full((2, 1, 16, 512), 7.0, dtype=torch.float32, device=dev)
    lse = torch.full((2, 16), 7.0, dtype=torch.float32, device=dev)
    tiny = torch.zeros((64,), dtype=torch.uint8, device=dev)
    with pytest.raises(mla.MlaError) as e:
        mla.mla_decode(qd, kvd, ld, inputs.SCALE, out=out, lse=lse, workspace=tiny)
    assert e.value.status == mla.MLA_ERR_WORKSPACE_TOO_SMALL
    torch.cuda.synchronize()
    assert (out == 7.0).all() and (lse == 7.0).all()


# ---- the five benchmark configurations, every output element against the oracle --------------------

@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_benchmark_configs_full_parity(oracle, cfg):
    print("case config", cfg, "generating", flush=True)
    q, kv, l = inputs.make_config(cfg, poison_tail=True)
    print("case config", cfg, "gpu", flush=True)
    out, lse = _run(q, kv, l)          # the automatic plan: the launch configuration bench.py times
    print("case config", cfg, "oracle", flush=True)
    ref_o, ref_l = _oracle(oracle, q, kv, l)
    _check(out, lse, ref_o, ref_l, label="config %d" % cfg)


# ---- fp16 inputs (the paper's own precision, Section 4.1) through mla_decode_typed ------------------
# One fp16 term of P: 11 significant bits, unit round-off 2^-11 per term.  The guaranteed bound on an
# output element is therefore 2^-11 max|v| (the weights sum to one), 2.4e-3 at max|v| = 4.9: reached
# only if every rounding error had the same sign and one row carried all the weight.  What binds is
# the RMSE: the error model in tests/test_oracle.py gives 2e-5 at KV 512 and less at longer KV.

F16_RMSE, F16_LSE = 4e-5, 2e-5
F16_UNIT_ROUNDOFF = 2.0 ** -11


def _f16_max_abs_bound(kv):
    vals = kv[:, :, :inputs.D_V].float()
    vals = vals[torch.isfinite(vals)]                          # the rows past the lengths are NaN
    return F16_UNIT_ROUNDOFF * (float(vals.abs().max()) if vals.numel() else 0.0) + 1e-5


def _oracle_f16(oracle, q, kv, lens, scale=inputs.SCALE):
    o, l = oracle.decode_general(inputs.bits16(q), inputs.bits16(kv), lens.numpy(), scale, inputs.D_V, dtype=oracle.F16)
    return o[:, 0], l[:, 0]


def _check_f16(out, lse, ref_o, ref_l, label, kv):
    _check(out, lse, ref_o, ref_l, tight=False, label=label)
    err = np.abs(out - ref_o)
    fin = np.isfinite(ref_l)
    assert err.max() <= _f16_max_abs_bound(kv) and math.sqrt(float((err ** 2).mean())) <= F16_RMSE, label
    assert not fin.any() or np.abs(lse[fin] - ref_l[fin]).max() <= F16_LSE, label


@pytest.mark.parametrize("num_wg", [None, 1, 7, 1000])
def test_fp16_small_ragged_elementwise(oracle, num_wg):
    lens = [1, 31, 32, 33, 127, 128, 129, 700, 1000, 0, 513, 640]
    q, kv, l = inputs.make_inputs(len(lens), 1000, lens, seed=201, poison_tail=True, dtype=torch.float16)
    ref_o, ref_l = _oracle_f16(oracle, q, kv, l)
    print("case fp16 small_ragged num_wg", num_wg, flush=True)
    out, lse = _run(q, kv, l, num_wg=num_wg)
    _check_f16(out, lse, ref_o, ref_l, "fp16 small_ragged num_wg=%s" % num_wg, kv)


@pytest.mark.parametrize("cfg", [1, 2, 4, 5])
def test_fp16_benchmark_configs_full_parity(oracle, cfg):
    print("case fp16 config", cfg, "generating", flush=True)
    q, kv, l = inputs.make_config(cfg, poison_tail=True, dtype=torch.float16)
    print("case fp16 config", cfg, "gpu", flush=True)
    out, lse = _run(q, kv, l)
    print("case fp16 config", cfg, "oracle", flush=True)
    ref_o, ref_l = _oracle_f16(oracle, q, kv, l)
    _check_f16(out, lse, ref_o, ref_l, "fp16 config %d" % cfg, kv)


# ---- more than one query token per sequence (Section 3.1: one or two tokens per decoding step) ------

def _oracle_general(oracle, q, kv, lens, dtype):
    return oracle.decode_general(inputs.bits16(q), inputs.bits16(kv), lens.numpy(), inputs.SCALE, inputs.D_V,
                                 dtype=oracle.F16 if dtype == torch.float16 else oracle.BF16)


def _run_general(q, kv, lens, num_wg=None):
    dev = _dev()
    out, lse = mla.mla_decode(q.to(dev), kv.to(dev), lens.to(dev), inputs.SCALE, num_workgroups=num_wg)
    torch.cuda.synchronize()
    b, ql = q.shape[0], q.shape[1]
    return (out.cpu().numpy().reshape(b * ql, 16, inputs.D_V).astype(np.float64),
            lse.cpu().numpy().reshape(b * ql, 16).astype(np.float64))


@pytest.mark.parametrize("q_len", [2, 3, 4, 5, 8])
@pytest.mark.parametrize("num_wg", [None, 1, 5, 300])
def test_several_query_tokens_small_ragged(oracle, q_len, num_wg):
    # lengths below q_len leave the first query tokens without any row (out 0, lse -inf)
    lens = [0, 1, 2, 3, 31, 33, 128, 129, 700, 1000, 257, 640]
    q, kv, l = inputs.make_inputs(len(lens), 1000, lens, seed=401 + q_len, poison_tail=True, q_len=q_len)
    ref_o, ref_l = _oracle_general(oracle, q, kv, l, torch.bfloat16)
    print("case q_len", q_len, "num_wg", num_wg, flush=True)
    out, lse = _run_general(q, kv, l, num_wg=num_wg)
    _check(out, lse, ref_o.reshape(-1, 16, inputs.D_V), ref_l.reshape(-1, 16), label="q_len=%d num_wg=%s" % (q_len, num_wg))


@pytest.mark.parametrize("q_len", [2, 4])
def test_several_query_tokens_many_sequences(oracle, q_len):
    # pieces that cross sequence boundaries, with one workgroup per team (2 tokens) and with teams of two (4)
    g = torch.Generator().manual_seed(4321)
    lens = torch.randint(0, 300, (70,), generator=g).tolist()
    q, kv, l = inputs.make_inputs(70, 300, lens, seed=412, poison_tail=True, q_len=q_len)
    ref_o, ref_l = _oracle_general(oracle, q, kv, l, torch.bfloat16)
    for nwg in (None, 9):
        print("case q_len", q_len, "many sequences num_wg", nwg, flush=True)
        out, lse = _run_general(q, kv, l, num_wg=nwg)
        _check(out, lse, ref_o.reshape(-1, 16, inputs.D_V), ref_l.reshape(-1, 16), label="q_len=%d many num_wg=%s" % (q_len, nwg))


def test_two_query_tokens_fp16(oracle):
    lens = [5, 640, 1, 2000]
    q, kv, l = inputs.make_inputs(4, 2000, lens, seed=411, poison_tail=True, q_len=2, dtype=torch.float16)
    ref_o, ref_l = _oracle_general(oracle, q, kv, l, torch.float16)
    print("case q_len 2 fp16", flush=True)
    out, lse = _run_general(q, kv, l)
    _check_f16(out, lse, ref_o.reshape(-1, 16, inputs.D_V), ref_l.reshape(-1, 16), "q_len=2 fp16", kv)


def test_two_query_tokens_headline_shape(oracle):
    """Batch 16, KV 65536, two query tokens: the launch configuration `bench.py --q-len 2` times."""
    print("case q_len 2 headline generating", flush=True)
    q, kv, l = inputs.make_inputs(16, 65536, None, seed=inputs.BASE_SEED + 42, q_len=2)
    print("case q_len 2 headline gpu", flush=True)
    out, lse = _run_general(q, kv, l)
    print("case q_len 2 headline oracle", flush=True)
    ref_o, ref_l = _oracle_general(oracle, q, kv, l, torch.bfloat16)
    _check(out, lse, ref_o.reshape(-1, 16, inputs.D_V), ref_l.reshape(-1, 16), label="q_len=2 headline")


def test_two_query_tokens_ragged_config(oracle):
    """Configuration 5 (batch 32, lengths 1024 ... 65536) with two query tokens: pieces that cross
    sequence boundaries at full size, in the launch configuration of the automatic plan."""
    print("case q_len 2 config 5 generating", flush=True)
    q, kv, l = inputs.make_config(5, poison_tail=True, q_len=2)
    print("case q_len 2 config 5 gpu", flush=True)
    out, lse = _run_general(q, kv, l)
    print("case q_len 2 config 5 oracle", flush=True)
    ref_o, ref_l = _oracle_general(oracle, q, kv, l, torch.bfloat16)
    _check(out, lse, ref_o.reshape(-1, 16, inputs.D_V), ref_l.reshape(-1, 16), label="q_len=2 config 5")


def test_two_query_tokens_repeat_is_bit_identical_and_workspace_contents_do_not_matter():
    """The wavefront pairs read each other's LDS tiles between barriers; the result must not depend on
    timing or on what the workspace held (0xFF.. is NaN as fp32)."""
    dev = _dev()
    q, kv, l = inputs.make_inputs(5, 3000, [3000, 2999, 2, 1500, 641], seed=131, poison_tail=True, q_len=2)
    qd, kvd, ld = q.to(dev), kv.to(dev), l.to(dev)
    need, _ = mla.mla_decode_workspace_size(5 * 2, 16, 3000, 0)
    ws = torch.empty((need,), dtype=torch.uint8, device=dev)
    outs = []
    for fill in (0x00, 0xFF, 0x7F, 0x00):
        ws.fill_(fill)
        out = torch.full((5, 2, 16, 512), float("nan"), dtype=torch.float32, device=dev)
        lse = torch.full((5, 2, 16), float("nan"), dtype=torch.float32, device=dev)
        print("case q_len 2 repeat fill", fill, flush=True)
        mla.mla_decode(qd, kvd, ld, inputs.SCALE, out=out, lse=lse, workspace=ws)
        torch.cuda.synchronize()
        outs.append((out.cpu(), lse.cpu()))
    assert torch.isfinite(outs[0][0]).all()
    for o, s in outs[1:]:
        assert torch.equal(o, outs[0][0]) and torch.equal(s, outs[0][1])


def test_automatic_plan_follows_the_shape():
    _dev()
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    long_kv = mla.mla_decode_planned_workgroups(16, 1, 65536)
    assert long_kv == cus * 13 // 16
    assert mla.mla_decode_planned_workgroups(16, 1, 4096) == cus          # 512 units: a short stream
    assert mla.mla_decode_planned_workgroups(16, 2, 65536) == cus         # several query tokens
    assert mla.mla_decode_workspace_size(16, 16, 65536, 0)[1] == long_kv


def test_seeded_random_small_cases(oracle):
    """Two hundred seeded draws of (batch, lengths, q_len, element type, number of workgroups): the piece
    boundaries, tile tails, causal limits and team shapes fall differently in each, at sizes the oracle
    finishes at once."""
    rng = np.random.default_rng(20250601)
    for case in range(200):
        batch = int(rng.integers(1, 12))
        q_len = int(rng.choice([1, 1, 2, 2, 3, 4, 5, 8]))
        max_len = int(rng.choice([33, 130, 300, 900, 2100]))
        lens = [int(x) for x in rng.integers(0, max_len + 1, size=batch)]
        if case % 5 == 0:
            lens[int(rng.integers(0, batch))] = max_len          # one sequence fills its allocation
        num_wg = int(rng.integers(1, 300)) if case % 3 else None
        dtype = torch.float16 if case % 4 == 3 else torch.bfloat16
        q, kv, l = inputs.make_inputs(batch, max_len, lens, seed=7000 + case, poison_tail=True, q_len=q_len, dtype=dtype)
        ref_o, ref_l = _oracle_general(oracle, q, kv, l, dtype)
        label = "random case %d: batch %d q_len %d lens %s num_wg %s %s" % (case, batch, q_len, lens, num_wg, str(dtype)[6:])
        print(label, flush=True)
        out, lse = _run_general(q, kv, l, num_wg=num_wg)
        if dtype == torch.float16:
            # One fp16 rounding of each probability: relative error at most 2^-11, 2^-11 / sqrt(3) rms
            # per term, so an output element is off by that times sqrt(sum_t w_t^2 v_t^2) rms: up to
            # 2.8e-4 |v| when one row carries all the weight, as in the shortest of these sequences, and by
            # at most 2^-11 max|v| (the weights sum to one).  Over a whole case, whose sequences are
            # mostly hundreds of rows long, the RMSE stays below 1.5e-4.
            o, rl = ref_o.reshape(-1, 16, inputs.D_V), ref_l.reshape(-1, 16)
            assert np.isfinite(out).all(), label
            err = np.abs(out - o)
            fin = np.isfinite(rl)
            assert np.isneginf(lse[~fin]).all(), label
            assert err.max() <= _f16_max_abs_bound(kv) and math.sqrt(float((err ** 2).mean())) <= 1.5e-4, label
            assert not fin.any() or np.abs(lse[fin] - rl[fin]).max() <= F16_LSE, label
        else:
            _check(out, lse, ref_o.reshape(-1, 16, inputs.D_V), ref_l.reshape(-1, 16), label=label)


# ---- the original (non-transposed) orientation of Section 3.1, kept for the comparison of the two ----

DIRECT = mla.PHASE_SPLIT | mla.PHASE_COMBINE | mla.ORIENT_DIRECT


def _run_direct(q, kv, lens, num_wg=None):
    dev = _dev()
    out, lse = mla.mla_decode(q.to(dev), kv.to(dev), lens.to(dev), inputs.SCALE, num_workgroups=num_wg, phases=DIRECT)
    torch.cuda.synchronize()
    return (out.cpu().numpy().reshape(q.shape[0], 16, inputs.D_V).astype(np.float64),
            lse.cpu().numpy().astype(np.float64))


@pytest.mark.parametrize("num_wg", [None, 1, 7, 300])
def test_direct_orientation_small_ragged(oracle, num_wg):
    lens = [1, 31, 32, 33, 127, 128, 129, 700, 1000, 0, 513, 640]
    q, kv, l = inputs.make_inputs(len(lens), 1000, lens, seed=501, poison_tail=True)
    ref_o, ref_l = _oracle(oracle, q, kv, l)
    print("case direct small_ragged num_wg", num_wg, flush=True)
    out, lse = _run_direct(q, kv, l, num_wg=num_wg)
    _check(out, lse, ref_o, ref_l, label="direct small_ragged num_wg=%s" % num_wg)


def test_direct_orientation_rescale_path(oracle):
    # per-head rescale factors: heads whose maxima jump at different tiles
    n = 2048
    q, kv, l = inputs.make_inputs(2, n, [n, n - 77], seed=502)
    ramp = torch.linspace(0.05, 6.0, n).view(1, n, 1)
    kv = (kv.float() * ramp).to(torch.bfloat16)
    ref_o, ref_l = _oracle(oracle, q, kv, l)
    print("case direct growing_scores", flush=True)
    out, lse = _run_direct(q, kv, l, num_wg=2)
    assert np.abs(out - ref_o).max() / np.abs(ref_o).max() < 2e-5
    assert np.abs(lse - ref_l).max() < 5e-5


@pytest.mark.parametrize("cfg", [1, 4, 5])
def test_direct_orientation_benchmark_configs(oracle, cfg):
    print("case direct config", cfg, "generating", flush=True)
    q, kv, l = inputs.make_config(cfg, poison_tail=True)
    print("case direct config", cfg, "gpu", flush=True)
    out, lse = _run_direct(q, kv, l)
    print("case direct config", cfg, "oracle", flush=True)
    ref_o, ref_l = _oracle(oracle, q, kv, l)
    _check(out, lse, ref_o, ref_l, label="direct config %d" % cfg)


# ---- the partition as the kernels derive it on the device, against its plain definition ---------------

def test_device_plan_equals_its_definition():
    """`mla_decode_plan_table` runs the kernels' own device functions (wavefront-wide sums and scans over
    the lengths, the range, locate and bound rules).  Here the same table is built from the definition
    with numpy prefix sums and a brute-force search over the teams' ranges."""
    dev = _dev()
    rng = np.random.default_rng(77)
    for case in range(120):
        batch = int(rng.integers(1, 40)) if case % 4 else int(rng.integers(65, 300))
        max_len = int(rng.choice([1, 33, 130, 700, 4096, 70000]))
        lens = rng.integers(-3, max_len + 50, size=batch)
        lens[rng.random(batch) < 0.15] = 0
        if case % 9 == 0:
            lens[:] = 0
        q_len = int(rng.choice([1, 1, 2, 3, 5, 8]))
        num_wg = int(rng.choice([1, 2, 7, 64, 208, 256, 999]))
        flags = [0, mla.UNIT_FINE, mla.UNIT_COARSE][case % 3]
        print("plan case %d: batch %d max_len %d q_len %d num_wg %d flags %d" % (case, batch, max_len, q_len, num_wg, flags), flush=True)
        ld = torch.tensor(lens, dtype=torch.int32, device=dev)
        table, teams, unit = mla.mla_decode_plan_table(ld, q_len, max_len, num_wg, flags)
        torch.cuda.synchronize()
        table = table.cpu().numpy()
        share = 2 if q_len >= 2 else 1
        members = -(-q_len // share)
        assert teams == max(1, num_wg // members)
        if flags == mla.UNIT_FINE:
            assert unit == 32
        elif flags == mla.UNIT_COARSE:
            assert unit == 128
        else:
            assert unit == (32 if 4 * batch * -(-max_len // 32) <= teams else 128)
        units = -(-np.clip(lens, 0, max_len) // unit)
        ends = np.cumsum(units)
        firsts = ends - units
        total = int(ends[-1])
        active = min(total, teams)
        ranges = [(k * total // active, (k + 1) * total // active) for k in range(active)]
        for k in range(teams):
            rec = table[k]
            assert rec[0] == total and rec[1] == active
            if k >= active:
                assert (rec[2:6] == -1).all()
                continue
            lo, hi = ranges[k]
            b = int(np.searchsorted(ends, lo, side="right"))
            assert (rec[2], rec[3], rec[4], rec[5], rec[6]) == (lo, hi, b, firsts[b], min(max(int(lens[b]), 0), max_len)), (k, rec)
        for b in range(batch):
            rec = table[teams + b]
            assert (rec[0], rec[1], rec[2]) == (total, firsts[b], units[b]), (b, rec)
            if units[b] == 0:
                assert rec[3] == -1 and rec[4] == -1
                continue
            meets = [k for k, (lo, hi) in enumerate(ranges) if lo < ends[b] and hi > firsts[b]]
            assert (rec[3], rec[4]) == (meets[0], meets[-1]) and meets == list(range(meets[0], meets[-1] + 1)), (b, rec)


# ---- the grid of the paper's Figure 1 (Section 4.1: batch 16 and 32, KV length 512 ... 64K), at its own shapes ----
# `bench.py --sweep` times these launches; here every output element of every point is compared with the
# oracle, in the automatic plan.  Few long sequences (where the widest merge runs) and many short ones are added.

_GRID = [(b, n) for b in (16, 32) for n in (512, 1024, 2048, 4096, 8192, 16384, 32768, 65536)] + \
        [(1, 65536), (2, 65536), (4, 65536), (128, 1024)]
_grid_cache = {}


def _grid_inputs(batch, n):
    """Seeded inputs of one grid point: the first n rows of one draw per batch size (seed by batch size), so
    that the sixteen points cost two draws of the longest shape."""
    full_n = 65536 if batch <= 32 else n
    if _grid_cache.get("key") != (batch, full_n):
        _grid_cache.clear()
        q, kv, _ = inputs.make_inputs(batch, full_n, None, seed=inputs.BASE_SEED + 100 + batch)
        _grid_cache.update(key=(batch, full_n), q=q, kv=kv)
    return _grid_cache["q"], _grid_cache["kv"][:, :n].contiguous(), torch.full((batch,), n, dtype=torch.int32)


@pytest.mark.parametrize("batch,n", _GRID)
def test_figure_grid_full_parity(oracle, batch, n):
    dev = _dev()
    print("case grid batch", batch, "kv", n, "generating", flush=True)
    q, kv, l = _grid_inputs(batch, n)
    need, nwg = mla.mla_decode_workspace_size(batch, 16, n, 0)
    ws = torch.full((need,), 0xFF, dtype=torch.uint8, device=dev)                  # NaN as fp32
    out = torch.full((batch, 1, 16, 512), float("nan"), dtype=torch.float32, device=dev)
    lse = torch.full((batch, 16), float("nan"), dtype=torch.float32, device=dev)
    print("case grid batch", batch, "kv", n, "gpu, workgroups", nwg, flush=True)
    mla.mla_decode(q.to(dev), kv.to(dev), l.to(dev), inputs.SCALE, out=out, lse=lse, workspace=ws)
    torch.cuda.synchronize()
    print("case grid batch", batch, "kv", n, "oracle", flush=True)
    ref_o, ref_l = _oracle(oracle, q, kv, l)
    _check(out.cpu().numpy().reshape(batch, 16, 512).astype(np.float64), lse.cpu().numpy().astype(np.float64),
           ref_o, ref_l, label="grid batch %d kv %d" % (batch, n))
    if (batch, n) == _GRID[-1]:
        _grid_cache.clear()


def test_two_threads_on_two_streams_equal_the_serial_results():
    """The entry points may be called from several threads.  Two threads, each with its own stream,
    workspace and outputs, call the library at the same time (ctypes releases the interpreter lock during
    a call) with different shapes and element types, fifty times each; every result must equal, bit for
    bit, what the same call returns when it runs alone."""
    import threading
    dev = _dev()
    jobs = []
    for seed, lens, q_len, dtype in ((301, [3000, 17, 1500, 640, 129], 1, torch.bfloat16),
                                     (302, [2048, 2047, 5, 900], 2, torch.float16)):
        q, kv, l = inputs.make_inputs(len(lens), max(lens), lens, seed=seed, poison_tail=True, q_len=q_len, dtype=dtype)
        qd, kvd, ld = q.to(dev), kv.to(dev), l.to(dev)
        need, _ = mla.mla_decode_workspace_size(len(lens) * q_len, 16, max(lens), 0)
        serial_o, serial_l = mla.mla_decode(qd, kvd, ld, inputs.SCALE)
        torch.cuda.synchronize()
        jobs.append(dict(q=qd, kv=kvd, lens=ld, need=need, want_o=serial_o.clone(), want_l=serial_l.clone(),
                         stream=torch.cuda.Stream(device=dev), bad=[]))
    start = threading.Barrier(2)

    def work(job):
        with torch.cuda.stream(job["stream"]):
            ws = torch.full((job["need"],), 0xFF, dtype=torch.uint8, device=dev)
            start.wait()
            for i in range(50):
                out = torch.full_like(job["want_o"], float("nan"))
                lse = torch.full_like(job["want_l"], float("nan"))
                mla.mla_decode(job["q"], job["kv"], job["lens"], inputs.SCALE, out=out, lse=lse, workspace=ws)
                job["stream"].synchronize()
                if not (torch.equal(out, job["want_o"]) and torch.equal(lse, job["want_l"])):
                    job["bad"].append(i)

    print("case two threads", flush=True)
    threads = [threading.Thread(target=work, args=(job,)) for job in jobs]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=100)
    assert not any(t.is_alive() for t in threads)
    assert jobs[0]["bad"] == [] and jobs[1]["bad"] == []


# ---- the other kernel variants at grid shapes: fp16 inputs and two query tokens -----------------------

@pytest.mark.parametrize("batch,n", [(16, 4096), (32, 16384)])
def test_figure_grid_fp16_and_two_tokens(oracle, batch, n):
    """Two points of the Figure-1 grid with fp16 inputs (the paper's own precision) and with two query
    tokens per sequence (Section 3.1), every output element against the oracle, automatic plan."""
    print("case grid variants batch", batch, "kv", n, "fp16", flush=True)
    q, kv, l = inputs.make_inputs(batch, n, None, seed=inputs.BASE_SEED + 300 + batch, dtype=torch.float16)
    out, lse = _run(q, kv, l)
    ref_o, ref_l = _oracle_f16(oracle, q, kv, l)
    _check_f16(out, lse, ref_o, ref_l, "grid fp16 batch %d kv %d" % (batch, n), kv)
    print("case grid variants batch", batch, "kv", n, "two tokens", flush=True)
    q, kv, l = inputs.make_inputs(batch, n, None, seed=inputs.BASE_SEED + 400 + batch, q_len=2)
    out, lse = _run_general(q, kv, l)
    ref_o, ref_l = _oracle_general(oracle, q, kv, l, torch.bfloat16)
    _check(out, lse, ref_o.reshape(-1, 16, inputs.D_V), ref_l.reshape(-1, 16), label="grid q_len 2 batch %d kv %d" % (batch, n))
