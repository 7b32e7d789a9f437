"""Pins for the fp64 CPU oracle (no GPU).

The paper prints no worked numeric example for the attention computation, so the
oracle is pinned by what the mathematics fixes: brute force in exact rational /
high-precision arithmetic on tiny inputs, closed forms, invariants, the
transposed formulation of equations (1)-(4), an LSE merge over arbitrary
partitions, and library routines (numpy / torch float64) on medium inputs.
Each check is chosen so that a plausible slip (dropped scale, wrong V slice,
softmax over the wrong axis, wrong sign in the rescale, base-2 log) fails it.
"""
import math
from decimal import Decimal, getcontext

import numpy as np
import pytest
import torch

from paper_2506_01969_amd import inputs

getcontext().prec = 60


def _decode_bf16(bits):
    """Independent bf16 -> float64 decode (numpy bit shift), not the oracle's."""
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def _small(batch, n, heads, d_qk, seed, seqlens=None):
    q, kv, lens = inputs.make_inputs(batch, n, seqlens, seed=seed, heads=heads, d_qk=d_qk)
    return inputs.bf16_bits(q), inputs.bf16_bits(kv), lens.numpy()


def _bits_from_float(a):
    return inputs.bf16_bits(torch.as_tensor(np.asarray(a, dtype=np.float32)).to(torch.bfloat16))


# ---- 1. brute force, exact-ish arithmetic, no max subtraction ------------------------------

@pytest.mark.parametrize("n", [1, 2, 3, 17])
def test_brute_force_decimal(oracle, n):
    heads, d_qk, d_v = 3, 8, 5
    scale = 0.37
    qb, kvb, lens = _small(2, n, heads, d_qk, seed=11 + n)
    out, lse = oracle.decode(qb, kvb, lens, scale, d_v)
    q = _decode_bf16(qb).reshape(2, heads, d_qk)
    kv = _decode_bf16(kvb)
    for b in range(2):
        for h in range(heads):
            s = [sum(Decimal(float(q[b, h, c])) * Decimal(float(kv[b, t, c])) for c in range(d_qk))
                 * Decimal(scale) for t in range(n)]
            e = [x.exp() for x in s]           # naive exp, no stabilisation
            z = sum(e)
            for d in range(d_v):
                ref = sum(e[t] * Decimal(float(kv[b, t, d])) for t in range(n)) / z
                assert abs(out[b, h, d] - float(ref)) < 1e-13
            assert abs(lse[b, h] - float(z.ln())) < 1e-13


def test_closed_form_three_tokens(oracle):
    # d_qk = 2, d_v = 1, scale = 1, q = (1, 0); keys (0, x), (1, x), (2, x) -> scores 0, 1, 2.
    q = _bits_from_float([[[[1.0, 0.0]]]])
    kv = _bits_from_float([[[0.0, 7.0], [1.0, -3.0], [2.0, 5.0]]])
    out, lse = oracle.decode(q, kv, np.array([3], dtype=np.int32), 1.0, 1)
    e = Decimal(1).exp()
    z = 1 + e + e * e
    assert abs(out[0, 0, 0] - float((e + 2 * e * e) / z)) < 1e-15
    assert abs(lse[0, 0] - float(z.ln())) < 1e-15
    # the same with scale = 0.5: scores 0, .5, 1 -> catches a dropped or squared scale
    out, lse = oracle.decode(q, kv, np.array([3], dtype=np.int32), 0.5, 1)
    r = Decimal("0.5").exp()
    z = 1 + r + r * r
    assert abs(out[0, 0, 0] - float((r + 2 * r * r) / z)) < 1e-15
    assert abs(lse[0, 0] - float(z.ln())) < 1e-15


# ---- 2. rows of P sum to one ----------------------------------------------------------------

def test_probabilities_sum_to_one(oracle):
    qb, kvb, lens = _small(2, 300, 4, 32, seed=5, seqlens=[300, 123])
    for b in range(2):
        for h in range(4):
            p = oracle.probs(qb, kvb, lens, 0.21, b, h)
            assert p.shape == (lens[b],)
            assert (p > 0).all()
            assert abs(math.fsum(p.tolist()) - 1.0) < 1e-12


def test_probabilities_by_value(oracle):
    """Each probability against exp(s_t - lse) with the scores and the log-sum-exp from numpy in float64 on
    independently decoded inputs (bf16 bits << 16 reinterpreted as float32): a dropped, squared or misplaced
    scale, a wrong head or a shifted row in the probability routine changes the values, not their sum."""
    qb, kvb, lens = _small(2, 300, 4, 32, seed=6, seqlens=[300, 123])
    dec = lambda bits: (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    qf, kvf = dec(qb), dec(kvb)
    scale = 0.21
    for b in range(2):
        for h in range(4):
            s = scale * (kvf[b, :lens[b]] @ qf[b].reshape(4, 32)[h])
            want = np.exp(s - (s.max() + np.log(np.exp(s - s.max()).sum())))
            got = oracle.probs(qb, kvb, lens, scale, b, h)
            np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-15)
            # and the probabilities reproduce the oracle's own output when applied to V by numpy
            out, _ = oracle.decode(qb, kvb, lens, scale, 20)
            np.testing.assert_allclose(out[b, h], got @ kvf[b, :lens[b], :20], rtol=0, atol=1e-13)


# ---- 3. constant K / zero q -----------------------------------------------------------------

def test_constant_k_returns_that_row(oracle):
    heads, d_qk, d_v, n = 4, 16, 12, 37
    g = torch.Generator().manual_seed(3)
    row = torch.randn((d_qk,), generator=g).to(torch.bfloat16)
    q = torch.randn((1, 1, heads, d_qk), generator=g).to(torch.bfloat16)
    kv = row.expand(1, n, d_qk).contiguous()
    scale = 0.3
    out, lse = oracle.decode(inputs.bf16_bits(q), inputs.bf16_bits(kv), np.array([n], np.int32), scale, d_v)
    rowd = row.double().numpy()
    for h in range(heads):
        np.testing.assert_allclose(out[0, h], rowd[:d_v], rtol=0, atol=1e-14)
        s = scale * float(np.dot(q[0, 0, h].double().numpy(), rowd))
        assert abs(lse[0, h] - (s + math.log(n))) < 1e-12


def test_zero_q_gives_mean_of_v(oracle):
    heads, d_qk, d_v, n = 2, 24, 20, 101
    qb, kvb, lens = _small(1, n, heads, d_qk, seed=8)
    qb = np.zeros_like(qb)
    out, lse = oracle.decode(qb, kvb, lens, 0.5, d_v)
    mean = _decode_bf16(kvb)[0, :, :d_v].mean(axis=0)
    for h in range(heads):
        np.testing.assert_allclose(out[0, h], mean, rtol=0, atol=1e-14)
        assert abs(lse[0, h] - math.log(n)) < 1e-13


# ---- 4. transposed formulation, equations (1)-(4) -------------------------------------------

def test_transposed_equals_direct(oracle):
    qb, kvb, lens = _small(3, 200, 16, 64, seed=21, seqlens=[200, 1, 77])
    o1, l1 = oracle.decode(qb, kvb, lens, 0.11, 48)
    o2, l2 = oracle.decode_transposed(qb, kvb, lens, 0.11, 48)
    np.testing.assert_allclose(o1, o2, rtol=0, atol=1e-13)
    np.testing.assert_allclose(l1, l2, rtol=0, atol=1e-13)


def test_transposed_real_dims(oracle):
    qb, kvb, lens = _small(1, 96, inputs.NUM_HEADS, inputs.D_QK, seed=22)
    o1, l1 = oracle.decode(qb, kvb, lens, inputs.SCALE, inputs.D_V)
    o2, l2 = oracle.decode_transposed(qb, kvb, lens, inputs.SCALE, inputs.D_V)
    np.testing.assert_allclose(o1, o2, rtol=0, atol=1e-13)
    np.testing.assert_allclose(l1, l2, rtol=0, atol=1e-13)


# ---- 5. special cases and invariances -------------------------------------------------------

def test_single_token(oracle):
    qb, kvb, lens = _small(2, 1, 4, 16, seed=2)
    scale = 0.25
    out, lse = oracle.decode(qb, kvb, lens, scale, 10)
    q = _decode_bf16(qb).reshape(2, 4, 16)
    kv = _decode_bf16(kvb)
    for b in range(2):
        for h in range(4):
            np.testing.assert_array_equal(out[b, h], kv[b, 0, :10])
            assert abs(lse[b, h] - scale * float(np.dot(q[b, h], kv[b, 0]))) < 1e-14


def test_one_dominant_token(oracle):
    heads, d_qk, d_v, n = 2, 8, 6, 50
    qb, kvb, lens = _small(1, n, heads, d_qk, seed=4)
    q = np.zeros((1, 1, heads, d_qk), np.float32); q[..., 7] = 1.0
    kv = _decode_bf16(kvb).astype(np.float32); kv[0, :, 7] = 0.0; kv[0, 13, 7] = 64.0
    out, lse = oracle.decode(_bits_from_float(q), _bits_from_float(kv), lens, 1.0, d_v)
    for h in range(heads):
        np.testing.assert_allclose(out[0, h], kv[0, 13, :d_v].astype(np.float64), atol=1e-12)
        assert abs(lse[0, h] - 64.0) < 1e-12


def test_shift_of_scores_moves_only_lse(oracle):
    # column 15 lies outside V (d_v = 12); q = 1 there; a constant in that key column adds
    # scale * constant to every score: out is unchanged, lse moves by exactly that.
    heads, d_qk, d_v, n = 3, 16, 12, 64
    qb, kvb, lens = _small(1, n, heads, d_qk, seed=6)
    q = _decode_bf16(qb).astype(np.float32).reshape(1, 1, heads, d_qk); q[..., 15] = 1.0
    kv = _decode_bf16(kvb).astype(np.float32)
    kv_a = kv.copy(); kv_a[..., 15] = 0.0
    kv_b = kv.copy(); kv_b[..., 15] = 8.0
    oa, la = oracle.decode(_bits_from_float(q), _bits_from_float(kv_a), lens, 0.5, d_v)
    ob, lb = oracle.decode(_bits_from_float(q), _bits_from_float(kv_b), lens, 0.5, d_v)
    np.testing.assert_allclose(oa, ob, rtol=0, atol=1e-14)
    np.testing.assert_allclose(lb - la, 4.0, rtol=0, atol=1e-13)


def test_token_permutation_invariance(oracle):
    qb, kvb, lens = _small(1, 129, 4, 32, seed=9)
    perm = np.random.default_rng(0).permutation(129)
    o1, l1 = oracle.decode(qb, kvb, lens, 0.2, 24)
    o2, l2 = oracle.decode(qb, np.ascontiguousarray(kvb[:, perm]), lens, 0.2, 24)
    np.testing.assert_allclose(o1, o2, rtol=0, atol=1e-14)
    np.testing.assert_allclose(l1, l2, rtol=0, atol=1e-14)


def test_length_mask_ignores_tail_rows(oracle):
    qb, kvb, lens = _small(2, 80, 4, 32, seed=10, seqlens=[80, 33])
    q, kv, _ = inputs.make_inputs(2, 80, [80, 33], seed=10, heads=4, d_qk=32, poison_tail=True)
    o1, l1 = oracle.decode(qb, kvb, lens, 0.2, 24)
    o2, l2 = oracle.decode(inputs.bf16_bits(q), inputs.bf16_bits(kv), lens, 0.2, 24)
    np.testing.assert_array_equal(o1, o2)
    np.testing.assert_array_equal(l1, l2)


def test_empty_sequence(oracle):
    qb, kvb, lens = _small(2, 16, 2, 8, seed=12, seqlens=[0, 5])
    out, lse = oracle.decode(qb, kvb, lens, 1.0, 4)
    assert (out[0] == 0).all() and np.isneginf(lse[0]).all()
    assert np.isfinite(out[1]).all() and np.isfinite(lse[1]).all()
    ot, lt = oracle.decode_transposed(qb, kvb, lens, 1.0, 4)
    assert (ot[0] == 0).all() and np.isneginf(lt[0]).all()


# ---- 6. split invariance: any partition merged by LSE gives the unsplit result --------------

@pytest.mark.parametrize("cuts", [[0, 250], [0, 1, 250], [0, 64, 128, 192, 250], [0, 100, 100, 249, 250, 300]])
def test_split_merge_invariance(oracle, cuts):
    heads, d_qk, d_v = 4, 32, 24
    qb, kvb, lens = _small(2, 250, heads, d_qk, seed=14, seqlens=[250, 90])
    full_o, full_l = oracle.decode(qb, kvb, lens, 0.3, d_v)
    parts = [oracle.decode_range(qb, kvb, lens, 0.3, d_v, cuts[i], cuts[i + 1]) for i in range(len(cuts) - 1)]
    for b in range(2):
        for h in range(heads):
            po = np.stack([p[0][b, h] for p in parts])
            pl = np.array([p[1][b, h] for p in parts])
            o, l = oracle.merge(po, pl)
            np.testing.assert_allclose(o, full_o[b, h], rtol=0, atol=1e-13)
            assert abs(l - full_l[b, h]) < 1e-13


def test_merge_matches_independent_formula(oracle):
    rng = np.random.default_rng(1)
    po = rng.standard_normal((5, 7))
    pl = rng.standard_normal(5) * 3
    pl[2] = -np.inf
    o, l = oracle.merge(po, pl)
    w = np.exp(pl)                                   # naive, no max subtraction
    np.testing.assert_allclose(o, (w[:, None] * po).sum(0) / w.sum(), rtol=1e-13)
    assert abs(l - math.log(w.sum())) < 1e-13
    o, l = oracle.merge(po[:2], np.array([-np.inf, -np.inf]))
    assert (o == 0).all() and l == -np.inf


# ---- 7. library cross-checks at the real head dimensions ------------------------------------

def test_against_numpy_and_torch_float64(oracle):
    q, kv, lens = inputs.make_inputs(2, 700, [700, 333], seed=30)
    qb, kvb = inputs.bf16_bits(q), inputs.bf16_bits(kv)
    out, lse = oracle.decode(qb, kvb, lens.numpy(), inputs.SCALE, inputs.D_V)
    for b in range(2):
        n = int(lens[b])
        qd = q[b, 0].double()
        kd = kv[b, :n].double()
        s = (qd @ kd.T) * inputs.SCALE
        ref = torch.softmax(s, dim=-1) @ kd[:, :inputs.D_V]
        np.testing.assert_allclose(out[b], ref.numpy(), rtol=0, atol=1e-13)
        np.testing.assert_allclose(lse[b], torch.logsumexp(s, dim=-1).numpy(), rtol=0, atol=1e-12)
        # numpy, naive exponentials (scores are O(5), no overflow)
        sn = (_decode_bf16(qb)[b, 0] @ _decode_bf16(kvb)[b, :n].T) * inputs.SCALE
        e = np.exp(sn)
        refn = (e / e.sum(-1, keepdims=True)) @ _decode_bf16(kvb)[b, :n, :inputs.D_V]
        np.testing.assert_allclose(out[b], refn, rtol=0, atol=1e-13)


def test_threads_do_not_change_result(oracle):
    qb, kvb, lens = _small(4, 64, 16, 64, seed=40)
    o1, l1 = oracle.decode(qb, kvb, lens, 0.1, 48, nthreads=1)
    o2, l2 = oracle.decode(qb, kvb, lens, 0.1, 48, nthreads=4)
    np.testing.assert_array_equal(o1, o2)
    np.testing.assert_array_equal(l1, l2)
    assert oracle.threads() >= 1


# ---- 8. what parity can be reached: emulate the kernel's number formats on the host ---------

def _kernel_number_model(q, kv, n, split_p):
    """fp32 scores from exact bf16 products, P cast to bf16 (one or two terms), fp32 accumulate."""
    qf = q.float(); kf = kv[:n].float()
    s = (qf.double() @ kf.double().T).float() * np.float32(inputs.SCALE)
    m = s.max(dim=-1, keepdim=True).values
    p = torch.exp(s - m)
    l = p.sum(-1, keepdim=True)
    p_hi = p.to(torch.bfloat16).float()
    acc = p_hi.double() @ kf[:, :inputs.D_V].double()
    if split_p:
        p_lo = (p - p_hi).to(torch.bfloat16).float()
        acc = acc + p_lo.double() @ kf[:, :inputs.D_V].double()
    return (acc / l.double()).numpy(), (m.double() + torch.log(l.double())).squeeze(-1).numpy()


def test_error_model_of_bf16_probabilities(oracle):
    """A single bf16 rounding of P misses the 1e-4 RMSE bound at short KV; a two-term
    (hi + lo) bf16 split of P is far inside it.  This fixes the kernel's P format."""
    q, kv, lens = inputs.make_config(1)
    ref_o, ref_l = oracle.decode(inputs.bf16_bits(q), inputs.bf16_bits(kv), lens.numpy(), inputs.SCALE, inputs.D_V)
    o1, l1 = _kernel_number_model(q[0, 0], kv[0], 512, split_p=False)
    o2, l2 = _kernel_number_model(q[0, 0], kv[0], 512, split_p=True)
    rmse1 = math.sqrt(((o1 - ref_o[0]) ** 2).mean())
    rmse2 = math.sqrt(((o2 - ref_o[0]) ** 2).mean())
    assert rmse1 > 1e-4          # single rounding: not good enough
    assert rmse2 < 2e-6          # hi + lo: two orders inside the bound
    assert np.abs(o2 - ref_o[0]).max() < 2e-5
    assert np.abs(l2 - ref_l[0]).max() < 1e-5


# ---- 9. the general entry: fp16 bit patterns and more than one query token --------------------

def test_fp16_decode_of_every_finite_bit_pattern(oracle):
    """d_qk = d_v = 1, one token, q = 1: out is the decoded KV element itself.  Every finite fp16
    bit pattern (normals, subnormals, both zeros) must decode to numpy's float16 value."""
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    vals = bits.view(np.float16).astype(np.float64)
    keep = np.isfinite(vals)
    bits, vals = bits[keep], vals[keep]
    n = bits.size
    q = np.full((n, 1, 1, 1), np.float16(1.0).view(np.uint16), dtype=np.uint16)
    kv = bits.reshape(n, 1, 1)
    out, lse = oracle.decode_general(q, kv, np.ones(n, dtype=np.int32), 0.5, 1, dtype=oracle.F16)
    np.testing.assert_array_equal(out.reshape(n), vals)          # exact, including signed zeros' value
    np.testing.assert_allclose(lse.reshape(n), 0.5 * vals, rtol=0, atol=0)


def test_general_with_bf16_and_one_query_token_is_the_plain_oracle(oracle):
    qb, kvb, lens = _small(3, 40, 4, 16, seed=51, seqlens=[40, 7, 0])
    o1, l1 = oracle.decode(qb, kvb, lens, 0.3, 12)
    o2, l2 = oracle.decode_general(qb, kvb, lens, 0.3, 12, dtype=oracle.BF16)
    np.testing.assert_array_equal(o1, o2[:, 0])
    np.testing.assert_array_equal(l1, l2[:, 0])


def test_fp16_against_numpy_float64(oracle):
    q, kv, lens = inputs.make_inputs(2, 300, [300, 77], seed=52, dtype=torch.float16)
    qb, kvb = inputs.bits16(q), inputs.bits16(kv)
    out, lse = oracle.decode_general(qb, kvb, lens.numpy(), inputs.SCALE, inputs.D_V, dtype=oracle.F16)
    for b in range(2):
        n = int(lens[b])
        qd = qb[b, 0].view(np.float16).astype(np.float64)          # numpy's own fp16 decode
        kd = kvb[b, :n].view(np.float16).astype(np.float64)
        s = (qd @ kd.T) * inputs.SCALE
        e = np.exp(s)
        np.testing.assert_allclose(out[b, 0], (e / e.sum(-1, keepdims=True)) @ kd[:, :inputs.D_V], rtol=0, atol=1e-13)
        np.testing.assert_allclose(lse[b, 0], np.log(e.sum(-1)), rtol=0, atol=1e-12)
    # the same bits read as bf16 give a different answer: the type argument is honoured
    out_b, _ = oracle.decode_general(qb, kvb, lens.numpy(), inputs.SCALE, inputs.D_V, dtype=oracle.BF16)
    assert np.abs(out_b - out).max() > 1e-3


def test_two_query_tokens_are_causal_among_themselves(oracle):
    """Query token j of q_len sees KV rows [0, N - (q_len - 1 - j)).  Checked against a dense
    float64 softmax with the mask written out as a matrix, for q_len 2 and 3."""
    for q_len in (2, 3):
        lens = [50, 3, q_len, 1]
        q, kv, l = inputs.make_inputs(4, 50, lens, seed=53 + q_len, heads=5, d_qk=24, q_len=q_len)
        qb, kvb = inputs.bf16_bits(q), inputs.bf16_bits(kv)
        out, lse = oracle.decode_general(qb, kvb, l.numpy(), 0.21, 20)
        for b in range(4):
            n = lens[b]
            kd = _decode_bf16(kvb)[b, :n]
            for j in range(q_len):
                vis = n - (q_len - 1 - j)
                mask = np.arange(n) < vis                         # [n]
                s = (_decode_bf16(qb)[b, j] @ kd.T) * 0.21        # [heads, n]
                if vis <= 0:
                    assert (out[b, j] == 0).all() and np.isneginf(lse[b, j]).all()
                    continue
                e = np.where(mask[None, :], np.exp(s), 0.0)
                np.testing.assert_allclose(out[b, j], (e / e.sum(-1, keepdims=True)) @ kd[:, :20], rtol=0, atol=1e-13)
                np.testing.assert_allclose(lse[b, j], np.log(e.sum(-1)), rtol=0, atol=1e-12)
        # the last query token is the plain one-token oracle on that query slice
        o1, l1 = oracle.decode(np.ascontiguousarray(qb[:, q_len - 1:q_len]), kvb, l.numpy(), 0.21, 20)
        np.testing.assert_array_equal(o1, out[:, q_len - 1])
        np.testing.assert_array_equal(l1, lse[:, q_len - 1])


def test_error_model_of_fp16_probabilities(oracle):
    """fp16 inputs: one fp16 rounding of P (11 significant bits) is inside the 1e-4 RMSE bound
    even at the shortest KV length, so the fp16 kernel needs no second term."""
    q, kv, lens = inputs.make_config(1, dtype=torch.float16)
    ref_o, ref_l = oracle.decode_general(inputs.bits16(q), inputs.bits16(kv), lens.numpy(), inputs.SCALE,
                                         inputs.D_V, dtype=oracle.F16)
    qf = q[0, 0].float(); kf = kv[0, :512].float()
    s = (qf.double() @ kf.double().T).float() * np.float32(inputs.SCALE)
    m = s.max(dim=-1, keepdim=True).values
    p = torch.exp(s - m)
    l = p.sum(-1, keepdim=True)
    acc = p.to(torch.float16).double() @ kf[:, :inputs.D_V].double()
    o = (acc / l.double()).numpy()
    rmse = math.sqrt(((o - ref_o[0, 0]) ** 2).mean())
    assert rmse < 4e-5
    assert np.abs(o - ref_o[0, 0]).max() < 2e-4
