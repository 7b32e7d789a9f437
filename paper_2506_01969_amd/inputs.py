"""Seeded synthetic inputs for MLA decode (shared by the tests, the benchmark and the oracle checks).

This module holds no attention arithmetic: it only draws numbers, rounds them to
bf16 and lays them out.  The workload shapes follow the paper's experimental
setup (Section 4.1: one query token, 16 heads, head dimension 576, batch 16 or
32, KV length 512 ... 64K); the paper used shapes only, no dataset, so seeded
N(0,1) values stand in for real activations.
"""
from __future__ import annotations

import math

import numpy as np
import torch

NUM_HEADS = 16
D_QK = 576          # 512 latent + 64 rope
D_V = 512           # V is the first 512 columns of the latent row
SCALE = 1.0 / math.sqrt(192.0)
BASE_SEED = 20250601

# id -> (batch, fixed KV length or None, (lo, hi) inclusive range for ragged lengths or None)
CONFIGS = {
    1: dict(batch=1, seqlen=512, ragged=None),
    2: dict(batch=16, seqlen=4096, ragged=None),
    3: dict(batch=16, seqlen=16384, ragged=None),
    4: dict(batch=16, seqlen=65536, ragged=None),
    5: dict(batch=32, seqlen=65536, ragged=(1024, 65536)),
}


def bf16_bits(t: torch.Tensor) -> np.ndarray:
    """bf16 CPU tensor -> numpy uint16 array of its bit patterns (no copy of values)."""
    if t.dtype != torch.bfloat16 or t.device.type != "cpu":
        raise TypeError("expected a CPU bf16 tensor")
    return t.contiguous().view(torch.int16).numpy().view(np.uint16)


def bits16(t: torch.Tensor) -> np.ndarray:
    """bf16 or fp16 CPU tensor -> numpy uint16 array of its bit patterns."""
    if t.dtype not in (torch.bfloat16, torch.float16) or t.device.type != "cpu":
        raise TypeError("expected a CPU bf16 or fp16 tensor")
    return t.contiguous().view(torch.int16).numpy().view(np.uint16)


def make_inputs(batch, max_seqlen, seqlens=None, seed=BASE_SEED, heads=NUM_HEADS, d_qk=D_QK,
                poison_tail=False, dtype=torch.bfloat16, q_len=1):
    """Draw q [batch, q_len, heads, d_qk] and kv [batch, max_seqlen, d_qk] ~ N(0,1), rounded to
    ``dtype`` (bf16 by default, or fp16).

    seqlens: None (every sequence is max_seqlen long) or an int sequence of length batch.
    Rows at or beyond a sequence's length are zero, or NaN when poison_tail is set
    (a correct kernel never lets them reach the result).
    Returns CPU tensors (q, kv in ``dtype``, seqlens int32).
    """
    g = torch.Generator().manual_seed(int(seed))
    q = torch.randn((batch, q_len, heads, d_qk), generator=g, dtype=torch.float32).to(dtype)
    if seqlens is None:
        lens = torch.full((batch,), max_seqlen, dtype=torch.int32)
    else:
        lens = torch.as_tensor(list(seqlens), dtype=torch.int32)
        if lens.shape != (batch,) or int(lens.min()) < 0 or int(lens.max()) > max_seqlen:
            raise ValueError("seqlens must have one entry in [0, max_seqlen] per sequence")
    kv = torch.empty((batch, max_seqlen, d_qk), dtype=dtype)
    for b in range(batch):
        n = int(lens[b])
        if n > 0:
            kv[b, :n] = torch.randn((n, d_qk), generator=g, dtype=torch.float32).to(dtype)
        if n < max_seqlen:
            kv[b, n:] = float("nan") if poison_tail else 0.0
    return q, kv, lens


def make_config(cfg_id, poison_tail=False, dtype=torch.bfloat16, q_len=1):
    """Inputs of one of the five benchmark configurations (seed = BASE_SEED + cfg_id)."""
    c = CONFIGS[cfg_id]
    seed = BASE_SEED + cfg_id
    seqlens = None
    if c["ragged"] is not None:
        lo, hi = c["ragged"]
        gl = torch.Generator().manual_seed(seed + 1000)
        seqlens = torch.randint(lo, hi + 1, (c["batch"],), generator=gl).tolist()
    return make_inputs(c["batch"], c["seqlen"], seqlens, seed=seed, poison_tail=poison_tail, dtype=dtype, q_len=q_len)


def algorithmic_bytes(seqlens, heads=NUM_HEADS, d_qk=D_QK, d_v=D_V) -> int:
    """Bytes the method must move per call: each KV row read once for all heads, plus
    q (bf16), out (fp32), lse (fp32) and the length of every sequence."""
    total_tokens = int(sum(int(n) for n in seqlens))
    per_seq = heads * d_qk * 2 + heads * d_v * 4 + heads * 4 + 4
    return total_tokens * d_qk * 2 + per_seq * len(seqlens)


def algorithmic_flops(seqlens, heads=NUM_HEADS, d_qk=D_QK, d_v=D_V) -> int:
    """2*(d_qk + d_v) flops per head per KV token (the two contractions)."""
    return 2 * (d_qk + d_v) * heads * int(sum(int(n) for n in seqlens))
