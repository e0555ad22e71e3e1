"""Seeded synthetic inputs shaped like the paper's workloads (many-shot prompts, long generation).

This module only draws random tensors and lays out shot boundaries.  It holds none of the method's
arithmetic and is used by the tests and the benchmark to feed identical bits to the GPU library and to
the CPU oracle.  It imports neither of them.

The inputs stand in for the paper's evaluation prompts (50-shot arithmetic prompts of more than 4K
tokens, 4096/8192-token inputs followed by ~4K generated tokens): only shapes, shot-length mixes and
value distributions are reproduced, never dataset content.
"""
from __future__ import annotations

import dataclasses
import math

import numpy as np
import torch

BASE_SEED = 250201941


@dataclasses.dataclass(frozen=True)
class PrefillShape:
    name: str
    n_problems: int          # independent (batch, layer) problems
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    window: int
    n_tokens: int
    n_shots: int
    dtype: torch.dtype
    budget_tokens: int
    len_lo: int = 120        # uniform shot lengths [len_lo, len_hi]
    len_hi: int = 250
    lognormal_median: int = 0  # > 0: lognormal lengths instead, clipped to [32, 2000]
    tail_tokens: int = 0     # > 0: rescale lengths so the question tail has exactly this many tokens
    skew_fraction: float = 0.0  # fraction of shots whose keys lean toward the mean window query
    skew_beta: float = 0.0

    @property
    def sm_scale(self) -> float:
        return 1.0 / math.sqrt(self.head_dim)


# The five workload shapes.  "tiny" is CPU-checkable end to end; "layer8k" is one Llama-3-8B-shaped
# layer; "model32k" is the 32-layer x batch-4 pass at 32K tokens (128 independent problems);
# "skew128k" is the long-context case with peaked per-shot scores.
TINY = PrefillShape("tiny", 1, 4, 4, 64, 16, 512, 8, torch.float32, 256, len_lo=40, len_hi=60)
LAYER8K = PrefillShape("layer8k", 1, 32, 8, 128, 32, 8192, 40, torch.bfloat16, (8192 * 40) // 100)
MODEL32K = PrefillShape("model32k", 128, 32, 8, 128, 32, 32768, 160, torch.bfloat16,
                        (32768 * 10) // 100, tail_tokens=512)
SKEW128K = PrefillShape("skew128k", 32, 32, 8, 128, 32, 131072, 400, torch.bfloat16, 2048,
                        lognormal_median=300, tail_tokens=256, skew_fraction=0.10, skew_beta=3.56)
# Sentence-sized semantic units (the document-QA setting of the paper treats each sentence as a unit):
# hundreds to more than a thousand 10-40 token spans per sequence.
SENTENCES16K = PrefillShape("sentences16k", 8, 32, 8, 128, 32, 16384, 600, torch.bfloat16,
                            (16384 * 30) // 100, len_lo=10, len_hi=40)
SENTENCES32K = PrefillShape("sentences32k", 32, 32, 8, 128, 32, 32768, 1240, torch.bfloat16,
                            (32768 * 30) // 100, len_lo=10, len_hi=40)
PREFILL_SHAPES = {s.name: s for s in (TINY, LAYER8K, MODEL32K, SKEW128K, SENTENCES16K, SENTENCES32K)}


@dataclasses.dataclass(frozen=True)
class DecodeShape:
    name: str
    n_seqs: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    prefill_count: int
    decode_budget: int
    n_steps: int
    dtype: torch.dtype

    @property
    def sm_scale(self) -> float:
        return 1.0 / math.sqrt(self.head_dim)


DECODE4K = DecodeShape("decode4k", 16, 32, 8, 128, 4096, 1024, 4096, torch.bfloat16)
DECODE_TINY = DecodeShape("decode_tiny", 1, 4, 4, 64, 48, 32, 320, torch.float32)
DECODE_SHAPES = {s.name: s for s in (DECODE4K, DECODE_TINY)}


def _seed(*ids: int) -> int:
    """Mix small integer ids into one 63-bit seed (splitmix64 finaliser on a running sum)."""
    x = BASE_SEED
    for i in ids:
        x = (x + 0x9E3779B97F4A7C15 * (int(i) + 1)) & 0xFFFFFFFFFFFFFFFF
        x ^= x >> 30
        x = (x * 0xBF58476D1CE4E5B9) & 0xFFFFFFFFFFFFFFFF
        x ^= x >> 27
        x = (x * 0x94D049BB133111EB) & 0xFFFFFFFFFFFFFFFF
        x ^= x >> 31
    return x & 0x7FFFFFFFFFFFFFFF


def shot_offsets(shape: PrefillShape, problem: int, seed: int = 0) -> np.ndarray:
    """Shot boundaries off[0..n] for one problem: shots are back to back starting at token 0, the
    remainder up to n_tokens is the question tail (which contains the observation window)."""
    rng = np.random.Generator(np.random.PCG64(_seed(seed, 1, problem)))
    n = shape.n_shots
    if shape.lognormal_median > 0:
        lens = np.rint(shape.lognormal_median * np.exp(0.5 * rng.standard_normal(n)))
        lens = np.clip(lens, 32, 2000).astype(np.int64)
    else:
        lens = rng.integers(shape.len_lo, shape.len_hi + 1, size=n).astype(np.int64)
    min_tail = shape.tail_tokens if shape.tail_tokens > 0 else 2 * shape.window
    room = shape.n_tokens - min_tail
    if shape.tail_tokens > 0 or lens.sum() > room:
        # proportional rescale, then hand the rounding remainder out one token at a time
        scaled = np.maximum(1, np.floor(lens * (room / lens.sum()))).astype(np.int64)
        if shape.tail_tokens > 0:
            short = room - int(scaled.sum())
            scaled[: max(short, 0)] += 1
        lens = scaled
    off = np.zeros(n + 1, dtype=np.int32)
    off[1:] = np.cumsum(lens)
    assert off[-1] <= shape.n_tokens - shape.window
    return off


def _randn(shape, dtype, device, seed):
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return torch.randn(shape, generator=g, device=device, dtype=torch.float32).to(dtype)


def prefill_problem(shape: PrefillShape, problem: int, device="cpu", seed: int = 0):
    """Q_obs [H, W, D], K and V [H_kv, N, D] for one problem, values ~ N(0, 1) rounded to shape.dtype.

    With skew_fraction > 0 a seeded subset of shots gets K rows shifted by skew_beta times the unit mean
    of its KV head's window queries (in fp32, before rounding), which makes those shots' scores peak.
    Returns (q_obs, k, v, offsets int32 numpy).
    """
    H, Hkv, D, W, N = shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.window, shape.n_tokens
    off = shot_offsets(shape, problem, seed)
    q = _randn((H, W, D), shape.dtype, device, _seed(seed, 2, problem))
    v = _randn((Hkv, N, D), shape.dtype, device, _seed(seed, 4, problem))
    if shape.skew_fraction <= 0.0:
        k = _randn((Hkv, N, D), shape.dtype, device, _seed(seed, 3, problem))
    else:
        k32 = _randn((Hkv, N, D), torch.float32, device, _seed(seed, 3, problem))
        G = H // Hkv
        u = q.to(torch.float32).reshape(Hkv, G * W, D).mean(dim=1)
        u = u / u.norm(dim=1, keepdim=True)
        rng = np.random.Generator(np.random.PCG64(_seed(seed, 5, problem)))
        n_skew = max(1, int(round(shape.skew_fraction * shape.n_shots)))
        for i in sorted(rng.choice(shape.n_shots, size=n_skew, replace=False).tolist()):
            k32[:, int(off[i]): int(off[i + 1]), :] += shape.skew_beta * u[:, None, :]
        k = k32.to(shape.dtype)
    return q, k, v, off


def prefill_all_queries(shape: PrefillShape, problem: int, q_obs, device="cpu", seed: int = 0):
    """Query rows of every prompt position [H, N, D] for one problem, for the entry point that computes the
    prompt's whole attention pass: N(0, 1) rows whose last W are the window queries q_obs of
    prefill_problem, so that both entry points see the same observation window."""
    H, D, W, N = shape.n_q_heads, shape.head_dim, shape.window, shape.n_tokens
    q = _randn((H, N, D), shape.dtype, device, _seed(seed, 6, problem))
    q[:, N - W:] = q_obs
    return q


def prefill_batch(shape: PrefillShape, device="cpu", seed: int = 0, n_problems: int | None = None):
    """All problems of a shape stacked: q_obs [P, H, W, D], k/v [P, H_kv, N, D], offsets [P, n+1] int32,
    budgets [P] int32 (every problem gets shape.budget_tokens)."""
    P = shape.n_problems if n_problems is None else n_problems
    H, Hkv, D, W, N = shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.window, shape.n_tokens
    q = torch.empty((P, H, W, D), dtype=shape.dtype, device=device)
    k = torch.empty((P, Hkv, N, D), dtype=shape.dtype, device=device)
    v = torch.empty((P, Hkv, N, D), dtype=shape.dtype, device=device)
    offs = np.zeros((P, shape.n_shots + 1), dtype=np.int32)
    for p in range(P):
        q[p], k[p], v[p], offs[p] = prefill_problem(shape, p, device, seed)
    budgets = np.full((P,), shape.budget_tokens, dtype=np.int32)
    return q, k, v, torch.from_numpy(offs).to(device), torch.from_numpy(budgets).to(device)


def decode_state(shape: DecodeShape, device="cpu", seed: int = 0, n_slots: int | None = None,
                 resident: int = 0):
    """Decode state for every sequence: a random-normal compressed prefill cache with prefill_count live
    rows and a slot pool of decode_budget + 1 slots.  `resident` generated tokens (indices 0..resident-1,
    random-normal K/V) already sit in the first slots, as if that many steps had run without eviction."""
    S, Hkv, D = shape.n_seqs, shape.n_kv_heads, shape.head_dim
    n_slots = shape.decode_budget + 1 if n_slots is None else n_slots
    assert 0 <= resident <= min(n_slots, shape.decode_budget)
    cap = shape.prefill_count
    kp = _randn((S, Hkv, cap, D), shape.dtype, device, _seed(seed, 10))
    vp = _randn((S, Hkv, cap, D), shape.dtype, device, _seed(seed, 11))
    k_dec = torch.zeros((S, Hkv, n_slots, D), dtype=shape.dtype, device=device)
    v_dec = torch.zeros((S, Hkv, n_slots, D), dtype=shape.dtype, device=device)
    slot_pos = torch.full((S, n_slots), -1, dtype=torch.int32, device=device)
    if resident > 0:
        k_dec[:, :, :resident] = _randn((S, Hkv, resident, D), shape.dtype, device, _seed(seed, 12))
        v_dec[:, :, :resident] = _randn((S, Hkv, resident, D), shape.dtype, device, _seed(seed, 13))
        slot_pos[:, :resident] = torch.arange(resident, dtype=torch.int32, device=device)
    return {
        "k_prefill": kp, "v_prefill": vp,
        "prefill_count": torch.full((S,), cap, dtype=torch.int32, device=device),
        "k_dec": k_dec, "v_dec": v_dec, "slot_pos": slot_pos,
        "n_slots": n_slots, "cap": cap, "decode_budget": shape.decode_budget,
    }


def decode_inputs(shape: DecodeShape, step: int, device="cpu", seed: int = 0):
    """Fresh N(0,1) q_new [S, H, D], k_new and v_new [S, H_kv, D] for one decoding step."""
    S, H, Hkv, D = shape.n_seqs, shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    q = _randn((S, H, D), shape.dtype, device, _seed(seed, 20, step))
    k = _randn((S, Hkv, D), shape.dtype, device, _seed(seed, 21, step))
    v = _randn((S, Hkv, D), shape.dtype, device, _seed(seed, 22, step))
    return q, k, v
