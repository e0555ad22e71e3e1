"""Seeded random shapes through the whole path, against the oracle: head counts, group sizes 1..8, head
dimensions, dtypes, window lengths, shot layouts, budgets, both selection modes and both head modes for
the prefill half; ragged live-row counts with NaN / Inf in the dead rows for the decode half."""
import math
import types

import numpy as np
import pytest
import torch

from helpers import check_prefill_problem, to_np
from oracle import shotkv_oracle as orc
from paper_2502_01941_amd import workloads as wl
from test_gpu_decode import OracleSeq, _compare_step

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def kv():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2502_01941_amd import shotkv
    shotkv.load_library()
    return shotkv


def _draw(rng):
    while True:
        Hkv, G = int(rng.choice([1, 2, 4, 8])), int(rng.integers(1, 9))
        if Hkv * G <= 64:
            break
    D = int(rng.choice([64, 128]))
    dtype = torch.bfloat16 if rng.random() < 0.7 else torch.float32
    W = int(rng.integers(1, min(64, 256 // G) + 1))
    return Hkv, G, D, dtype, W


@pytest.mark.parametrize("seed", range(24))
def test_random_prefill(kv, seed):
    rng = np.random.default_rng(1000 + seed)
    Hkv, G, D, dtype, W = _draw(rng)
    H = Hkv * G
    N, P, n = int(rng.integers(W + 40, 1500)), int(rng.integers(1, 4)), int(rng.integers(0, 12))
    prefix, tail_min = int(rng.integers(0, 10)), int(rng.integers(0, W + 20))
    mode, head_mode = int(rng.integers(0, 2)), int(rng.integers(0, 2))
    g = torch.Generator(device="cuda").manual_seed(seed)
    q = torch.randn((P, H, W, D), generator=g, device="cuda").to(dtype)
    k = torch.randn((P, Hkv, N, D), generator=g, device="cuda").to(dtype)
    v = torch.randn((P, Hkv, N, D), generator=g, device="cuda").to(dtype)
    offs = np.zeros((P, n + 1), dtype=np.int32)
    for p in range(P):
        hi = max(prefix + n + 1, N - tail_min)
        cuts = np.sort(rng.choice(np.arange(prefix + 1, hi + 1), size=n, replace=False))
        offs[p] = np.concatenate([[prefix], cuts])
    off = torch.from_numpy(offs).cuda()
    budgets = rng.integers(N // 4, N + 1, size=P).astype(np.int32)
    scale = float(rng.choice([1.0 / math.sqrt(D), 0.3]))
    res = kv.prefill_compress(q, k, v, off, torch.from_numpy(budgets).cuda(), N, scale, select_mode=mode,
                              head_mode=head_mode)
    torch.cuda.synchronize()
    near = []
    for p in range(P):
        if head_mode == kv.HEADS_PER_LAYER:
            check_prefill_problem(res, p, q[p], k[p], v[p], offs[p], int(budgets[p]), N, scale, mode, report=near)
            continue
        view = types.SimpleNamespace(
            status=res.status.reshape(-1), kept_count=res.kept_count.reshape(-1),
            shot_scores=res.shot_scores.reshape(P * Hkv, n), shot_selected=res.shot_selected.reshape(P * Hkv, n),
            kept_positions=res.kept_positions.reshape(P * Hkv, N), k_out=res.k_out.reshape(P * Hkv, 1, N, D),
            v_out=res.v_out.reshape(P * Hkv, 1, N, D))
        refs = orc.prefill_compress_per_kv_head(to_np(q[p]), to_np(k[p]), to_np(v[p]), offs[p],
                                                int(budgets[p]), scale, mode)
        for gg in range(Hkv):
            check_prefill_problem(view, p * Hkv + gg, q[p, gg * G:(gg + 1) * G], k[p, gg:gg + 1], v[p, gg:gg + 1],
                                  offs[p], int(budgets[p]), N, scale, mode, report=near, ref=refs[gg])
    assert not near, near


@pytest.mark.parametrize("seed", range(16))
def test_random_decode(kv, seed):
    rng = np.random.default_rng(2000 + seed)
    Hkv, G, D, dtype, _ = _draw(rng)
    H = Hkv * G
    S, cap, budget = int(rng.integers(1, 4)), int(rng.integers(1, 700)), int(rng.integers(1, 9))
    shape = wl.DecodeShape("random", S, H, Hkv, D, cap, budget, 0, dtype)
    st = wl.decode_state(shape, "cuda", seed)
    st["prefill_count"] = torch.from_numpy(rng.integers(0, cap + 1, size=S).astype(np.int32)).cuda()
    seqs = []
    for s in range(S):
        c = int(st["prefill_count"][s].item())
        st["k_prefill"][s, :, c:] = float("nan")       # dead rows must never matter
        st["v_prefill"][s, :, c:] = float("inf")
        seq = OracleSeq(st, s)
        seq.kp, seq.vp = seq.kp[:, :c].copy(), seq.vp[:, :c].copy()
        seqs.append(seq)
    state = kv.DecodeState(st["k_prefill"], st["v_prefill"], st["prefill_count"], st["k_dec"], st["v_dec"],
                           st["slot_pos"], budget, H, shape.sm_scale)
    near = []
    for step in range(budget + 4):
        qn, kn, vn = wl.decode_inputs(shape, step, "cuda", seed)
        kv.decode_step(state, step, qn, kn, vn)
        torch.cuda.synchronize()
        assert torch.isfinite(state.out).all()
        for s, seq in enumerate(seqs):
            r = seq.step(budget, step, qn[s], kn[s], vn[s], shape.sm_scale)
            _compare_step(state, s, r, seq, near)
    assert not near, near
