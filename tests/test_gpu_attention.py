"""GPU parity of the entry point that fuses Eq. 3's scoring into the prompt's causal attention pass:
attention output against the oracle's textbook attention, scores / selection / compacted cache against the
oracle's prefill compression, and agreement with the stand-alone entry point."""
import numpy as np
import pytest
import torch

from helpers import check_prefill_problem, to_np
from oracle import shotkv_oracle as orc
from paper_2502_01941_amd import workloads as wl

pytestmark = pytest.mark.gpu

OUT_TOL = 1e-3        # |dO| <= OUT_TOL * max|O| per query row (weights reach the matrix cores with 11 significant bits)


@pytest.fixture(scope="module")
def kv():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2502_01941_amd import shotkv
    shotkv.load_library()
    return shotkv


def _problem_batch(shape, seed):
    q_obs, k, v, off, bud = wl.prefill_batch(shape, "cuda", seed)
    q = torch.stack([wl.prefill_all_queries(shape, p, q_obs[p], "cuda", seed) for p in range(shape.n_problems)])
    return q, q_obs, k, v, off, bud


def _check_rows(attn, q, k, v, rows, scale):
    """Output rows of one problem against the oracle: a row's weights are the oracle's window weights of
    the prompt cut off after that row (window_attention is pinned to equal causal_attention's last rows)."""
    qh, kh, vh = to_np(q), to_np(k), to_np(v)
    G = qh.shape[0] // kh.shape[0]
    for i in rows:
        p = orc.window_attention(qh[:, i:i + 1], kh[:, : i + 1], scale)      # [H, 1, i+1]
        ref = np.stack([p[h, 0] @ vh[h // G, : i + 1].astype(np.float64) for h in range(qh.shape[0])])
        got = attn[:, i].cpu().numpy().astype(np.float64)
        bound = OUT_TOL * np.abs(ref).max(axis=1, keepdims=True)
        assert np.all(np.abs(got - ref) <= bound), (i, np.abs(got - ref).max(), bound.min())


@pytest.mark.parametrize("H,H_kv,W,N,n_shots,P", [
    (8, 2, 32, 700, 5, 2),       # several query tiles, a ragged last one
    (4, 4, 16, 333, 3, 1),       # G = 1, window of 16, one block that is not full
    (8, 2, 32, 1030, 7, 1),      # the window straddles two query tiles (1030 = 8 * 128 + 6)
    (12, 4, 20, 515, 4, 2),      # G = 3, window 20: 60 rows per KV head, not a multiple of 32
    (32, 8, 32, 2048, 12, 1),    # the benchmark's head layout
])
def test_attention_and_compression_match_the_oracle(kv, H, H_kv, W, N, n_shots, P):
    budget = N // 2
    shape = wl.PrefillShape("attn", P, H, H_kv, 128, W, N, n_shots, torch.bfloat16, budget,
                            len_lo=max(8, N // (2 * n_shots)), len_hi=max(9, N // (n_shots + 1)))
    q, q_obs, k, v, off, bud = _problem_batch(shape, 21)
    attn, res = kv.prefill_attention_compress(q, k, v, off, bud, budget, W, shape.sm_scale)
    torch.cuda.synchronize()
    assert torch.isfinite(attn).all()
    for p in range(P):
        if N <= 1100:      # the whole output against the textbook definition
            ref = orc.causal_attention(to_np(q[p]), to_np(k[p]), to_np(v[p]), shape.sm_scale)
            got = attn[p].cpu().numpy().astype(np.float64)
            bound = OUT_TOL * np.abs(ref).max(axis=2, keepdims=True)
            assert np.all(np.abs(got - ref) <= bound), np.abs(got - ref).max()
        else:
            _check_rows(attn[p], q[p], k[p], v[p], [0, 1, 31, 32, 127, 128, 1000, N - W - 1, N - W, N - 1], shape.sm_scale)
        report = []
        check_prefill_problem(res, p, q_obs[p], k[p], v[p], off[p].cpu().numpy(), budget, budget, shape.sm_scale,
                              report=report)
        assert not report, report
    # and against the stand-alone entry point: same scores to rounding, same selection
    res2 = kv.prefill_compress(q_obs, k, v, off, bud, budget, shape.sm_scale)
    torch.cuda.synchronize()
    np.testing.assert_allclose(res.shot_scores.cpu().numpy(), res2.shot_scores.cpu().numpy(), rtol=2e-5)
    assert torch.equal(res.shot_selected, res2.shot_selected) and torch.equal(res.kept_count, res2.kept_count)


@pytest.mark.parametrize("factors", [(1e-30, 1.0), (3e4, 1e30), (2.0 ** -120, 2.0 ** 100), (0.0, 1.0)])
def test_value_magnitudes(kv, factors):
    """The weighted-value product runs in fp16 behind an exact per-plane power-of-two scale: value planes
    of very different magnitudes (one factor per KV head, an all-zero plane among them) keep the same
    relative accuracy."""
    H, H_kv, W, N, n_shots, budget = 4, 2, 16, 900, 5, 450
    shape = wl.PrefillShape("attn", 1, H, H_kv, 128, W, N, n_shots, torch.bfloat16, budget, len_lo=90, len_hi=150)
    q, q_obs, k, v, off, bud = _problem_batch(shape, 33)
    v = (v.float() * torch.tensor(factors, device="cuda").view(1, H_kv, 1, 1)).to(torch.bfloat16)
    attn, res = kv.prefill_attention_compress(q, k, v, off, bud, budget, W, shape.sm_scale)
    torch.cuda.synchronize()
    assert torch.isfinite(attn).all()
    ref = orc.causal_attention(to_np(q[0]), to_np(k[0]), to_np(v[0]), shape.sm_scale)
    got = attn[0].cpu().numpy().astype(np.float64)
    bound = OUT_TOL * np.abs(ref).max(axis=2, keepdims=True)
    assert np.all(np.abs(got - ref) <= bound), np.abs(got - ref).max()
    check_prefill_problem(res, 0, q_obs[0], k[0], v[0], off[0].cpu().numpy(), budget, budget, shape.sm_scale)


def test_flat_and_peaked_rows(kv):
    """Rows whose weights are all equal (zero queries: the output is the running mean of V, thousands of
    weights of 2^-11 of the total each) next to rows with one dominating key."""
    H, H_kv, W, N, n_shots, budget = 4, 2, 16, 3000, 6, 1500
    shape = wl.PrefillShape("attn", 1, H, H_kv, 128, W, N, n_shots, torch.bfloat16, budget, len_lo=300, len_hi=450)
    q, q_obs, k, v, off, bud = _problem_batch(shape, 34)
    q[0, 0] = 0                                   # head 0: uniform attention at every position
    q[0, 1] = (k[0, 0] * 4).to(q.dtype)           # head 1: every position attends to itself almost exclusively
    q_obs = q[:, :, N - W:].contiguous()
    attn, res = kv.prefill_attention_compress(q, k, v, off, bud, budget, W, shape.sm_scale)
    torch.cuda.synchronize()
    vh = to_np(v[0]).astype(np.float64)
    mean = np.cumsum(vh[0], axis=0) / np.arange(1, N + 1)[:, None]
    got = attn[0].cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got[0] - mean) <= OUT_TOL * np.abs(mean).max(axis=1, keepdims=True))
    _check_rows(attn[0], q[0], k[0], v[0], [0, 5, 100, 1023, 2047, N - 1], shape.sm_scale)
    check_prefill_problem(res, 0, q_obs[0], k[0], v[0], off[0].cpu().numpy(), budget, budget, shape.sm_scale)


def test_layer8k_fused(kv):
    """One Llama-3-8B-shaped layer at 8192 tokens: sampled output rows, every score, the selection and the
    compacted cache."""
    shape = wl.LAYER8K
    q, q_obs, k, v, off, bud = _problem_batch(shape, 0)
    N, W = shape.n_tokens, shape.window
    attn, res = kv.prefill_attention_compress(q, k, v, off, bud, shape.budget_tokens, W, shape.sm_scale)
    torch.cuda.synchronize()
    assert torch.isfinite(attn).all()
    _check_rows(attn[0], q[0], k[0], v[0], [0, 5, 127, 128, 2047, 4096, 6001, N - W - 1, N - W, N - 17, N - 1],
                shape.sm_scale)
    report = []
    check_prefill_problem(res, 0, q_obs[0], k[0], v[0], off[0].cpu().numpy(), shape.budget_tokens,
                          shape.budget_tokens, shape.sm_scale, report=report)
    assert not report, report


def test_attn32k_fused(kv):
    """The 32768-token problem bench.py times (one problem of the 32K workload's shape): sampled output rows
    across the whole triangle, every score, the selection and the compacted cache against the oracle, and
    the scores against the stand-alone entry point."""
    import dataclasses
    shape = dataclasses.replace(wl.PREFILL_SHAPES["model32k"], n_problems=1)
    q, q_obs, k, v, off, bud = _problem_batch(shape, 0)
    N, W = shape.n_tokens, shape.window
    attn, res = kv.prefill_attention_compress(q, k, v, off, bud, shape.budget_tokens, W, shape.sm_scale)
    torch.cuda.synchronize()
    assert torch.isfinite(attn).all()
    _check_rows(attn[0], q[0], k[0], v[0], [0, 31, 4095, 16384, 16511, 30000, N - W - 1, N - W, N - 1], shape.sm_scale)
    report = []
    check_prefill_problem(res, 0, q_obs[0], k[0], v[0], off[0].cpu().numpy(), shape.budget_tokens,
                          shape.budget_tokens, shape.sm_scale, report=report)
    assert not report, report
    res2 = kv.prefill_compress(q_obs, k, v, off, bud, shape.budget_tokens, shape.sm_scale)
    torch.cuda.synchronize()
    np.testing.assert_allclose(res.shot_scores.cpu().numpy(), res2.shot_scores.cpu().numpy(), rtol=2e-5)
    assert torch.equal(res.shot_selected, res2.shot_selected) and torch.equal(res.kept_count, res2.kept_count)


def test_fused_per_kv_head(kv):
    """The per-KV-head variant through the fused entry point: the attention output is the same (it does not
    depend on the head mode), every KV head selects over its own query group exactly as the stand-alone
    entry point does, and the result matches the oracle's per-KV-head compression."""
    import types
    H, H_kv, W, N, n_shots, P = 8, 4, 16, 1100, 7, 2
    budget, G = N // 2, 2
    shape = wl.PrefillShape("attn", P, H, H_kv, 128, W, N, n_shots, torch.bfloat16, budget, len_lo=90, len_hi=140)
    q, q_obs, k, v, off, bud = _problem_batch(shape, 41)
    attn, res = kv.prefill_attention_compress(q, k, v, off, bud, budget, W, shape.sm_scale,
                                              head_mode=kv.HEADS_PER_KV_HEAD)
    attn_layer, _ = kv.prefill_attention_compress(q, k, v, off, bud, budget, W, shape.sm_scale)
    res2 = kv.prefill_compress(q_obs, k, v, off, bud, budget, shape.sm_scale, head_mode=kv.HEADS_PER_KV_HEAD)
    torch.cuda.synchronize()
    assert torch.equal(attn, attn_layer)
    assert res.kept_count.shape == (P, H_kv) and res.kept_positions.shape == (P, H_kv, budget)
    np.testing.assert_allclose(res.shot_scores.cpu().numpy(), res2.shot_scores.cpu().numpy(), rtol=2e-5)
    assert torch.equal(res.shot_selected, res2.shot_selected) and torch.equal(res.kept_count, res2.kept_count)
    view = types.SimpleNamespace(
        status=res.status.reshape(-1), kept_count=res.kept_count.reshape(-1),
        shot_scores=res.shot_scores.reshape(P * H_kv, n_shots), shot_selected=res.shot_selected.reshape(P * H_kv, n_shots),
        kept_positions=res.kept_positions.reshape(P * H_kv, budget),
        k_out=res.k_out.reshape(P * H_kv, 1, budget, 128), v_out=res.v_out.reshape(P * H_kv, 1, budget, 128))
    for p in range(P):
        refs = orc.prefill_compress_per_kv_head(to_np(q_obs[p]), to_np(k[p]), to_np(v[p]), off[p].cpu().numpy(),
                                                budget, shape.sm_scale, orc.SELECT_PREFIX)
        for g in range(H_kv):
            check_prefill_problem(view, p * H_kv + g, q_obs[p, g * G:(g + 1) * G], k[p, g:g + 1], v[p, g:g + 1],
                                  off[p].cpu().numpy(), budget, budget, shape.sm_scale, orc.SELECT_PREFIX,
                                  ref=refs[g])
    _check_rows(attn[0], q[0], k[0], v[0], [0, 63, 500, N - 1], shape.sm_scale)


def test_fused_entry_point_rejects_what_it_does_not_cover(kv):
    shape = wl.TINY            # fp32, head_dim 64
    q_obs, k, v, off, bud = wl.prefill_batch(shape, "cuda")
    q = torch.stack([wl.prefill_all_queries(shape, 0, q_obs[0], "cuda")])
    with pytest.raises(kv.ShotKVError):
        kv.prefill_attention_compress(q, k, v, off, bud, shape.budget_tokens, shape.window, shape.sm_scale)
