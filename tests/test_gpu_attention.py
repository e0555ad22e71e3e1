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

OUT_TOL = 1e-3        # |dO| <= OUT_TOL * max|O| per query row (weights reach the matrix cores as bf16 hi + lo)


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


def test_fused_entry_point_rejects_what_it_does_not_cover(kv):
    shape = wl.TINY            # fp32, head_dim 64
    q_obs, k, v, off, bud = wl.prefill_batch(shape, "cuda")
    q = torch.stack([wl.prefill_all_queries(shape, 0, q_obs[0], "cuda")])
    with pytest.raises(kv.ShotKVError):
        kv.prefill_attention_compress(q, k, v, off, bud, shape.budget_tokens, shape.window, shape.sm_scale)
