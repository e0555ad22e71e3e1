"""Shared glue for the GPU parity tests: moves one problem to the host and runs the oracle on it."""
import numpy as np
import torch

from oracle import shotkv_oracle as orc

SCORE_RTOL = 1e-3      # stated tolerance for scores (fp32 accumulation on the device)
MARGIN_EXACT = 1e-6    # selections must agree end to end when the decision margin is at least this


def to_np(t: torch.Tensor) -> np.ndarray:
    """Device tensor -> float32/int numpy on the host (bf16 widens exactly)."""
    t = t.detach().cpu()
    if t.dtype == torch.bfloat16:
        t = t.to(torch.float32)
    return t.numpy()


def oracle_prefill(q, k, v, off, budget, sm_scale, mode=orc.SELECT_PREFIX, scores_override=None):
    return orc.prefill_compress(to_np(q), to_np(k), to_np(v), np.asarray(off), int(budget), sm_scale,
                                mode, scores_override)


def bits(t) -> np.ndarray:
    """Raw bit patterns for bit-exact comparison."""
    if isinstance(t, np.ndarray):
        return t.view(np.int32) if t.dtype == np.float32 else t
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy()
    if t.dtype == torch.float32:
        return t.view(torch.int32).numpy()
    return t.numpy()


def check_selection_valid(sel, kept, pos, off, n_tokens, budget):
    """What must hold for any correct selection: whole shots, budget, ascending positions that are
    exactly the always-kept tokens plus the selected shots."""
    off = np.asarray(off, dtype=np.int64)
    lengths = np.diff(off)
    n_always = int(off[0]) + int(n_tokens - off[-1])
    assert kept == n_always + int((lengths * sel).sum())
    assert kept <= budget
    assert np.all(np.diff(pos) > 0)
    expect = [np.arange(0, off[0])]
    expect += [np.arange(off[i], off[i + 1]) for i in range(len(lengths)) if sel[i]]
    expect.append(np.arange(off[-1], n_tokens))
    np.testing.assert_array_equal(pos, np.concatenate(expect))


def replay_selection(gpu_scores, off, n_tokens, budget, mode):
    """The oracle's ranked walk run on the scores a device produced: (keep mask, kept positions).
    None when the tokens outside the shots alone exceed the budget."""
    off = np.asarray(off, dtype=np.int64)
    shot_budget = int(budget) - int(off[0]) - int(n_tokens - off[-1])
    if shot_budget < 0:
        return None
    keep = orc.select_shots(np.asarray(gpu_scores), np.diff(off), shot_budget, mode)
    return keep, orc.kept_positions_from_mask(keep, off, n_tokens)


def check_prefill_problem(res, p, q, k, v, off, budget, cap, sm_scale, mode=orc.SELECT_PREFIX,
                          report=None, ref=None):
    """Compare problem p of a device PrefillResult with the oracle, element by element.

    (i) scores within SCORE_RTOL; (ii) always: the device's selection, kept positions and compacted K/V
    are bit-exact what the oracle's ranked walk gives on the device's own scores; (iii) the same against
    the oracle end to end whenever the oracle's decision margin is at least MARGIN_EXACT (with exact
    arithmetic the result is unique; a closer call may legitimately flip in fp32 and is recorded in
    `report` as (problem, margin, agrees)).  `ref` passes in an oracle result computed elsewhere for the
    same inputs.
    """
    budget = min(int(budget), cap)
    if ref is None:
        ref = oracle_prefill(q, k, v, off, budget, sm_scale, mode)
    status = int(res.status[p].item())
    assert status == ref["status"], (p, status, ref["status"])
    kept = int(res.kept_count[p].item())
    if ref["status"] == orc.STATUS_BAD_OFFSETS:
        assert kept == 0
        return ref
    gpu_scores = res.shot_scores[p].cpu().numpy()
    np.testing.assert_allclose(gpu_scores, ref["scores"], rtol=SCORE_RTOL, atol=0)
    sel = res.shot_selected[p].cpu().numpy()
    if ref["status"] != orc.STATUS_OK:
        assert kept == 0 and not sel.any()
        return ref
    pos = res.kept_positions[p, :kept].cpu().numpy()
    check_selection_valid(sel, kept, pos, off, k.shape[1], budget)
    # (ii) the selection rule itself, independent of score rounding
    keep_replay, pos_replay = replay_selection(gpu_scores, off, k.shape[1], budget, mode)
    assert sel.tolist() == keep_replay.tolist(), f"problem {p}: selection differs from the walk on its own scores"
    np.testing.assert_array_equal(pos, pos_replay)
    k_host, v_host = to_np(k), to_np(v)
    np.testing.assert_array_equal(to_np(res.k_out[p, :, :kept]), k_host[:, pos_replay])
    np.testing.assert_array_equal(to_np(res.v_out[p, :, :kept]), v_host[:, pos_replay])
    agrees = sel.tolist() == ref["selected"].tolist()
    if ref["margin"] >= MARGIN_EXACT:
        assert agrees, f"problem {p}: margin {ref['margin']}"
        assert kept == ref["kept_count"]
        np.testing.assert_array_equal(pos, ref["kept_positions"])
        np.testing.assert_array_equal(to_np(res.k_out[p, :, :kept]), ref["k_out"].astype(np.float32))
        np.testing.assert_array_equal(to_np(res.v_out[p, :, :kept]), ref["v_out"].astype(np.float32))
    elif report is not None:
        report.append((p, ref["margin"], agrees))
    return ref
