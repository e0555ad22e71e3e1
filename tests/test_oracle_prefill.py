"""Pins for the prefill half of the CPU oracle (no GPU).

Each test checks the oracle against something other than itself: hand-derived fractions, closed forms
that follow from softmax rows summing to one, a library attention routine, or brute-force enumeration.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import shotkv_oracle as orc
from paper_2502_01941_amd import workloads as wl


def _read_golden(path):
    out = {}
    with open(path) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *vals = line.split()
            out[key] = [Fraction(v) for v in vals]
    return out


def _rand_problem(rng, H, Hkv, D, W, N):
    q = rng.standard_normal((H, W, D))
    k = rng.standard_normal((Hkv, N, D))
    v = rng.standard_normal((Hkv, N, D))
    return q, k, v


# ---- hand-derived worked example (Eq. 3) ---------------------------------------------------------

def test_hand_example_mass_and_scores(golden_dir):
    gold = _read_golden(os.path.join(golden_dir, "prefill_hand_example.txt"))
    ln2 = math.log(2.0)
    q = np.array([[[ln2], [ln2]], [[0.0], [0.0]]])            # [H=2, W=2, D=1]
    k = np.array([[[0.0], [1.0], [0.0], [1.0], [1.0], [0.0]]])  # [H_kv=1, N=6, D=1]
    p = orc.window_attention(q, k, 1.0)
    assert p[0, 0, 5] == 0.0 and p[1, 0, 5] == 0.0             # key 5 is after query j=0 (position 4)
    mass = orc.token_mass(p)
    np.testing.assert_allclose(mass, [float(f) for f in gold["mass"]], rtol=1e-14)
    scores = orc.shot_scores_from_mass(mass, [1, 3, 4])
    np.testing.assert_allclose(scores, [float(f) for f in gold["scores"]], rtol=1e-14)


def test_hand_example_end_to_end(golden_dir):
    """Same example through prefill_compress: budget 4 = 3 always-kept tokens + room for one token,
    so only shot 1 (length 1, the higher score) fits; PREFIX stops there."""
    ln2 = math.log(2.0)
    q = np.array([[[ln2], [ln2]], [[0.0], [0.0]]])
    k = np.array([[[0.0], [1.0], [0.0], [1.0], [1.0], [0.0]]])
    v = np.arange(6, dtype=np.float64).reshape(1, 6, 1) * 10
    r = orc.prefill_compress(q, k, v, [1, 3, 4], 4, 1.0)
    assert r["status"] == orc.STATUS_OK
    assert r["selected"].tolist() == [0, 1]
    assert r["kept_positions"].tolist() == [0, 3, 4, 5]
    assert r["v_out"][0, :, 0].tolist() == [0.0, 30.0, 40.0, 50.0]
    # budget 6 keeps both shots, budget 2 cannot even hold the always-kept tokens
    assert orc.prefill_compress(q, k, v, [1, 3, 4], 6, 1.0)["kept_positions"].tolist() == list(range(6))
    assert orc.prefill_compress(q, k, v, [1, 3, 4], 2, 1.0)["status"] == orc.STATUS_BUDGET_TOO_SMALL


# ---- softmax against a library attention routine -------------------------------------------------

@pytest.mark.parametrize("H,Hkv,D,W,N", [(4, 2, 8, 3, 17), (6, 2, 16, 5, 40), (2, 2, 4, 1, 9)])
def test_window_attention_matches_library_sdpa(H, Hkv, D, W, N):
    """With V = identity, scaled_dot_product_attention returns the weight matrix itself; grouped-query
    head mapping is the library's (enable_gqa)."""
    rng = np.random.default_rng(7)
    q, k, _ = _rand_problem(rng, H, Hkv, D, W, N)
    scale = 0.37
    p = orc.window_attention(q, k, scale)
    tq = torch.from_numpy(q)[None]                               # [1, H, W, D]
    tk = torch.from_numpy(k)[None]                               # [1, Hkv, N, D]
    eye = torch.eye(N, dtype=torch.float64).expand(1, Hkv, N, N)
    visible = torch.arange(N)[None, :] <= (N - W + torch.arange(W))[:, None]
    lib = torch.nn.functional.scaled_dot_product_attention(
        tq, tk, eye, attn_mask=visible, scale=scale, enable_gqa=True)[0].numpy()
    np.testing.assert_allclose(p, lib, rtol=1e-12, atol=1e-15)


def test_rows_sum_to_one_and_mask_is_exact_zero():
    rng = np.random.default_rng(1)
    q, k, _ = _rand_problem(rng, 4, 2, 8, 6, 50)
    p = orc.window_attention(q, k, 1.0 / math.sqrt(8))
    np.testing.assert_allclose(p.sum(axis=2), 1.0, rtol=0, atol=1e-12)
    for j in range(6):
        assert np.all(p[:, j, 50 - 6 + j + 1:] == 0.0)
        assert np.all(p[:, j, : 50 - 6 + j + 1] > 0.0)


# ---- closed forms ---------------------------------------------------------------------------------

def test_mass_conservation_closed_form():
    """sum_i k_i*Score_i + mass outside the shots = H*W, because each of the H*W rows sums to 1."""
    rng = np.random.default_rng(2)
    H, Hkv, D, W, N = 8, 2, 16, 4, 300
    q, k, v = _rand_problem(rng, H, Hkv, D, W, N)
    off = np.array([5, 40, 90, 91, 180, 250])
    r = orc.prefill_compress(q, k, v, off, 300, 0.25)
    lengths = np.diff(off)
    outside = r["mass"][:5].sum() + r["mass"][250:].sum()
    assert abs((lengths * r["scores"]).sum() + outside - H * W) < 1e-10


def test_uniform_keys_closed_form_and_tie_break():
    """All keys equal: every row is uniform over its visible keys, so every token outside the window
    has mass sum_rows 1/visible_r and all shots tie.  The tie must go to the lowest indices."""
    H, Hkv, D, W, N = 4, 2, 8, 3, 64
    rng = np.random.default_rng(3)
    q = rng.standard_normal((H, W, D))
    k = np.tile(rng.standard_normal((1, 1, D)), (Hkv, N, 1))
    v = rng.standard_normal((Hkv, N, D))
    off = np.array([0, 10, 20, 30, 40, 50])
    expect = H * sum(1.0 / (N - W + j + 1) for j in range(W))
    r = orc.prefill_compress(q, k, v, off, 14 + 25, 1.0)        # tail = 14 tokens, room for 2 shots
    np.testing.assert_allclose(r["scores"], expect, rtol=1e-12)
    # make the tie exact, then check the order of equal keys
    keep = orc.select_shots(np.full(5, expect), np.diff(off), 25)
    assert keep.tolist() == [1, 1, 0, 0, 0]
    assert orc.rank_shots([1.0, 2.0, 2.0, 1.0]) == [1, 2, 0, 3]


def test_one_hot_shot_closed_form():
    """One shot's keys aligned with every query and scaled up: it takes all the mass, H*W/k_i."""
    H, Hkv, D, W, N = 4, 2, 8, 2, 80
    u = np.ones(D) / math.sqrt(D)
    q = np.tile(u, (H, W, 1)) * 3.0
    k = np.zeros((Hkv, N, D))
    k[:, 20:30, :] = 40.0 * u
    v = np.zeros((Hkv, N, D))
    off = np.array([0, 20, 30, 60])
    r = orc.prefill_compress(q, k, v, off, 80, 1.0)
    np.testing.assert_allclose(r["scores"][1], H * W / 10.0, rtol=1e-12)
    assert r["scores"][0] < 1e-30 and r["scores"][2] < 1e-30


def test_length_normalisation():
    """Doubling a shot's span over keys of equal mass leaves its score unchanged (the 1/k_i factor)."""
    mass = np.array([0.5] * 12)
    s = orc.shot_scores_from_mass(mass, [0, 4, 12])
    np.testing.assert_allclose(s, [0.5, 0.5])
    s = orc.shot_scores_from_mass(np.arange(6, dtype=float), [1, 3, 6])
    np.testing.assert_allclose(s, [(1 + 2) / 2, (3 + 4 + 5) / 3])


def test_shot_permutation_property():
    """Reordering whole shots (K rows moved with them) permutes the scores; the window and tail are
    untouched so the causal mask is unaffected."""
    rng = np.random.default_rng(5)
    H, Hkv, D, W, N = 4, 4, 8, 4, 120
    q, k, v = _rand_problem(rng, H, Hkv, D, W, N)
    off = np.array([0, 20, 50, 65, 100])
    base = orc.prefill_compress(q, k, v, off, N, 0.3)["scores"]
    perm = [2, 0, 3, 1]
    spans = [(off[i], off[i + 1]) for i in range(4)]
    k2 = np.concatenate([k[:, a:b] for a, b in (spans[i] for i in perm)] + [k[:, 100:]], axis=1)
    lens = [spans[i][1] - spans[i][0] for i in perm]
    off2 = np.concatenate([[0], np.cumsum(lens)])
    got = orc.prefill_compress(q, k2, v, off2, N, 0.3)["scores"]
    np.testing.assert_allclose(got, base[perm], rtol=1e-12)


# ---- selection: brute force + invariants ---------------------------------------------------------

@pytest.mark.parametrize("mode", [orc.SELECT_PREFIX, orc.SELECT_FIRST_FIT])
def test_selection_equals_bruteforce_enumeration(mode):
    rng = np.random.default_rng(11)
    for trial in range(60):
        n = int(rng.integers(1, 11))
        lengths = rng.integers(1, 30, size=n)
        scores = rng.standard_normal(n)
        if trial % 3 == 0:                                     # force ties
            scores = np.round(scores)
        budget = int(rng.integers(0, lengths.sum() + 5))
        got = orc.select_shots(scores, lengths, budget, mode)
        want = orc.bruteforce_select(scores, lengths, budget, mode)
        assert got.tolist() == want.tolist(), (trial, scores, lengths, budget)


def test_tiny_workload_bruteforce_and_invariants():
    """The tiny workload end to end: 2^8 subsets, whole shots, budget, maximality."""
    shape = wl.TINY
    q, k, v, off = wl.prefill_problem(shape, 0, "cpu")
    r = orc.prefill_compress(q.numpy(), k.numpy(), v.numpy(), off, shape.budget_tokens, shape.sm_scale)
    assert r["status"] == orc.STATUS_OK
    lengths = np.diff(off)
    n_always = int(off[0]) + shape.n_tokens - int(off[-1])
    shot_budget = shape.budget_tokens - n_always
    want = orc.bruteforce_select(r["scores"], lengths, shot_budget)
    assert r["selected"].tolist() == want.tolist()
    assert r["kept_count"] <= shape.budget_tokens
    assert r["kept_count"] == n_always + int((lengths * r["selected"]).sum())
    pos = r["kept_positions"]
    assert np.all(np.diff(pos) > 0)
    kept = set(pos.tolist())
    for i in range(shape.n_shots):                             # whole shots only
        span = set(range(off[i], off[i + 1]))
        assert span <= kept if r["selected"][i] else not (span & kept)
    order = orc.rank_shots(r["scores"])
    n_kept = int(r["selected"].sum())
    assert all(r["selected"][i] for i in order[:n_kept])       # a prefix of the ranking
    if n_kept < shape.n_shots:                                 # maximal: the next one does not fit
        assert (lengths * r["selected"]).sum() + lengths[order[n_kept]] > shot_budget
    np.testing.assert_array_equal(r["k_out"], k.numpy()[:, pos])
    np.testing.assert_array_equal(r["v_out"], v.numpy()[:, pos])
    assert abs((lengths * r["scores"]).sum() + r["mass"][off[-1]:].sum() - 4 * 16) < 1e-9


def test_prefix_vs_first_fit_differ_when_a_long_shot_blocks():
    scores = [5.0, 4.0, 3.0]
    lengths = [10, 50, 10]
    assert orc.select_shots(scores, lengths, 25, orc.SELECT_PREFIX).tolist() == [1, 0, 0]
    assert orc.select_shots(scores, lengths, 25, orc.SELECT_FIRST_FIT).tolist() == [1, 0, 1]
    assert orc.select_shots([1.0, 9.0], [5, 50], 20, orc.SELECT_PREFIX).tolist() == [0, 0]


def test_decision_margin():
    # ranking 0,1,2,3 ; budget holds the top two ; only the 1<->2 swap changes the kept set
    scores = np.array([4.0, 3.0, 2.97, 1.0])
    lengths = [10, 10, 10, 10]
    m = orc.decision_margin(scores, lengths, 20)
    assert abs(m - 0.01) < 1e-12
    # equal lengths and room for everything: no swap matters
    assert orc.decision_margin(scores, lengths, 40) == np.inf
    # the first rejected shot is long, the one after it would fit: swapping those two matters (gap
    # 0.1/3), and so does swapping the top two (gap 1/4: the long shot would then block everything)
    m = orc.decision_margin(np.array([4.0, 3.0, 2.9]), [10, 30, 5], 20)
    assert abs(m - (0.1 / 3.0)) < 1e-12
    m = orc.decision_margin(np.array([4.0, 3.0, 2.0]), [10, 30, 5], 20)
    assert abs(m - 0.25) < 1e-12


def test_degenerate_inputs():
    rng = np.random.default_rng(9)
    q, k, v = _rand_problem(rng, 2, 1, 4, 2, 12)
    assert orc.prefill_compress(q, k, v, [0, 5, 5], 12, 1.0)["status"] == orc.STATUS_BAD_OFFSETS
    assert orc.prefill_compress(q, k, v, [3, 2], 12, 1.0)["status"] == orc.STATUS_BAD_OFFSETS
    assert orc.prefill_compress(q, k, v, [0, 13], 12, 1.0)["status"] == orc.STATUS_BAD_OFFSETS
    r = orc.prefill_compress(q, k, v, [4], 12, 1.0)            # no shots: keep everything
    assert r["status"] == orc.STATUS_OK and r["kept_positions"].tolist() == list(range(12))
    assert orc.prefill_compress(q, k, v, [4], 11, 1.0)["status"] == orc.STATUS_BUDGET_TOO_SMALL
    r = orc.prefill_compress(q, k, v, [0, 6], 6, 1.0)          # tail alone fills the budget
    assert r["status"] == orc.STATUS_OK and r["kept_positions"].tolist() == list(range(6, 12))


def test_boundary_cases_of_the_offset_check_and_a_window_as_long_as_the_prompt():
    """The last shot may end at the last token, and the window may be the whole prompt (then every query
    row is causally masked); one past either is an error."""
    assert orc.offsets_valid([0, 4, 8], 8, 2) and not orc.offsets_valid([0, 4, 9], 8, 2)
    assert orc.offsets_valid([0, 1], 4, 4) and not orc.offsets_valid([0, 1], 4, 5)
    # W = N = 3, keys all equal: query j sees keys 0..j with weight 1/(j+1), so over H heads
    # mass = H * (1 + 1/2 + 1/3, 1/2 + 1/3, 1/3); the one shot [0, 3) has score H * 3 / 3
    H = 2
    q = np.ones((H, 3, 2)); k = np.zeros((1, 3, 2)); v = np.arange(6.0).reshape(1, 3, 2)
    r = orc.prefill_compress(q, k, v, [0, 3], 3, 1.0)
    assert r["status"] == orc.STATUS_OK and r["kept_positions"].tolist() == [0, 1, 2]
    np.testing.assert_allclose(r["mass"], [float(H * Fraction(11, 6)), float(H * Fraction(5, 6)), float(H * Fraction(1, 3))],
                               rtol=1e-14)
    np.testing.assert_allclose(r["scores"], [float(H)], rtol=1e-14)
    assert orc.prefill_compress(q, k, v, [0, 4], 3, 1.0)["status"] == orc.STATUS_BAD_OFFSETS


def test_softmax_is_shift_invariant_at_logits_that_overflow_a_plain_exponential():
    """Logits x_t + 1000 with x = (0, ln 2, ln 3): the weights are 1/6, 2/6, 3/6 whatever the common offset
    (exp(1000) is not representable, so this only holds when the maximum is taken out first)."""
    k = np.array([[[0.0, 1.0], [math.log(2.0), 1.0], [math.log(3.0), 1.0]]])      # [1, 3, 2]
    q = np.array([[[1.0, 1000.0]]])                                                # [1, 1, 2]: W = 1 sees all keys
    p = orc.window_attention(q, k, 1.0)
    np.testing.assert_allclose(p[0, 0], [1 / 6, 2 / 6, 3 / 6], rtol=1e-12)
    v = np.array([[[6.0, 0.0], [12.0, 0.0], [18.0, 0.0]]])
    qs = np.repeat(q, 3, axis=1)                                                   # the same query at every position
    out = orc.causal_attention(qs, k, v, 1.0)
    np.testing.assert_allclose(out[0, :, 0], [6.0, (6 + 2 * 12) / 3, (6 + 2 * 12 + 3 * 18) / 6], rtol=1e-12)


def test_scores_given_from_outside_decide_the_selection():
    """The walk can be replayed on scores that come from elsewhere (a device's): they rank the shots and
    set the margin, while the result still reports the scores computed here."""
    rng = np.random.default_rng(31)
    q, k, v = _rand_problem(rng, 2, 1, 4, 2, 20)
    off = [0, 6, 12, 18]
    own = orc.prefill_compress(q, k, v, off, 8, 1.0)              # room for one shot
    best = int(np.argmax(own["scores"]))
    assert own["selected"].tolist() == [int(i == best) for i in range(3)]
    other = (best + 1) % 3
    given = np.array([1.0, 1.0, 1.0]); given[other] = 2.0; given[best] = 0.5
    r = orc.prefill_compress(q, k, v, off, 8, 1.0, scores_override=given)
    assert r["selected"].tolist() == [int(i == other) for i in range(3)]
    np.testing.assert_array_equal(r["scores"], own["scores"])
    assert r["kept_positions"].tolist() == list(range(6 * other, 6 * other + 6)) + [18, 19]
    assert abs(r["margin"] - 0.5) < 1e-12                          # (2 - 1) / 2, from the given scores
    np.testing.assert_array_equal(r["k_out"], k[:, r["kept_positions"]])


def test_workload_layouts():
    for shape in wl.PREFILL_SHAPES.values():
        for p in (0, 1):
            off = wl.shot_offsets(shape, p)
            assert off[0] == 0 and np.all(np.diff(off) > 0)
            assert off[-1] <= shape.n_tokens - shape.window
            assert orc.offsets_valid(off, shape.n_tokens, shape.window)
            if shape.tail_tokens:
                assert shape.n_tokens - off[-1] == shape.tail_tokens
        assert np.array_equal(wl.shot_offsets(shape, 3), wl.shot_offsets(shape, 3))


# ---- per-KV-head variant ---------------------------------------------------------------------------

def test_per_kv_head_scores_add_up_to_the_layer_score():
    """Eq. 3 is a sum over heads, so the per-KV-head scores (each summing its own G query heads) add up
    to the per-layer score, and each head's mass sums to G * W."""
    rng = np.random.default_rng(11)
    H, Hkv, D, W, N = 8, 4, 16, 4, 96
    q, k, v = _rand_problem(rng, H, Hkv, D, W, N)
    off = [3, 20, 41, 60, 85]
    layer = orc.prefill_compress(q, k, v, off, 60, 0.25)
    heads = orc.prefill_compress_per_kv_head(q, k, v, off, 60, 0.25)
    assert len(heads) == Hkv
    np.testing.assert_allclose(sum(h["scores"] for h in heads), layer["scores"], rtol=1e-12)
    for h in heads:
        assert abs(h["mass"].sum() - (H // Hkv) * W) < 1e-10


def test_per_kv_head_selection_is_bruteforce_optimal_per_head():
    rng = np.random.default_rng(12)
    H, Hkv, D, W, N = 4, 2, 8, 2, 64
    q, k, v = _rand_problem(rng, H, Hkv, D, W, N)
    off = np.array([2, 9, 17, 22, 30, 41, 47, 56])
    lengths = off[1:] - off[:-1]
    n_always = 2 + (N - 56)
    for mode in (orc.SELECT_PREFIX, orc.SELECT_FIRST_FIT):
        heads = orc.prefill_compress_per_kv_head(q, k, v, off, n_always + 25, 0.35, mode)
        differ = False
        for g, h in enumerate(heads):
            np.testing.assert_array_equal(h["selected"], orc.bruteforce_select(h["scores"], lengths, 25, mode))
            assert h["kept_count"] <= n_always + 25
            np.testing.assert_array_equal(h["k_out"][0], k[g][h["kept_positions"]])
            np.testing.assert_array_equal(h["v_out"][0], v[g][h["kept_positions"]])
            differ |= not np.array_equal(h["selected"], heads[0]["selected"])
        assert differ or mode == orc.SELECT_FIRST_FIT   # seed chosen so the heads disagree (ragged caches)


def test_per_kv_head_with_identical_heads_equals_the_layer_selection():
    """Copies of one KV head (and of its query group) rank the shots identically, and the per-layer score
    is H_kv times each head's, so both variants keep the same shots."""
    rng = np.random.default_rng(13)
    G, Hkv, D, W, N = 2, 3, 8, 3, 80
    q1, k1, v1 = _rand_problem(rng, G, 1, D, W, N)
    q, k, v = np.tile(q1, (Hkv, 1, 1)), np.tile(k1, (Hkv, 1, 1)), np.tile(v1, (Hkv, 1, 1))
    off = [0, 11, 25, 33, 52, 70]
    layer = orc.prefill_compress(q, k, v, off, 45, 0.3)
    for h in orc.prefill_compress_per_kv_head(q, k, v, off, 45, 0.3):
        np.testing.assert_array_equal(h["selected"], layer["selected"])
        np.testing.assert_array_equal(h["kept_positions"], layer["kept_positions"])
        np.testing.assert_allclose(h["scores"] * Hkv, layer["scores"], rtol=1e-12)


# ---- causal_attention: the prompt's own attention pass (for the entry point that fuses scoring into it)

def test_causal_attention_hand_example_and_closed_forms():
    """H=1, D=1, three tokens, sm_scale = ln 2 so that weights are powers of two:
    q = (1, 1, 2), k = (0, 1, 2), v = (8, 4, 2).  Row 0 sees key 0 only -> 8.  Row 1: weights 2^0 : 2^1 ->
    (8 + 2*4)/3 = 16/3.  Row 2 (q=2): weights 2^0 : 2^2 : 2^4 -> (8 + 4*4 + 16*2)/21 = 56/21 = 8/3."""
    q = np.array([[[1.0], [1.0], [2.0]]]); k = np.array([[[0.0], [1.0], [2.0]]]); v = np.array([[[8.0], [4.0], [2.0]]])
    out = orc.causal_attention(q, k, v, np.log(2.0))
    np.testing.assert_allclose(out[0, :, 0], [8.0, 16.0 / 3.0, 8.0 / 3.0], rtol=1e-14)
    # all keys equal: every row is the running mean of V, whatever the queries are
    rng = np.random.default_rng(5)
    q = rng.standard_normal((4, 9, 8)); k = np.tile(rng.standard_normal((2, 1, 8)), (1, 9, 1))
    v = rng.standard_normal((2, 9, 8))
    out = orc.causal_attention(q, k, v, 0.3)
    running = np.cumsum(v, axis=1) / np.arange(1, 10)[None, :, None]
    for h in range(4):
        np.testing.assert_allclose(out[h], running[h // 2], rtol=1e-12)


def test_causal_attention_matches_library_attention_and_the_window_weights():
    """Third opinion: torch's scaled_dot_product_attention (causal, grouped heads) in float64.  And the last
    W rows are the window rows of Eq. 3: out[:, N-W:] = window_attention weights @ V."""
    rng = np.random.default_rng(11)
    H, H_kv, N, D, W = 6, 2, 37, 16, 5
    q = rng.standard_normal((H, N, D)); k = rng.standard_normal((H_kv, N, D)); v = rng.standard_normal((H_kv, N, D))
    scale = 1.0 / np.sqrt(D)
    out = orc.causal_attention(q, k, v, scale)
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q)[None], torch.from_numpy(k)[None], torch.from_numpy(v)[None], is_causal=True,
        scale=scale, enable_gqa=True)[0].numpy()
    np.testing.assert_allclose(out, ref, rtol=1e-10, atol=1e-12)
    p = orc.window_attention(q[:, N - W:], k, scale)             # [H, W, N]
    G = H // H_kv
    for h in range(H):
        np.testing.assert_allclose(out[h, N - W:], p[h] @ v[h // G], rtol=1e-12, atol=1e-14)
    # a transposed operand or a dropped mask would show: the first row is v[0], row i ignores keys > i
    np.testing.assert_allclose(out[:, 0], np.repeat(v[:, 0], G, axis=0), rtol=1e-14)
    k2 = k.copy(); v2 = v.copy(); k2[:, 20:] += 3.0; v2[:, 20:] -= 1.0
    np.testing.assert_array_equal(orc.causal_attention(q, k2, v2, scale)[:, :20], out[:, :20])
