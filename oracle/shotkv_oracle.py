"""CPU oracle for ShotKV's two-phase KV-cache compression (arXiv 2502.01941, Section 5 and Algorithm 1).

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain definition of what the GPU library must
compute.  It shares no code with the HIP path, imports nothing from it, and must never be called by
product code: only the tests, the smoke check and the benchmark's CPU-baseline leg use it.

Everything is numpy in float64.  Inputs arrive as numpy arrays holding the exact values the GPU sees
(bf16 inputs are widened to float32/float64 by the caller, which is exact).

Where the paper leaves a point open the reading taken is stated at the function that needs it.
No function here is "parity unpinned": tests/test_oracle_*.py pin each one against hand-derived
values, closed forms, a library attention routine, or brute force.
"""
from __future__ import annotations

import itertools

import numpy as np

# Selection modes (Section 5.1, text after Eq. 3: shots are taken in descending score order "until"
# the budget is reached).
SELECT_PREFIX = 0     # stop at the first ranked shot that does not fit (literal "until")
SELECT_FIRST_FIT = 1  # skip a shot that does not fit and keep walking the ranking

# Per-problem status values, identical in meaning to the device-side status words.
STATUS_OK = 0
STATUS_BAD_OFFSETS = -1      # offsets not strictly increasing / outside [0, N] / window longer than N
STATUS_BUDGET_TOO_SMALL = -2  # tokens outside every shot already exceed the budget
STATUS_NO_FREE_SLOT = -3     # decode: slot pool exhausted


# --------------------------------------------------------------------------------------------------
# Prefill phase
# --------------------------------------------------------------------------------------------------

def window_attention(q_obs, k, sm_scale):
    """Attention weights of the observation-window queries over all prefill keys.

    alpha in Eq. 3 is the attention a key receives; the paper does not say from which queries.  The
    reading here: the last W prefill positions are the observation window, each window query attends
    causally (query j sits at position N-W+j and sees keys 0..N-W+j), and weights are a softmax of
    sm_scale * <q, k>.  Query head h reads KV head h // G with G = H / H_kv (grouped-query attention).

    q_obs: [H, W, D]; k: [H_kv, N, D].  Returns p: [H, W, N] float64, rows summing to 1 over the
    visible keys and exactly 0 on the masked ones.
    """
    q = np.asarray(q_obs, dtype=np.float64)
    kk = np.asarray(k, dtype=np.float64)
    H, W, D = q.shape
    H_kv, N, D2 = kk.shape
    assert D == D2 and H % H_kv == 0 and W <= N
    G = H // H_kv
    p = np.zeros((H, W, N), dtype=np.float64)
    for h in range(H):
        g = h // G
        z = float(sm_scale) * (q[h] @ kk[g].T)          # [W, N] logits
        for j in range(W):
            last = N - W + j                             # position of this query = last visible key
            row = z[j, : last + 1]
            e = np.exp(row - row.max())
            p[h, j, : last + 1] = e / e.sum()
    return p


def token_mass(p):
    """sum_h alpha_{t,h} of Eq. 3 with alpha accumulated over the window rows: [H, W, N] -> [N]."""
    return p.sum(axis=(0, 1))


def shot_scores_from_mass(mass, shot_offsets):
    """Eq. 3: Score(s_i) = (1/k_i) * sum_{t in s_i} mass[t]; shot i spans [off[i], off[i+1])."""
    off = np.asarray(shot_offsets, dtype=np.int64)
    n = off.size - 1
    scores = np.zeros(n, dtype=np.float64)
    for i in range(n):
        scores[i] = mass[off[i]: off[i + 1]].sum() / float(off[i + 1] - off[i])
    return scores


def offsets_valid(shot_offsets, n_tokens, window):
    off = np.asarray(shot_offsets, dtype=np.int64)
    if window > n_tokens or off.size < 1:
        return False
    if off[0] < 0 or off[-1] > n_tokens:
        return False
    return bool(np.all(off[1:] > off[:-1]))


def rank_shots(scores):
    """Ranking used by the selection: score descending, ties to the lower shot index."""
    s = np.asarray(scores)
    return sorted(range(s.size), key=lambda i: (-s[i], i))


def select_shots(scores, lengths, shot_budget, mode=SELECT_PREFIX):
    """Eq. 5-6 / Algorithm 1 phase 1: walk the ranking, keeping whole shots while they fit.

    `scores` are compared exactly as given (any float dtype), so the same routine ranks the oracle's
    float64 scores or a device's float32 scores.  Returns a uint8 keep mask.
    """
    lengths = np.asarray(lengths, dtype=np.int64)
    keep = np.zeros(lengths.size, dtype=np.uint8)
    used = 0
    for i in rank_shots(scores):
        if used + lengths[i] <= shot_budget:
            keep[i] = 1
            used += int(lengths[i])
        elif mode == SELECT_PREFIX:
            break
    return keep


def bruteforce_select(scores, lengths, shot_budget, mode=SELECT_PREFIX):
    """Characterisation of the selection by enumeration of all 2^n shot subsets (n small).

    PREFIX: the largest feasible subset that is closed under the ranking (contains every shot ranked
    above any member).  FIRST_FIT: the feasible subset whose indicator vector, read in rank order, is
    lexicographically greatest.  Feasible = total length <= shot_budget (Eq. 6).
    """
    lengths = np.asarray(lengths, dtype=np.int64)
    n = lengths.size
    order = rank_shots(scores)
    pos = {shot: r for r, shot in enumerate(order)}
    best_key, best = None, None
    for bits in itertools.product((0, 1), repeat=n):
        if sum(int(lengths[i]) for i in range(n) if bits[i]) > shot_budget:
            continue
        in_rank_order = tuple(bits[order[r]] for r in range(n))
        if mode == SELECT_PREFIX:
            members = [pos[i] for i in range(n) if bits[i]]
            if members and max(members) != len(members) - 1:
                continue                                   # not a prefix of the ranking
            key = (sum(bits),)
        else:
            key = in_rank_order
        if best_key is None or key > best_key:
            best_key, best = key, bits
    return np.array(best, dtype=np.uint8)


def decision_margin(scores, lengths, shot_budget, mode=SELECT_PREFIX):
    """Smallest relative score gap between two rank-adjacent shots whose swap changes the kept set.

    With exact arithmetic the selection is unique; in floating point it can flip only when such a pair
    is closer than the score error.  inf when no adjacent swap matters.
    """
    s = np.asarray(scores, dtype=np.float64)
    order = rank_shots(s)
    base = select_shots(s, lengths, shot_budget, mode)
    margin = np.inf
    for r in range(len(order) - 1):
        a, b = order[r], order[r + 1]
        # rank b strictly above a, everything else unchanged (synthetic strictly decreasing scores)
        alt_order = order[:r] + [b, a] + order[r + 2:]
        alt_scores = np.empty_like(s)
        alt_scores[alt_order] = np.arange(len(order), 0, -1, dtype=np.float64)
        if not np.array_equal(select_shots(alt_scores, lengths, shot_budget, mode), base):
            gap = abs(s[a] - s[b]) / max(abs(s[a]), abs(s[b]), 1e-300)
            margin = min(margin, gap)
    return margin


def kept_positions_from_mask(keep, shot_offsets, n_tokens):
    """Retained token positions, ascending: everything outside the shots plus the kept shots."""
    off = np.asarray(shot_offsets, dtype=np.int64)
    parts = [np.arange(0, off[0])]
    for i in range(off.size - 1):
        if keep[i]:
            parts.append(np.arange(off[i], off[i + 1]))
    parts.append(np.arange(off[-1], n_tokens))
    return np.concatenate(parts).astype(np.int32)


def prefill_compress(q_obs, k, v, shot_offsets, budget_tokens, sm_scale, mode=SELECT_PREFIX,
                     scores_override=None):
    """One (batch, layer) problem of Algorithm 1 phase 1.

    Steps: window attention -> per-token mass summed over all H heads (Eq. 3 sums h = 1..H, so one
    selection per layer, shared by the KV heads) -> length-normalised shot scores -> ranked whole-shot
    selection under the budget (Eq. 5-6) -> Compress = gather of the retained K/V rows (Eq. 4; the
    compression operator of Section 3 keeps a subset of the original rows, so the output is bit-exact).

    Readings of open points: tokens outside every shot (prefix before the first shot, question tail
    including the window) are always retained and are charged to the budget first, so that the retained
    total never exceeds it; retained rows are stored in ascending original position.

    scores_override: rank these scores instead of the oracle's own (used to replay the selection on the
    scores a device produced).
    """
    k = np.asarray(k)
    v = np.asarray(v)
    H, W, D = np.asarray(q_obs).shape
    H_kv, N, _ = k.shape
    off = np.asarray(shot_offsets, dtype=np.int64)
    n = off.size - 1
    out = {
        "status": STATUS_OK, "scores": np.zeros(n), "selected": np.zeros(n, dtype=np.uint8),
        "kept_positions": np.zeros(0, dtype=np.int32), "kept_count": 0,
        "k_out": k[:, :0, :].copy(), "v_out": v[:, :0, :].copy(), "margin": np.inf,
    }
    if not offsets_valid(off, N, W):
        out["status"] = STATUS_BAD_OFFSETS
        return out
    p = window_attention(q_obs, k, sm_scale)
    mass = token_mass(p)
    scores = shot_scores_from_mass(mass, off)
    out["scores"] = scores
    out["mass"] = mass
    rank_on = scores if scores_override is None else np.asarray(scores_override)
    lengths = off[1:] - off[:-1]
    n_always = int(off[0]) + int(N - off[-1])
    shot_budget = int(budget_tokens) - n_always
    if shot_budget < 0:
        out["status"] = STATUS_BUDGET_TOO_SMALL
        return out
    keep = select_shots(rank_on, lengths, shot_budget, mode)
    pos = kept_positions_from_mask(keep, off, N)
    out["selected"] = keep
    out["kept_positions"] = pos
    out["kept_count"] = int(pos.size)
    out["k_out"] = k[:, pos, :].copy()
    out["v_out"] = v[:, pos, :].copy()
    out["margin"] = decision_margin(rank_on, lengths, shot_budget, mode)
    return out


def causal_attention(q, k, v, sm_scale):
    """Textbook causal softmax attention of a whole prompt, grouped-query layout.

    This is the attention pass the prefill phase of a decoder runs anyway; its last W query rows are the
    observation-window rows whose weights Eq. 3 pools (window_attention gives exactly those weights), so a
    kernel that computes this pass can emit the scores of Eq. 3 without reading K a second time.

    q: [H, N, D]; k, v: [H_kv, N, D].  Query i of head h sees keys 0..i of KV head h // G, weights are
    softmax(sm_scale * <q_i, k_t>).  Returns out [H, N, D] float64.
    """
    q = np.asarray(q, dtype=np.float64)
    kk = np.asarray(k, dtype=np.float64)
    vv = np.asarray(v, dtype=np.float64)
    H, N, D = q.shape
    H_kv = kk.shape[0]
    assert kk.shape == (H_kv, N, D) and vv.shape == (H_kv, N, D) and H % H_kv == 0
    G = H // H_kv
    out = np.zeros((H, N, D), dtype=np.float64)
    for h in range(H):
        g = h // G
        z = float(sm_scale) * (q[h] @ kk[g].T)           # [N, N] logits
        for i in range(N):
            row = z[i, : i + 1]
            e = np.exp(row - row.max())
            out[h, i] = (e / e.sum()) @ vv[g, : i + 1]
    return out


def prefill_compress_per_kv_head(q_obs, k, v, shot_offsets, budget_tokens, sm_scale,
                                 mode=SELECT_PREFIX, scores_override=None):
    """Variant of phase 1 in which every KV head keeps its own set of shots.

    Eq. 3 sums the attention weights over all H query heads, which gives one selection per layer.
    Under grouped-query attention the KV head g is read only by the G = H / H_kv query heads
    g*G .. g*G+G-1; restricting the head sum of Eq. 3 to that group scores each shot once per KV head,
    and Eq. 4-6 then run independently per KV head with the same shot boundaries and the same token
    budget.  The caches of different heads may therefore retain different shots (ragged caches).

    Returns a list of H_kv results, each shaped like prefill_compress's for a single KV head
    (k_out/v_out are [1][kept][D]).  scores_override, if given, is [H_kv][n].
    """
    q_obs = np.asarray(q_obs)
    k = np.asarray(k)
    v = np.asarray(v)
    H = q_obs.shape[0]
    H_kv = k.shape[0]
    G = H // H_kv
    results = []
    for g in range(H_kv):
        override = None if scores_override is None else np.asarray(scores_override)[g]
        results.append(prefill_compress(q_obs[g * G:(g + 1) * G], k[g:g + 1], v[g:g + 1], shot_offsets,
                                        budget_tokens, sm_scale, mode, override))
    return results


# --------------------------------------------------------------------------------------------------
# Decoding phase
# --------------------------------------------------------------------------------------------------

def decode_step(k_prefill, v_prefill, prefill_count, k_dec, v_dec, slot_pos, decode_budget,
                step_index, q_new, k_new, v_new, sm_scale):
    """One decoding step of one sequence at one layer (Algorithm 1 phase 2, Eq. 7-9).

    State: the fixed compressed prefill cache k_prefill/v_prefill [H_kv, cap, D] of which the first
    prefill_count rows are live, and a pool of decode slots k_dec/v_dec [H_kv, n_slots, D] with
    slot_pos[n_slots] = index of the generated token each slot holds, -1 when free.  k_dec, v_dec and
    slot_pos are updated in place.

    1. The new token's key/value go into the lowest-numbered free slot.
    2. Every query head attends over the union of the prefill cache and the occupied slots (Eq. 9).
    3. Score(t) = sum over heads of the weight the current query gives decode token t (Eq. 7; the score
       is that of the current step only).
    4. Retention (Eq. 8) in capacity form: the decode cache holds at most decode_budget tokens; when
       the new token makes it exceed that, the lowest-scored previously generated token is evicted
       (the current token is not a candidate; among equal scores the newest token goes, so the kept set
       is the top decode_budget by score descending then token index ascending).

    Returns dict(out [H, D] float64, token_scores [n_slots] (0 on free slots), evicted_pos, evicted_slot,
    new_slot, margin (relative gap between the two lowest candidate scores), status).
    """
    kp = np.asarray(k_prefill, dtype=np.float64)
    vp = np.asarray(v_prefill, dtype=np.float64)
    q = np.asarray(q_new, dtype=np.float64)
    H, D = q.shape
    H_kv = kp.shape[0]
    G = H // H_kv
    n_slots = slot_pos.shape[0]
    res = {"status": STATUS_OK, "out": np.zeros((H, D)), "token_scores": np.zeros(n_slots),
           "evicted_pos": -1, "evicted_slot": -1, "new_slot": -1}
    free = np.flatnonzero(slot_pos < 0)
    if free.size == 0:
        res["status"] = STATUS_NO_FREE_SLOT
        return res
    f = int(free[0])
    k_dec[:, f, :] = k_new
    v_dec[:, f, :] = v_new
    slot_pos[f] = step_index
    res["new_slot"] = f
    occ = np.flatnonzero(slot_pos >= 0)
    pc = int(prefill_count)
    kd = np.asarray(k_dec, dtype=np.float64)
    vd = np.asarray(v_dec, dtype=np.float64)
    scores = np.zeros(n_slots)
    for h in range(H):
        g = h // G
        # logits over the union [live prefill rows | occupied decode slots], one softmax over both
        z = float(sm_scale) * np.concatenate([kp[g, :pc] @ q[h], kd[g, occ] @ q[h]])
        e = np.exp(z - z.max())
        w = e / e.sum()
        res["out"][h] = w[:pc] @ vp[g, :pc] + w[pc:] @ vd[g, occ]
        scores[occ] += w[pc:]
    res["token_scores"] = scores
    res["margin"] = eviction_margin(scores, slot_pos, f)
    if occ.size > decode_budget:
        cand = [s for s in occ if s != f]
        # lowest score goes; among equals the newest (largest token index)
        e_slot = min(cand, key=lambda s: (scores[s], -int(slot_pos[s])))
        res["evicted_slot"] = int(e_slot)
        res["evicted_pos"] = int(slot_pos[e_slot])
        slot_pos[e_slot] = -1
    return res


def eviction_margin(token_scores, slot_pos, new_slot):
    """Relative gap between the two lowest candidate scores of a decode step (inf if < 2 candidates)."""
    cand = [s for s in np.flatnonzero(np.asarray(slot_pos) >= 0) if s != new_slot]
    if len(cand) < 2:
        return np.inf
    vals = np.sort(np.asarray(token_scores, dtype=np.float64)[cand])
    return float((vals[1] - vals[0]) / max(vals[1], 1e-300))
