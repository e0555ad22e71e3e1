"""GPU parity: decode steps through the C ABI against the CPU oracle, in lock step on the same inputs."""
import numpy as np
import pytest
import torch

from helpers import to_np
from oracle import shotkv_oracle as orc
from paper_2502_01941_amd import workloads as wl

pytestmark = pytest.mark.gpu

OUT_TOL = 1e-3        # |dO| <= OUT_TOL * max|O| per head row (fp32 accumulation on the device)
SCORE_RTOL = 1e-3
MARGIN_EXACT = 1e-6   # eviction must agree when the two lowest candidate scores differ by more


@pytest.fixture(scope="module")
def kv():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2502_01941_amd import shotkv
    shotkv.load_library()
    return shotkv


class OracleSeq:
    """Host-side state of one sequence, advanced only by the oracle's own decisions."""

    def __init__(self, st, s):
        self.kp = to_np(st["k_prefill"][s]).astype(np.float64)
        self.vp = to_np(st["v_prefill"][s]).astype(np.float64)
        self.pc = int(st["prefill_count"][s].item())
        self.kd = to_np(st["k_dec"][s]).copy(); self.vd = to_np(st["v_dec"][s]).copy()
        self.slot_pos = st["slot_pos"][s].cpu().numpy().copy()

    def step(self, budget, step, q, kn, vn, scale):
        return orc.decode_step(self.kp, self.vp, self.pc, self.kd, self.vd, self.slot_pos, budget, step,
                               to_np(q), to_np(kn), to_np(vn), scale)


def _make_state(kv, shape, st):
    return kv.DecodeState(st["k_prefill"], st["v_prefill"], st["prefill_count"], st["k_dec"], st["v_dec"],
                          st["slot_pos"], st["decode_budget"], shape.n_q_heads, shape.sm_scale)


class PoolMirror:
    """A device copy of the oracle's slot pool of one sequence, for the long lock-step test: every step the
    row the oracle appended is uploaded and the device pool is compared with the copy on the device, whole
    and bitwise; that the copy still equals the oracle's arrays is checked on the host every `every` steps
    and by the caller at the end (check_against_oracle)."""

    def __init__(self, state, seq, every=64):
        self.k = torch.from_numpy(seq.kd).to(state.k_dec.dtype).cuda()
        self.v = torch.from_numpy(seq.vd).to(state.v_dec.dtype).cuda()
        self.every, self.n = every, 0

    def check_against_oracle(self, seq):
        np.testing.assert_array_equal(to_np(self.k), seq.kd)
        np.testing.assert_array_equal(to_np(self.v), seq.vd)

    def step(self, state, s, r, seq):
        slot = r["new_slot"]
        if slot >= 0:
            self.k[:, slot] = torch.from_numpy(np.ascontiguousarray(seq.kd[:, slot])).to(self.k.dtype).cuda()
            self.v[:, slot] = torch.from_numpy(np.ascontiguousarray(seq.vd[:, slot])).to(self.v.dtype).cuda()
        assert torch.equal(state.k_dec[s], self.k) and torch.equal(state.v_dec[s], self.v)
        self.n += 1
        if self.n % self.every == 0:
            self.check_against_oracle(seq)


def _compare_step(state, s, r, seq, near_ties, mirror=None):
    """Device results of sequence s against the oracle's step result r."""
    assert int(state.status[s].item()) == r["status"]
    out = state.out[s].cpu().numpy().astype(np.float64)
    scale = np.abs(r["out"]).max(axis=1, keepdims=True)
    assert np.all(np.abs(out - r["out"]) <= OUT_TOL * scale), np.abs(out - r["out"]).max()
    ts = state.token_scores[s].cpu().numpy()
    np.testing.assert_allclose(ts, r["token_scores"], rtol=SCORE_RTOL, atol=1e-30)
    ev = int(state.evicted_pos[s].item())
    if ev != r["evicted_pos"]:
        # only legitimate when the two lowest scores are closer than the arithmetic can resolve: then
        # the device must have taken the other one of the pair; follow it so the states stay aligned
        assert r["margin"] < MARGIN_EXACT, (ev, r["evicted_pos"], r["margin"])
        alt_slot = int(np.flatnonzero(seq.slot_pos == ev)[0])
        cand = sorted((r["token_scores"][i], i) for i in np.flatnonzero(seq.slot_pos >= 0) if i != r["new_slot"])
        assert alt_slot == cand[0][1]          # after the oracle's eviction the runner-up is now the lowest
        seq.slot_pos[r["evicted_slot"]] = r["evicted_pos"]
        seq.slot_pos[alt_slot] = -1
        near_ties.append((s, ev))
    np.testing.assert_array_equal(state.slot_pos[s].cpu().numpy(), seq.slot_pos)
    # the slot pool itself: the appended K/V rows are bit-exact copies, nothing else is touched
    if mirror is not None:
        mirror.step(state, s, r, seq)
    else:
        np.testing.assert_array_equal(to_np(state.k_dec[s]), seq.kd)
        np.testing.assert_array_equal(to_np(state.v_dec[s]), seq.vd)


def test_tiny_free_running_320_steps(kv):
    """S=1, H=4, D=64, fp32, budget 32: every step's output, token scores, eviction and slot map."""
    shape = wl.DECODE_TINY
    st = wl.decode_state(shape, "cuda")
    state = _make_state(kv, shape, st)
    seq = OracleSeq(st, 0)
    kp_before = st["k_prefill"].clone()
    near = []
    for step in range(shape.n_steps):
        q, kn, vn = wl.decode_inputs(shape, step, "cuda")
        kv.decode_step(state, step, q, kn, vn)
        torch.cuda.synchronize()
        r = seq.step(shape.decode_budget, step, q[0], kn[0], vn[0], shape.sm_scale)
        _compare_step(state, 0, r, seq, near)
        occupied = int((state.slot_pos[0] >= 0).sum().item())
        assert occupied == min(step + 1, shape.decode_budget)
    assert len(near) == 0, near
    assert torch.equal(st["k_prefill"], kp_before)            # the prefill cache stays fixed
    np.testing.assert_array_equal(to_np(st["k_dec"][0]), seq.kd)
    np.testing.assert_array_equal(to_np(st["v_dec"][0]), seq.vd)


@pytest.mark.parametrize("group", range(4))
def test_decode4k_bf16_lockstep(kv, group):
    """The long-generation shape (16 sequences, 4096-token prefill cache, budget 1024) from a partly
    filled pool through the point where eviction starts and on into the steady state: the state holds
    768 generated tokens, 512 more steps follow (256 that fill the pool, 256 that evict every step).
    All 16 sequences are decoded in every launch; the four parametrisations follow four sequences each
    with the oracle at every step, so together every sequence is followed."""
    shape = wl.DECODE4K
    resident, steps = 768, 512
    st = wl.decode_state(shape, "cuda", resident=resident)
    state = _make_state(kv, shape, st)
    tracked = {s: OracleSeq(st, s) for s in range(group, shape.n_seqs, 4)}
    mirrors = {s: PoolMirror(state, seq) for s, seq in tracked.items()}
    vsum_before = st["v_prefill"].float().sum().item()
    near = []
    for step in range(resident, resident + steps):
        q, kn, vn = wl.decode_inputs(shape, step, "cuda")
        kv.decode_step(state, step, q, kn, vn)
        torch.cuda.synchronize()
        for s, seq in tracked.items():
            r = seq.step(shape.decode_budget, step, q[s], kn[s], vn[s], shape.sm_scale)
            _compare_step(state, s, r, seq, near, mirrors[s])
            assert (r["evicted_pos"] >= 0) == (step >= shape.decode_budget)
        assert state.status.cpu().tolist() == [0] * shape.n_seqs
    for s, seq in tracked.items():
        mirrors[s].check_against_oracle(seq)
        np.testing.assert_array_equal(to_np(state.k_dec[s]), seq.kd)
        np.testing.assert_array_equal(to_np(state.v_dec[s]), seq.vd)
    counts = (state.slot_pos >= 0).sum(dim=1).cpu().tolist()
    assert counts == [shape.decode_budget] * shape.n_seqs
    assert st["v_prefill"].float().sum().item() == vsum_before
    # 4 x 256 evictions among ~1000 candidates each: a pair of lowest scores within 1e-6 is rare
    print(f"\n[decode4k group {group}] near-tie evictions followed: {near}")
    assert len(near) <= 4, near


def test_partial_prefill_and_unbounded_budget(kv):
    """prefill_count below cap (rows past it must be ignored), G=2, and the prefill-only ablation:
    with an unbounded budget nothing is ever evicted; a full pool reports its own status."""
    shape = wl.DecodeShape("odd", 3, 8, 4, 128, 100, kv.INT32_MAX, 0, torch.bfloat16)
    st = wl.decode_state(shape, "cuda", n_slots=6)
    st["prefill_count"] = torch.tensor([100, 37, 0], dtype=torch.int32, device="cuda")
    state = _make_state(kv, shape, st)
    seqs = [OracleSeq(st, s) for s in range(3)]
    near = []
    for step in range(7):
        q, kn, vn = wl.decode_inputs(shape, step, "cuda")
        kv.decode_step(state, step, q, kn, vn)
        torch.cuda.synchronize()
        for s in range(3):
            r = seqs[s].step(kv.INT32_MAX, step, q[s], kn[s], vn[s], shape.sm_scale)
            if step < 6:
                _compare_step(state, s, r, seqs[s], near)
                assert r["evicted_pos"] == -1
            else:
                assert r["status"] == orc.STATUS_NO_FREE_SLOT
                assert int(state.status[s].item()) == orc.STATUS_NO_FREE_SLOT
                np.testing.assert_array_equal(state.slot_pos[s].cpu().numpy(), seqs[s].slot_pos)


@pytest.mark.parametrize("H,H_kv,D,dtype", [(4, 4, 64, torch.float32), (8, 2, 128, torch.bfloat16)])
def test_equal_scores_evict_newest_previous_token(kv, H, H_kv, D, dtype):
    """All decode keys identical -> equal token scores; the evicted token must be the newest earlier
    one, never the token just appended: checked against the hand-written sequence and, strictly (a tie is
    no excuse here), against the oracle at every step."""
    shape = wl.DecodeShape("ties", 1, H, H_kv, D, 8, 3, 0, dtype)
    st = wl.decode_state(shape, "cuda")
    state = _make_state(kv, shape, st)
    seq = OracleSeq(st, 0)
    q = torch.ones((1, H, D), device="cuda").to(dtype)
    kn = torch.full((1, H_kv, D), 0.25, device="cuda").to(dtype)
    vn = torch.ones((1, H_kv, D), device="cuda").to(dtype)
    evicted = []
    for step in range(6):
        kv.decode_step(state, step, q, kn, vn)
        torch.cuda.synchronize()
        evicted.append(int(state.evicted_pos[0].item()))
        r = seq.step(shape.decode_budget, step, q[0], kn[0], vn[0], shape.sm_scale)
        assert evicted[-1] == r["evicted_pos"] and (step < 3 or r["margin"] == 0.0)
        np.testing.assert_array_equal(state.slot_pos[0].cpu().numpy(), seq.slot_pos)
        if step >= 1:       # the decode tokens' scores are equal to the last bit on the device as well
            ts = state.token_scores[0].cpu().numpy()
            held = ts[seq.slot_pos >= 0].tolist()
            if r["evicted_slot"] >= 0:
                held.append(ts[r["evicted_slot"]])
            assert len(set(held)) == 1
    assert evicted == [-1, -1, -1, 2, 3, 4]


def test_ratio_form_retention(kv):
    """Eq. 8 as printed, k = r_d * |KV_decoding|: the caller raises the budget to ceil(r_d * tokens
    generated so far) each step; one eviction per step keeps the decode cache at that size."""
    shape = wl.DecodeShape("ratio", 2, 8, 2, 128, 64, 1, 0, torch.bfloat16)
    r_d, steps = 0.4, 60
    n_slots = int(np.ceil(r_d * steps)) + 2
    st = wl.decode_state(shape, "cuda", n_slots=n_slots)
    state = _make_state(kv, shape, st)
    seqs = [OracleSeq(st, s) for s in range(2)]
    near = []
    for step in range(steps):
        budget = max(1, int(np.ceil(r_d * (step + 1))))
        state.decode_budget = budget
        state.c_state.decode_budget = budget
        q, kn, vn = wl.decode_inputs(shape, step, "cuda")
        kv.decode_step(state, step, q, kn, vn)
        torch.cuda.synchronize()
        for s in range(2):
            r = seqs[s].step(budget, step, q[s], kn[s], vn[s], shape.sm_scale)
            _compare_step(state, s, r, seqs[s], near)
            assert int((state.slot_pos[s] >= 0).sum().item()) == min(budget, step + 1)
    assert not near, near


def test_long_cache_many_splits(kv):
    """A 70 000-row prefill cache for one sequence: more than 64 token ranges per (sequence, KV head)."""
    shape = wl.DecodeShape("long", 1, 32, 8, 128, 70000, 16, 0, torch.bfloat16)
    st = wl.decode_state(shape, "cuda", 3, resident=16)
    state = _make_state(kv, shape, st)
    seq = OracleSeq(st, 0)
    near = []
    for step in range(16, 19):
        q, kn, vn = wl.decode_inputs(shape, step, "cuda", 3)
        kv.decode_step(state, step, q, kn, vn)
        torch.cuda.synchronize()
        r = seq.step(shape.decode_budget, step, q[0], kn[0], vn[0], shape.sm_scale)
        _compare_step(state, 0, r, seq, near)
        assert r["evicted_pos"] >= 0
    assert not near


@pytest.mark.parametrize("H,H_kv,D,dtype", [(28, 4, 128, torch.bfloat16), (40, 8, 128, torch.bfloat16),
                                             (12, 4, 128, torch.bfloat16), (6, 2, 64, torch.float32)])
def test_group_sizes_that_are_not_powers_of_two(kv, H, H_kv, D, dtype):
    """G = 7, 5, 3: the kernels run on the next power of two and must neither read nor write the padding
    heads.  Dead rows of the prefill cache hold NaN / Inf."""
    shape = wl.DecodeShape("g", 2, H, H_kv, D, 500, 6, 0, dtype)
    st = wl.decode_state(shape, "cuda", 5)
    st["prefill_count"] = torch.tensor([500, 333], dtype=torch.int32, device="cuda")
    st["k_prefill"][1, :, 333:] = float("nan")
    st["v_prefill"][1, :, 333:] = float("inf")
    state = _make_state(kv, shape, st)
    seqs = [OracleSeq(st, s) for s in range(2)]
    seqs[1].kp, seqs[1].vp = seqs[1].kp[:, :333].copy(), seqs[1].vp[:, :333].copy()
    near = []
    guard = torch.full_like(state.out, 12345.0)
    for step in range(10):
        q, kn, vn = wl.decode_inputs(shape, step, "cuda", 5)
        state.out.copy_(guard)
        kv.decode_step(state, step, q, kn, vn)
        torch.cuda.synchronize()
        assert torch.isfinite(state.out).all()
        for s, seq in enumerate(seqs):
            r = seq.step(shape.decode_budget, step, q[s], kn[s], vn[s], shape.sm_scale)
            _compare_step(state, s, r, seq, near)
    assert not near


@pytest.mark.parametrize("H,H_kv", [(32, 8), (8, 8), (16, 2)])
def test_new_token_without_weight_is_still_appended(kv, H, H_kv):
    """Algorithm 1 phase 2 appends the generated token's K/V unconditionally.  Here the new key is
    opposed to every query of its group by about 180 nats, so its weight is exactly zero in fp32 at the
    step that appends it; the value row must land in the pool all the same, because later steps (with
    ordinary queries) give that token real weight.  Pool contents are compared bit for bit after every
    step."""
    shape = wl.DecodeShape("noweight", 2, H, H_kv, 128, 300, 64, 0, torch.bfloat16)
    st = wl.decode_state(shape, "cuda", 9, n_slots=12)
    st["v_dec"].fill_(7.0)                       # a stale row would be visible in the output
    state = _make_state(kv, shape, st)
    seqs = [OracleSeq(st, s) for s in range(2)]
    near = []
    for step in range(6):
        q, kn, vn = wl.decode_inputs(shape, step, "cuda", 9)
        if step in (0, 2, 3):
            q = torch.full_like(q, 4.0)
            kn = torch.full_like(kn, -4.0)
        kv.decode_step(state, step, q, kn, vn)
        torch.cuda.synchronize()
        for s, seq in enumerate(seqs):
            r = seq.step(shape.decode_budget, step, q[s], kn[s], vn[s], shape.sm_scale)
            if step in (0, 2, 3):
                assert float(state.token_scores[s, r["new_slot"]].item()) == 0.0   # the case is really hit
            _compare_step(state, s, r, seq, near)
            slot = r["new_slot"]
            assert torch.equal(state.v_dec[s, :, slot], vn[s]) and torch.equal(state.k_dec[s, :, slot], kn[s])
    assert not near
