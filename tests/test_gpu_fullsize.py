"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times: all problems of
the 32K-token (128 problems), 128K-token skewed (32 problems) and sentence-unit workloads in one call,
and the oracle on EVERY problem of each (in slices, so that no single test stays silent for long).
Problems whose decision margin is below 1e-6 are listed, not hidden: they are checked against the
oracle's walk on the device's own scores like every other problem, and reported at the end."""
import numpy as np
import pytest
import torch

import helpers
from helpers import check_prefill_problem
from paper_2502_01941_amd import workloads as wl

pytestmark = pytest.mark.gpu

N_SLICES = 8
NEAR_TIES = {}      # workload name -> [(problem, margin, device agrees with the oracle end to end)]
CHECKED = {}        # workload name -> set of problems the oracle has been run on


@pytest.fixture(scope="module")
def kv():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2502_01941_amd import shotkv
    shotkv.load_library()
    return shotkv


@pytest.fixture(scope="module", params=["model32k", "skew128k", "sentences16k"])
def full(request, kv):
    """One call over the whole workload; the inputs and the result stay on the GPU for the module's tests."""
    shape = wl.PREFILL_SHAPES[request.param]
    q, k, v, off, bud = wl.prefill_batch(shape, "cuda")
    res = kv.prefill_compress(q, k, v, off, bud, shape.budget_tokens, shape.sm_scale)
    torch.cuda.synchronize()
    NEAR_TIES[shape.name] = []
    CHECKED[shape.name] = set()
    yield {"shape": shape, "q": q, "k": k, "v": v, "off": off, "bud": bud, "res": res}
    del q, k, v, res
    torch.cuda.empty_cache()


def test_properties_on_every_problem(full):
    """Hold at any size: status, budget, whole shots, ascending positions, bit-exact gather, the mass
    bound sum_i k_i * Score_i <= H * W (the rest of the H*W unit rows sits outside the shots), and the
    selection rule replayed on the device's own scores."""
    shape, k, v, off, res = full["shape"], full["k"], full["v"], full["off"], full["res"]
    P, N = shape.n_problems, shape.n_tokens
    assert res.status.cpu().tolist() == [0] * P
    kept = res.kept_count.cpu().numpy()
    assert kept.max() <= shape.budget_tokens
    offs = off.cpu().numpy()
    sel = res.shot_selected.cpu().numpy()
    scores32 = res.shot_scores.cpu().numpy()
    pos_all = res.kept_positions.cpu().numpy()
    for p in range(P):
        helpers.check_selection_valid(sel[p], int(kept[p]), pos_all[p, : kept[p]], offs[p], N, shape.budget_tokens)
        mass = float((np.diff(offs[p]) * scores32[p].astype(np.float64)).sum())
        assert 0.0 < mass <= shape.n_q_heads * shape.window * (1 + 1e-5)
        keep_replay, pos_replay = helpers.replay_selection(scores32[p], offs[p], N, shape.budget_tokens, 0)
        assert sel[p].tolist() == keep_replay.tolist(), p
        np.testing.assert_array_equal(pos_all[p, : kept[p]], pos_replay)
        idx = res.kept_positions[p, : kept[p]].long()
        assert torch.equal(res.k_out[p, :, : kept[p]], k[p][:, idx])
        assert torch.equal(res.v_out[p, :, : kept[p]], v[p][:, idx])


@pytest.mark.parametrize("part", range(N_SLICES))
def test_oracle_on_every_problem(full, part):
    """Problems part, part + 8, ... of the workload against the oracle, element by element."""
    shape, q, k, v, off, res = full["shape"], full["q"], full["k"], full["v"], full["off"], full["res"]
    for p in range(part, shape.n_problems, N_SLICES):
        check_prefill_problem(res, p, q[p], k[p], v[p], off[p].cpu().numpy(), shape.budget_tokens,
                              shape.budget_tokens, shape.sm_scale, report=NEAR_TIES[shape.name])
        CHECKED[shape.name].add(p)


def test_near_tie_report(full, record_property):
    """Every problem has been through the oracle; the near ties (margin < 1e-6) are listed."""
    shape = full["shape"]
    assert CHECKED[shape.name] == set(range(shape.n_problems))
    near = sorted(NEAR_TIES[shape.name])
    record_property(f"near_ties_{shape.name}", repr(near))
    print(f"\n[{shape.name}] oracle on all {shape.n_problems} problems; margin < {helpers.MARGIN_EXACT:g} on "
          f"{len(near)}: {near}")
    # a near tie is rare by construction (relative score gaps are ~1e-5 at these sizes)
    assert len(near) <= max(2, shape.n_problems // 16), near
    if shape.name == "skew128k":    # the skewed shots dominate: everything kept comes from the shifted 10 %
        sel = full["res"].shot_selected.cpu().numpy()
        scores = full["res"].shot_scores.cpu().numpy()
        for p in range(shape.n_problems):
            assert scores[p][sel[p] == 1].min() > 1.2 * np.median(scores[p])


def test_decode_over_the_compressed_caches(kv, full):
    """The decode half of the benchmark step: one launch over all compressed caches (ragged live-row
    counts below cap, empty slot pools of budget + 1 slots), a few steps, every sequence followed by
    the oracle in lock step.  For the 32K workload (what the benchmark step decodes over) all 128 caches;
    for the other workloads the first 8."""
    shape, res = full["shape"], full["res"]
    from test_gpu_decode import OracleSeq, _compare_step
    if shape.name != "model32k":
        import types
        n = min(8, shape.n_problems)
        res = types.SimpleNamespace(k_out=res.k_out[:n].contiguous(), v_out=res.v_out[:n].contiguous(),
                                    kept_count=res.kept_count[:n].contiguous())
        shape = wl.PrefillShape(shape.name, n, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.window,
                                shape.n_tokens, shape.n_shots, shape.dtype, shape.budget_tokens)
    P, cap, budget = shape.n_problems, shape.budget_tokens, 1024
    n_slots = budget + 1
    k_dec = torch.zeros((P, shape.n_kv_heads, n_slots, shape.head_dim), dtype=shape.dtype, device="cuda")
    v_dec = torch.zeros_like(k_dec)
    slot_pos = torch.full((P, n_slots), -1, dtype=torch.int32, device="cuda")
    assert int(res.kept_count.min().item()) <= cap
    # rows past the live count are whatever the allocator left: make them hostile
    k_pre, v_pre = res.k_out.clone(), res.v_out.clone()
    for p in range(P):
        c = int(res.kept_count[p].item())
        k_pre[p, :, c:] = float("nan")
        v_pre[p, :, c:] = float("inf")
    state = kv.DecodeState(k_pre, v_pre, res.kept_count, k_dec, v_dec, slot_pos, budget,
                           shape.n_q_heads, shape.sm_scale)
    st = {"k_prefill": k_pre, "v_prefill": v_pre, "prefill_count": res.kept_count, "k_dec": k_dec,
          "v_dec": v_dec, "slot_pos": slot_pos}
    seqs = {}
    for p in range(P):
        seq = OracleSeq(st, p)
        c = seq.pc                                              # the oracle never looks past the live rows
        seq.kp, seq.vp = seq.kp[:, :c].copy(), seq.vp[:, :c].copy()
        seqs[p] = seq
    dshape = wl.DecodeShape("bench", P, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, cap, budget, 0,
                            shape.dtype)
    near = []
    for step in range(3):
        qn, kn, vn = wl.decode_inputs(dshape, step, "cuda")
        kv.decode_step(state, step, qn, kn, vn)
        torch.cuda.synchronize()
        assert state.status.cpu().tolist() == [0] * P
        assert torch.isfinite(state.out).all()
        for p, seq in seqs.items():
            r = seq.step(budget, step, qn[p], kn[p], vn[p], shape.sm_scale)
            _compare_step(state, p, r, seq, near)
    assert not near
    assert ((slot_pos >= 0).sum(dim=1) == 3).all()
