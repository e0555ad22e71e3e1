"""The library only enqueues kernels on the caller's stream (no allocation, no synchronisation, no memset),
so a whole compression + decode step can be captured into a HIP graph and replayed."""
import pytest
import torch

from paper_2502_01941_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def kv():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2502_01941_amd import shotkv
    shotkv.load_library()
    return shotkv


def test_capture_and_replay_matches_eager(kv):
    shape = wl.PrefillShape("graph", 3, 32, 8, 128, 32, 3000, 12, torch.bfloat16, 1200)
    q, k, v, off, bud = wl.prefill_batch(shape, "cuda", 9)
    P, cap = shape.n_problems, shape.budget_tokens
    ws = torch.empty(kv.prefill_workspace_bytes(32, 8, 128, 32, torch.bfloat16, P, shape.n_tokens, shape.n_shots),
                     dtype=torch.uint8, device="cuda")
    out = kv._alloc_prefill_outputs(k, P, 8, cap, 128, shape.n_shots)
    n_slots, budget = 7, 6
    k_dec = torch.zeros((P, 8, n_slots, 128), dtype=torch.bfloat16, device="cuda")
    v_dec = torch.zeros_like(k_dec)
    slot_pos = torch.full((P, n_slots), -1, dtype=torch.int32, device="cuda")
    state = kv.DecodeState(out.k_out, out.v_out, out.kept_count, k_dec, v_dec, slot_pos, budget, 32, shape.sm_scale)
    dshape = wl.DecodeShape("graph", P, 32, 8, 128, cap, budget, 0, torch.bfloat16)

    def run(step, qn, kn, vn):
        kv.prefill_compress(q, k, v, off, bud, cap, shape.sm_scale, out=out, workspace=ws)
        kv.decode_step(state, step, qn, kn, vn)

    # fill the slot pool eagerly so that the captured step evicts
    for step in range(budget):
        run(step, *wl.decode_inputs(dshape, step, "cuda", 9))
    torch.cuda.synchronize()
    snap = [t.clone() for t in (k_dec, v_dec, slot_pos)]
    qn, kn, vn = wl.decode_inputs(dshape, budget, "cuda", 9)

    # eager reference of the step that will be captured
    run(budget, qn, kn, vn)
    torch.cuda.synchronize()
    def live():   # rows past kept_count are never written: compare what the library defines
        kept = out.kept_count.cpu().tolist()
        rows = [out.kept_positions[p, :kept[p]].clone() for p in range(P)]
        rows += [out.k_out[p, :, :kept[p]].clone() for p in range(P)]
        rows += [out.v_out[p, :, :kept[p]].clone() for p in range(P)]
        return rows + [t.clone() for t in (out.kept_count, out.shot_scores, out.shot_selected, state.out,
                                            state.token_scores, state.evicted_pos, slot_pos, k_dec, v_dec)]

    want = live()
    assert int(state.evicted_pos.min().item()) >= 0

    def restore():
        for t, s in zip((k_dec, v_dec, slot_pos), snap):
            t.copy_(s)
        for t in (out.kept_positions, out.kept_count, out.shot_scores, state.out, state.token_scores,
                  state.evicted_pos):
            t.zero_()

    restore()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            run(budget, qn, kn, vn)
    torch.cuda.current_stream().wait_stream(side)
    for _ in range(3):
        restore()                       # eager work and a synchronisation between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = live()
        assert len(got) == len(want)
        for g, w in zip(got, want):
            assert torch.equal(g, w)


def test_caller_owned_timing_events(kv):
    """shotkv_config.timing_events: the library records the caller's HIP events around each kernel of a
    call and nothing else changes - same results bit for bit, positive durations for the kinds that ran,
    and no recording once the events are withdrawn."""
    shape = wl.PrefillShape("timed", 2, 32, 8, 128, 32, 3000, 12, torch.bfloat16, 1200)
    q, k, v, off, bud = wl.prefill_batch(shape, "cuda", 4)
    plain = kv.prefill_compress(q, k, v, off, bud, shape.budget_tokens, shape.sm_scale)
    torch.cuda.synchronize()
    timers = kv.KernelTimers()
    with timers:
        timed = kv.prefill_compress(q, k, v, off, bud, shape.budget_tokens, shape.sm_scale)
        ms = timers.read(("plan", "score", "row_stats", "chunk_mass", "reduce_select", "compact"))
    assert all(x > 0.0 for x in ms.values()), ms
    assert ms["score"] < 50.0 and ms["plan"] < 50.0
    for a, b in ((plain.shot_scores, timed.shot_scores), (plain.shot_selected, timed.shot_selected),
                 (plain.kept_count, timed.kept_count), (plain.status, timed.status)):
        assert torch.equal(a, b)
    kept = int(plain.kept_count[0])
    assert torch.equal(plain.k_out[0, :, :kept], timed.k_out[0, :, :kept])
    # decode: a state made outside the context is timed inside it and not outside
    dshape = wl.DecodeShape("timed", 2, 32, 8, 128, shape.budget_tokens, 8, 0, torch.bfloat16)
    k_dec = torch.zeros((2, 8, 9, 128), dtype=torch.bfloat16, device="cuda")
    state = kv.DecodeState(plain.k_out, plain.v_out, plain.kept_count, k_dec, torch.zeros_like(k_dec),
                           torch.full((2, 9), -1, dtype=torch.int32, device="cuda"), 8, 32, shape.sm_scale)
    qn, kn, vn = wl.decode_inputs(dshape, 0, "cuda", 4)
    with timers:
        kv.decode_step(state, 0, qn, kn, vn)
        dms = timers.read(("decode_partial", "decode_finish"))
    assert all(x > 0.0 for x in dms.values()), dms
    kv.decode_step(state, 1, qn, kn, vn)
    torch.cuda.synchronize()
    assert state.cfg.timing_events is None and int(state.status.abs().sum().item()) == 0
