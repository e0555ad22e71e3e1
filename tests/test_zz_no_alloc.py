"""shotkv_decode_step_static (the entry point that allocates nothing) against shotkv_decode_step: same
inputs, two calls in a row, the second on a smaller problem; every output and the whole decode state must
agree bit for bit, since both run the same kernels and differ only in where the scratch memory lives."""
import ctypes

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


def _state(kv, shape, seed, resident):
    st = wl.decode_state(shape, "cuda", seed, resident=resident)
    return st, kv.DecodeState(st["k_prefill"], st["v_prefill"], st["prefill_count"], st["k_dec"], st["v_dec"],
                              st["slot_pos"], st["decode_budget"], shape.n_q_heads, shape.sm_scale)


def _same(a, b, st_a, st_b):
    assert torch.equal(a.status, b.status) and int(a.status.abs().sum().item()) == 0
    assert torch.equal(a.out.view(torch.int32), b.out.view(torch.int32))
    assert torch.equal(a.token_scores.view(torch.int32), b.token_scores.view(torch.int32))
    assert torch.equal(a.evicted_pos, b.evicted_pos)
    for key in ("slot_pos", "k_dec", "v_dec"):
        assert torch.equal(st_a[key], st_b[key]), key


def test_static_scratch_matches_the_workspace_entry_point(kv):
    big = wl.DecodeShape("big", 16, 32, 8, 128, 4096, 1024, 0, torch.bfloat16)     # the 16-sequence decode shape
    small = wl.DecodeShape("small", 3, 8, 4, 128, 700, 5, 0, torch.bfloat16)
    st_ref, ref = _state(kv, big, 1, 1024)
    st_new, new = _state(kv, big, 1, 1024)
    assert ref.workspace.numel() <= kv.STATIC_SCRATCH_BYTES
    for step in (1024, 1025):                    # pool full: each step appends and evicts
        q, kn, vn = wl.decode_inputs(big, step, "cuda", 1)
        kv.decode_step(ref, step, q, kn, vn)
        new.out.fill_(-1.0)
        kv.decode_step_static(new, step, q, kn, vn)
        torch.cuda.synchronize()
        _same(ref, new, st_ref, st_new)
        assert int(new.evicted_pos.min().item()) >= 0
    # a smaller problem right after: the scratch buffer still holds the larger call's contents
    st_ref2, ref2 = _state(kv, small, 2, 5)
    st_new2, new2 = _state(kv, small, 2, 5)
    for step in range(5, 9):
        q, kn, vn = wl.decode_inputs(small, step, "cuda", 2)
        kv.decode_step(ref2, step, q, kn, vn)
        kv.decode_step_static(new2, step, q, kn, vn)
        torch.cuda.synchronize()
        _same(ref2, new2, st_ref2, st_new2)
    # and the large one again
    q, kn, vn = wl.decode_inputs(big, 1026, "cuda", 1)
    kv.decode_step(ref, 1026, q, kn, vn)
    kv.decode_step_static(new, 1026, q, kn, vn)
    torch.cuda.synchronize()
    _same(ref, new, st_ref, st_new)


def test_static_scratch_rejects_what_does_not_fit(kv):
    """128 sequences x 1025 slots need ~27 MB of scratch: a clear error, nothing enqueued, state untouched."""
    shape = wl.DecodeShape("toolarge", 128, 32, 8, 128, 256, 1024, 0, torch.bfloat16)
    st, state = _state(kv, shape, 3, 0)
    assert state.workspace.numel() > kv.STATIC_SCRATCH_BYTES
    q, kn, vn = wl.decode_inputs(shape, 0, "cuda", 3)
    with pytest.raises(kv.ShotKVError, match="static"):
        kv.decode_step_static(state, 0, q, kn, vn)
    torch.cuda.synchronize()
    assert int((st["slot_pos"] >= 0).sum().item()) == 0
    lib = kv.load_library()
    assert lib.shotkv_strerror(kv.E_SCRATCH).startswith(b"problem needs more scratch")
    rc = lib.shotkv_decode_step_static(ctypes.byref(state.cfg), shape.n_seqs, None, 0, None, None, None, None,
                                       None, None, None, None)
    assert rc == -1
