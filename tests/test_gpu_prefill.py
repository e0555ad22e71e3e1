"""GPU parity: prefill compression through the C ABI against the CPU oracle on the same seeded inputs."""
import math

import numpy as np
import pytest
import torch

import helpers
from helpers import check_prefill_problem, oracle_prefill, to_np
from oracle import shotkv_oracle as orc
from paper_2502_01941_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def kv():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2502_01941_amd import shotkv
    shotkv.load_library()
    return shotkv


def _run_shape(kv, shape, n_problems=None, mode=orc.SELECT_PREFIX, seed=0):
    q, k, v, off, bud = wl.prefill_batch(shape, "cuda", seed=seed, n_problems=n_problems)
    res = kv.prefill_compress(q, k, v, off, bud, shape.budget_tokens, shape.sm_scale, mode)
    torch.cuda.synchronize()
    return q, k, v, off, bud, res


def test_tiny_fp32_full_parity(kv):
    """fp32, D=64, G=1, W=16, 8 shots: every output against the oracle."""
    shape = wl.TINY
    q, k, v, off, bud, res = _run_shape(kv, shape)
    ref = check_prefill_problem(res, 0, q[0], k[0], v[0], off[0].cpu().numpy(), shape.budget_tokens,
                                shape.budget_tokens, shape.sm_scale)
    assert ref["margin"] >= helpers.MARGIN_EXACT
    # tighter than the stated bound: fp32 inputs, 512 keys
    np.testing.assert_allclose(res.shot_scores[0].cpu().numpy(), ref["scores"], rtol=2e-5)


def test_layer8k_bf16_full_parity(kv):
    """One Llama-3-8B-shaped layer, 8192 tokens, 40 shots, budget 40 %."""
    shape = wl.LAYER8K
    q, k, v, off, bud, res = _run_shape(kv, shape)
    report = []
    ref = check_prefill_problem(res, 0, q[0], k[0], v[0], off[0].cpu().numpy(), shape.budget_tokens,
                                shape.budget_tokens, shape.sm_scale, report=report)
    assert not report, report
    # mass conservation on the device's own scores: sum k_i*Score_i <= H*W, the rest sits in the tail
    lengths = np.diff(off[0].cpu().numpy())
    gpu_mass = float((lengths * res.shot_scores[0].cpu().numpy().astype(np.float64)).sum())
    tail_mass = float(ref["mass"][off[0, -1].item():].sum())
    assert abs(gpu_mass + tail_mass - 32 * 32) < 1e-2


def _ragged_problem(P, H, Hkv, D, W, N, dtype, seed, n_shots, prefix, tail_min):
    """Uneven shots with a non-empty prefix, sizes that are not multiples of any tile."""
    g = torch.Generator(device="cuda").manual_seed(seed)
    q = torch.randn((P, H, W, D), generator=g, device="cuda").to(dtype)
    k = torch.randn((P, Hkv, N, D), generator=g, device="cuda").to(dtype)
    v = torch.randn((P, Hkv, N, D), generator=g, device="cuda").to(dtype)
    rng = np.random.default_rng(seed)
    offs = np.zeros((P, n_shots + 1), dtype=np.int32)
    for p in range(P):
        cuts = np.sort(rng.choice(np.arange(prefix + 1, N - tail_min), size=n_shots, replace=False))
        offs[p] = np.concatenate([[prefix], cuts])
    return q, k, v, torch.from_numpy(offs).cuda()


@pytest.mark.parametrize("H,Hkv,D,W,N,dtype,n_shots", [
    (32, 8, 128, 32, 2999, torch.bfloat16, 17),   # the Llama shape, ragged everything
    (8, 2, 128, 32, 1537, torch.bfloat16, 9),     # G=4, fewer heads
    (16, 8, 128, 32, 700, torch.bfloat16, 5),     # G=2 -> 64 rows per KV head
    (8, 8, 128, 32, 650, torch.bfloat16, 4),      # G=1 -> 32 rows
    (16, 4, 128, 16, 900, torch.bfloat16, 6),     # W=16, G=4 -> 64 rows
    (8, 4, 64, 16, 777, torch.float32, 6),        # fp32, D=64
    (4, 4, 128, 8, 300, torch.float32, 3),        # fp32, D=128
    (8, 2, 64, 24, 500, torch.bfloat16, 5),       # bf16, D=64, W not a power of two
    (8, 4, 128, 64, 800, torch.bfloat16, 5),      # the widest window, G=2 -> 128 rows (matrix-core path)
    (8, 2, 128, 64, 600, torch.bfloat16, 4),      # the widest window, G=4 -> 256 rows (eight row blocks on the matrix-core path)
    (64, 8, 128, 32, 450, torch.bfloat16, 3),     # the most query heads, G=8 -> 256 rows
    (4, 4, 128, 1, 200, torch.bfloat16, 3),       # a single window query
    (28, 4, 128, 32, 1100, torch.bfloat16, 6),    # G=7 -> 224 rows, padded to 256 on the matrix-core path
    (40, 8, 128, 32, 900, torch.bfloat16, 5),     # G=5 -> 160 rows
    (12, 4, 128, 32, 800, torch.bfloat16, 5),     # G=3 -> 96 rows
    (24, 4, 128, 20, 700, torch.bfloat16, 4),     # G=6, W=20 -> 120 rows
    (6, 2, 64, 16, 500, torch.float32, 4),        # G=3 on the generic path
    (24, 4, 128, 32, 900, torch.bfloat16, 5),     # G=6 -> 192 rows, six blocks
])
def test_ragged_shapes(kv, H, Hkv, D, W, N, dtype, n_shots):
    P = 3
    q, k, v, off = _ragged_problem(P, H, Hkv, D, W, N, dtype, 1234 + N, n_shots, prefix=7, tail_min=W + 3)
    budgets = torch.tensor([N // 2, N // 3, N], dtype=torch.int32, device="cuda")
    cap = N
    scale = 1.0 / math.sqrt(D)
    res = kv.prefill_compress(q, k, v, off, budgets, cap, scale)
    torch.cuda.synchronize()
    for p in range(P):
        check_prefill_problem(res, p, q[p], k[p], v[p], off[p].cpu().numpy(), budgets[p].item(), cap, scale)


def test_shot_reaching_into_the_window(kv):
    """The last shot may contain window positions: its keys are then causally masked per query row."""
    H, Hkv, D, W, N = 8, 2, 128, 32, 600
    q, k, v, _ = _ragged_problem(1, H, Hkv, D, W, N, torch.bfloat16, 5, 3, 0, 40)
    off = torch.tensor([[0, 200, 410, 590]], dtype=torch.int32, device="cuda")   # window = [568, 600)
    bud = torch.tensor([N], dtype=torch.int32, device="cuda")
    res = kv.prefill_compress(q, k, v, off, bud, N, 0.1)
    torch.cuda.synchronize()
    check_prefill_problem(res, 0, q[0], k[0], v[0], off[0].cpu().numpy(), N, N, 0.1)


@pytest.mark.parametrize("H,Hkv,D,W,dtype", [(8, 2, 128, 32, torch.bfloat16), (4, 4, 64, 16, torch.float32),
                                             (16, 2, 128, 32, torch.bfloat16)])
def test_no_tail_and_a_window_as_long_as_the_prompt(kv, H, Hkv, D, W, dtype):
    """The last shot ends at the last token (nothing after the shots, the window lies inside the last shot),
    and prompts of exactly W and W + 1 tokens (every key row is causally masked for some query)."""
    scale = 1.0 / math.sqrt(D)
    N = 600
    q, k, v, _ = _ragged_problem(2, H, Hkv, D, W, N, dtype, 17, 3, 0, 40)
    off = torch.tensor([[0, 200, 410, N], [5, 90, 300, N]], dtype=torch.int32, device="cuda")
    bud = torch.tensor([N, 420], dtype=torch.int32, device="cuda")
    res = kv.prefill_compress(q, k, v, off, bud, N, scale)
    torch.cuda.synchronize()
    for p in range(2):
        check_prefill_problem(res, p, q[p], k[p], v[p], off[p].cpu().numpy(), bud[p].item(), N, scale)
    assert res.kept_count.cpu().tolist()[0] == N
    for N in (W, W + 1):
        q, k, v, _ = _ragged_problem(2, H, Hkv, D, W, N + 64, dtype, 18 + N, 2, 0, 40)
        k, v = k[:, :, :N].contiguous(), v[:, :, :N].contiguous()
        off = torch.tensor([[0, W // 3, N], [1, W // 2, N - 1]], dtype=torch.int32, device="cuda")
        bud = torch.tensor([N, N - W // 2 + 1], dtype=torch.int32, device="cuda")
        res = kv.prefill_compress(q, k, v, off, bud, N, scale)
        torch.cuda.synchronize()
        for p in range(2):
            check_prefill_problem(res, p, q[p], k[p], v[p], off[p].cpu().numpy(), bud[p].item(), N, scale)
    with pytest.raises(kv.ShotKVError):          # a prompt shorter than the window
        kv.prefill_scores(q, k[:, :, : W - 1].contiguous(), torch.tensor([[0, 3], [0, 3]], dtype=torch.int32, device="cuda"),
                          scale)


def test_degenerate_problems_in_one_batch(kv):
    """Bad offsets, a budget smaller than the always-kept tokens, an exact fit and a zero shot budget,
    side by side with a healthy problem: each gets its own status and the others are unaffected."""
    H, Hkv, D, W, N, n = 8, 2, 128, 32, 1000, 4
    q, k, v, _ = _ragged_problem(5, H, Hkv, D, W, N, torch.bfloat16, 77, n, 0, 40)
    off = np.array([[10, 200, 400, 600, 900],
                    [10, 200, 200, 600, 900],     # not strictly increasing
                    [10, 200, 400, 600, 900],
                    [10, 200, 400, 600, 900],
                    [10, 200, 400, 600, 1001]],   # beyond n_tokens
                   dtype=np.int32)
    budgets = np.array([500, 500, 109, 110, 500], dtype=np.int32)   # always-kept = 10 + 100 = 110
    res = kv.prefill_compress(q, k, v, torch.from_numpy(off).cuda(), torch.from_numpy(budgets).cuda(), 600, 0.09)
    torch.cuda.synchronize()
    assert res.status.cpu().tolist() == [orc.STATUS_OK, orc.STATUS_BAD_OFFSETS, orc.STATUS_BUDGET_TOO_SMALL,
                                         orc.STATUS_OK, orc.STATUS_BAD_OFFSETS]
    for p in range(5):
        check_prefill_problem(res, p, q[p], k[p], v[p], off[p], budgets[p], 600, 0.09)
    assert res.kept_count.cpu().tolist()[3] == 110


def test_no_shots_keeps_everything(kv):
    H, Hkv, D, W, N = 4, 4, 64, 16, 200
    q, k, v, _ = _ragged_problem(2, H, Hkv, D, W, N, torch.float32, 3, 1, 0, 40)
    off = torch.tensor([[50], [0]], dtype=torch.int32, device="cuda")
    bud = torch.tensor([200, 199], dtype=torch.int32, device="cuda")
    res = kv.prefill_compress(q, k, v, off, bud, 256, 0.125)
    torch.cuda.synchronize()
    assert res.status.cpu().tolist() == [orc.STATUS_OK, orc.STATUS_BUDGET_TOO_SMALL]
    assert res.kept_count.cpu().tolist() == [200, 0]
    assert res.kept_positions[0, :200].cpu().tolist() == list(range(200))
    np.testing.assert_array_equal(helpers.bits(res.k_out[0, :, :200]), helpers.bits(k[0]))


def test_uniform_keys_tie_break(kv):
    """All keys identical: all shot scores are (nearly) equal, and with truly equal scores fed to the
    selection half the lowest indices must win."""
    H, Hkv, D, W, N, n = 8, 2, 128, 32, 1200, 10
    g = torch.Generator(device="cuda").manual_seed(11)
    q = torch.randn((1, H, W, D), generator=g, device="cuda").to(torch.bfloat16)
    k = torch.randn((1, 1, 1, D), generator=g, device="cuda").to(torch.bfloat16).expand(1, Hkv, N, D).contiguous()
    v = torch.randn((1, Hkv, N, D), generator=g, device="cuda").to(torch.bfloat16)
    off = torch.arange(0, 1001, 100, dtype=torch.int32, device="cuda")[None]
    bud = torch.tensor([200 + 350], dtype=torch.int32, device="cuda")
    scores, status = kv.prefill_scores(q, k, off, 0.2)
    torch.cuda.synchronize()
    expect = H * sum(1.0 / (N - W + j + 1) for j in range(W))   # closed form for uniform attention
    np.testing.assert_allclose(scores[0].cpu().numpy(), expect, rtol=1e-5)
    equal = torch.full((1, n), float(expect), dtype=torch.float32, device="cuda")
    res = kv.select_and_compact(equal, k, v, off, bud, 600, H, W)
    torch.cuda.synchronize()
    assert res.shot_selected[0].cpu().tolist() == [1, 1, 1] + [0] * 7


@pytest.mark.parametrize("mode", [orc.SELECT_PREFIX, orc.SELECT_FIRST_FIT])
def test_select_and_compact_synthetic_scores(kv, mode):
    """The selection/compaction half on generator-made scores (with ties, -inf free): bit-exact against
    the oracle's selection on the same scores, for many problems at once."""
    P, H, Hkv, D, W, N, n = 64, 8, 2, 128, 32, 3000, 37
    rng = np.random.default_rng(2024 + mode)
    _, k, v, off = _ragged_problem(P, H, Hkv, D, W, N, torch.bfloat16, 99, n, 5, 50)
    scores = rng.standard_normal((P, n)).astype(np.float32)
    scores[::3] = np.round(scores[::3] * 2) / 2                     # heavy ties
    budgets = rng.integers(50, N, size=P).astype(np.int32)
    cap = 2048                                                      # some budgets get clamped to cap
    res = kv.select_and_compact(torch.from_numpy(scores).cuda(), k, v, off, torch.from_numpy(budgets).cuda(),
                                cap, H, W, mode)
    torch.cuda.synchronize()
    offs = off.cpu().numpy()
    for p in range(P):
        b = min(int(budgets[p]), cap)
        lengths = np.diff(offs[p])
        n_always = int(offs[p, 0]) + N - int(offs[p, -1])
        if b - n_always < 0:
            assert res.status[p].item() == orc.STATUS_BUDGET_TOO_SMALL and res.kept_count[p].item() == 0
            continue
        keep = orc.select_shots(scores[p], lengths, b - n_always, mode)
        assert res.status[p].item() == orc.STATUS_OK
        assert res.shot_selected[p].cpu().numpy().tolist() == keep.tolist(), p
        pos = orc.kept_positions_from_mask(keep, offs[p], N)
        kept = res.kept_count[p].item()
        assert kept == pos.size
        np.testing.assert_array_equal(res.kept_positions[p, :kept].cpu().numpy(), pos)
        idx = torch.from_numpy(pos).long().cuda()
        np.testing.assert_array_equal(helpers.bits(res.k_out[p, :, :kept]), helpers.bits(k[p][:, idx]))
        np.testing.assert_array_equal(helpers.bits(res.v_out[p, :, :kept]), helpers.bits(v[p][:, idx]))


@pytest.mark.parametrize("n", [1, 2, 63, 64, 65, 127, 129, 1000, 1023, 1024, 1025, 2047, 2049, 4095, 4096])
def test_ranking_sizes_and_special_scores(kv, n):
    """The ranking at every size class of the sorting network (one, two and four keys per thread; with and
    without the transposed passes; padding of 0..n_pad-1 entries), on scores with heavy ties, both zeros,
    negative values, infinities and denormals: selection and positions bit-exact against the oracle."""
    P, H, Hkv, D, W = 4, 2, 1, 128, 8
    N = 3 * n + 300
    _, k, v, off = _ragged_problem(P, H, Hkv, D, W, N, torch.bfloat16, 500 + n, n, 2, 40)
    rng = np.random.default_rng(900 + n)
    scores = rng.standard_normal((P, n)).astype(np.float32)
    scores[1] = np.round(scores[1] * 2) / 2                          # heavy ties, +0.0 and -0.0 among them
    scores[2] = rng.choice(np.array([0.0, -0.0, 1.0, -1.0, np.inf, -np.inf, 1e-42, -1e-42, 3.5],
                                    dtype=np.float32), size=n)
    scores[3] = -np.abs(scores[3])                                   # all negative
    offs = off.cpu().numpy()
    always = offs[:, 0] + N - offs[:, -1]                            # tokens outside every shot
    in_shots = offs[:, -1] - offs[:, 0]
    budgets = (always + in_shots // np.array([2, 3, 2, 1])).astype(np.int32)
    for mode in (orc.SELECT_PREFIX, orc.SELECT_FIRST_FIT):
        res = kv.select_and_compact(torch.from_numpy(scores).cuda(), k, v, off, torch.from_numpy(budgets).cuda(),
                                    N, H, W, mode)
        torch.cuda.synchronize()
        assert res.status.cpu().tolist() == [orc.STATUS_OK] * P
        for p in range(P):
            n_always = int(offs[p, 0]) + N - int(offs[p, -1])
            keep = orc.select_shots(scores[p], np.diff(offs[p]), int(budgets[p]) - n_always, mode)
            assert res.shot_selected[p].cpu().numpy().tolist() == keep.tolist(), (mode, p)
            pos = orc.kept_positions_from_mask(keep, offs[p], N)
            kept = res.kept_count[p].item()
            np.testing.assert_array_equal(res.kept_positions[p, :kept].cpu().numpy(), pos)
            idx = torch.from_numpy(pos).long().cuda()
            np.testing.assert_array_equal(helpers.bits(res.k_out[p, :, :kept]), helpers.bits(k[p][:, idx]))


def test_many_shots_selection(kv):
    """Sentence-sized units: thousands of short spans stress the sort, the scans and the copy plan."""
    P, H, Hkv, D, W, N, n = 2, 8, 2, 128, 32, 40000, 3000
    _, k, v, off = _ragged_problem(P, H, Hkv, D, W, N, torch.bfloat16, 31, n, 3, 100)
    rng = np.random.default_rng(8)
    scores = rng.standard_normal((P, n)).astype(np.float32)
    budgets = np.array([N // 10, N // 2], dtype=np.int32)
    res = kv.select_and_compact(torch.from_numpy(scores).cuda(), k, v, off, torch.from_numpy(budgets).cuda(),
                                N // 2, H, W)
    torch.cuda.synchronize()
    offs = off.cpu().numpy()
    for p in range(P):
        n_always = int(offs[p, 0]) + N - int(offs[p, -1])
        keep = orc.select_shots(scores[p], np.diff(offs[p]), int(budgets[p]) - n_always)
        assert res.shot_selected[p].cpu().numpy().tolist() == keep.tolist()
        pos = orc.kept_positions_from_mask(keep, offs[p], N)
        kept = res.kept_count[p].item()
        np.testing.assert_array_equal(res.kept_positions[p, :kept].cpu().numpy(), pos)
        idx = torch.from_numpy(pos).long().cuda()
        np.testing.assert_array_equal(helpers.bits(res.v_out[p, :, :kept]), helpers.bits(v[p][:, idx]))


def test_maximum_number_of_shots_end_to_end(kv):
    """SHOTKV_MAX_SHOTS units of 5-13 tokens through the whole path: every unit is a chunk of its own."""
    P, H, Hkv, D, W, N, n = 1, 8, 2, 128, 32, 37000, 4096
    g = torch.Generator(device="cuda").manual_seed(77)
    q = torch.randn((P, H, W, D), generator=g, device="cuda").to(torch.bfloat16)
    k = torch.randn((P, Hkv, N, D), generator=g, device="cuda").to(torch.bfloat16)
    v = torch.randn((P, Hkv, N, D), generator=g, device="cuda").to(torch.bfloat16)
    rng = np.random.default_rng(77)
    off = np.concatenate([[11], 11 + np.cumsum(rng.integers(5, 14, size=n))]).astype(np.int32)
    assert off[-1] < N - W
    offs = torch.from_numpy(off[None]).cuda()
    budget = N // 4
    bud = torch.tensor([budget], dtype=torch.int32, device="cuda")
    res = kv.prefill_compress(q, k, v, offs, bud, budget, 1.0 / math.sqrt(D))
    torch.cuda.synchronize()
    check_prefill_problem(res, 0, q[0], k[0], v[0], off, budget, budget, 1.0 / math.sqrt(D))
    with pytest.raises(kv.ShotKVError):          # one more shot than the library takes
        kv.prefill_scores(q, k, torch.zeros((1, n + 2), dtype=torch.int32, device="cuda"), 0.1)


def test_one_million_tokens(kv):
    """A context of 2^20 + 37 tokens with the largest number of shots (lengths 1 to ~2500): row offsets past
    2^28 bytes inside a plane, a thousand score workgroups per KV head, eight thousand chunks, a copy plan of
    350 K positions."""
    P, H, Hkv, D, W, n = 1, 4, 1, 128, 32, 4096
    N = (1 << 20) + 37
    q, k, v, off = _ragged_problem(P, H, Hkv, D, W, N, torch.bfloat16, 991, n, prefix=3, tail_min=W + 500)
    budget = N // 3
    bud = torch.tensor([budget], dtype=torch.int32, device="cuda")
    scale = 1.0 / math.sqrt(D)
    res = kv.prefill_compress(q, k, v, off, bud, budget, scale)
    torch.cuda.synchronize()
    report = []
    check_prefill_problem(res, 0, q[0], k[0], v[0], off[0].cpu().numpy(), budget, budget, scale, report=report)
    print("near ties:", report)


@pytest.mark.parametrize("H,Hkv", [(8, 2), (4, 2), (2, 2), (12, 2), (16, 2)])
def test_units_of_one_to_three_tokens(kv, H, Hkv):
    """Units of one to three tokens: up to thirty-two chunk boundaries inside one 32-key block, at every
    element position of both lane halves, for one to four query blocks per wave (G = 4, 2, 1, 6, 8)."""
    P, D, W, N, n = 2, 128, 32, 2100, 1000
    g = torch.Generator(device="cuda").manual_seed(4242 + H)
    q = torch.randn((P, H, W, D), generator=g, device="cuda").to(torch.bfloat16)
    k = torch.randn((P, Hkv, N, D), generator=g, device="cuda").to(torch.bfloat16)
    v = torch.randn((P, Hkv, N, D), generator=g, device="cuda").to(torch.bfloat16)
    rng = np.random.default_rng(4242 + H)
    off = np.stack([np.concatenate([[s0], s0 + np.cumsum(rng.integers(1, 4, size=n))]).astype(np.int32)
                    for s0 in (0, 5)])
    assert off.max() < N - W
    budget = N // 3
    bud = torch.full((P,), budget, dtype=torch.int32, device="cuda")
    scale = 1.0 / math.sqrt(D)
    res = kv.prefill_compress(q, k, v, torch.from_numpy(off).cuda(), bud, budget, scale)
    torch.cuda.synchronize()
    for p in range(P):
        check_prefill_problem(res, p, q[p], k[p], v[p], off[p], budget, budget, scale)


def test_inputs_are_not_modified_and_runs_repeat_bitwise(kv):
    shape = wl.LAYER8K
    q, k, v, off, bud = wl.prefill_batch(shape, "cuda")
    k0, v0, q0 = k.clone(), v.clone(), q.clone()
    a = kv.prefill_compress(q, k, v, off, bud, shape.budget_tokens, shape.sm_scale)
    b = kv.prefill_compress(q, k, v, off, bud, shape.budget_tokens, shape.sm_scale)
    torch.cuda.synchronize()
    assert torch.equal(k, k0) and torch.equal(v, v0) and torch.equal(q, q0)
    assert torch.equal(a.shot_scores, b.shot_scores)              # fixed summation order: no atomics
    assert torch.equal(a.kept_positions[:, : a.kept_count[0]], b.kept_positions[:, : b.kept_count[0]])


def test_host_side_errors(kv):
    q = torch.zeros((1, 8, 32, 128), dtype=torch.bfloat16, device="cuda")
    k = torch.zeros((1, 2, 100, 128), dtype=torch.bfloat16, device="cuda")
    off = torch.tensor([[0, 10]], dtype=torch.int32, device="cuda")
    bud = torch.tensor([50], dtype=torch.int32, device="cuda")
    small = torch.empty(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(kv.ShotKVError, match="workspace"):
        kv.prefill_compress(q, k, k, off, bud, 64, 0.1, workspace=small)
    with pytest.raises(kv.ShotKVError, match="shape"):                 # window longer than the prompt
        kv.prefill_compress(q, k[:, :, :20].contiguous(), k[:, :, :20].contiguous(), off, bud, 64, 0.1)
    with pytest.raises(kv.ShotKVError, match="aligned"):
        ws = torch.empty(kv.prefill_workspace_bytes(8, 2, 128, 32, torch.bfloat16, 1, 100, 1) + 16,
                         dtype=torch.uint8, device="cuda")
        kv.prefill_compress(q, k, k, off, bud, 64, 0.1, workspace=ws[8:])


def test_logits_far_above_the_running_reference(kv):
    """Inside one shot the first 32 keys are small and a later block holds keys whose logits exceed the
    reference found so far by more than 2^100: the score kernel must fall back to the exact online
    update there (and must not overflow)."""
    H, Hkv, D, W, N = 32, 8, 128, 32, 1024
    g = torch.Generator(device="cuda").manual_seed(21)
    u = torch.zeros(D, device="cuda"); u[:4] = 0.5                       # unit vector
    q = (4.0 * u).expand(1, H, W, D).contiguous().to(torch.bfloat16)
    k = (0.01 * torch.randn((1, Hkv, N, D), generator=g, device="cuda")).to(torch.bfloat16)
    k[:, :, 300:340, :] = (30.0 * u).to(torch.bfloat16)                   # logits 120 with sm_scale 1
    k[:, :, 700:705, :] = (31.0 * u).to(torch.bfloat16)                   # and a still larger, later group
    v = torch.zeros_like(k)
    off = torch.tensor([[0, 256, 512, 768, 960]], dtype=torch.int32, device="cuda")
    scores, status = kv.prefill_scores(q, k, off, 1.0)
    torch.cuda.synchronize()
    assert status.cpu().tolist() == [0]
    ref = oracle_prefill(q[0], k[0], v[0], off[0].cpu().numpy(), N, 1.0)
    got = scores[0].cpu().numpy()
    assert np.all(np.isfinite(got))
    np.testing.assert_allclose(got, ref["scores"], rtol=1e-3, atol=1e-30)
    assert got[2] > 1.0 and got[0] < 1e-20                                 # the mass sits in shot 2


def test_reference_carried_across_chunks_with_opposed_rows(kv):
    """Half of the query rows point along +u, half along -u, and consecutive short shots alternate
    between keys along +u and -u.  For every row the softmax reference it carries from one shot to the
    next is alternately far above the next shot's logits (their terms nearly vanish against it) and far
    below them (the update must fall back to the exact rescale).  Short shots make every 32-key block a
    chunk of its own."""
    H, Hkv, D, W, N = 32, 8, 128, 32, 2048
    g = torch.Generator(device="cuda").manual_seed(22)
    u = torch.zeros(D, device="cuda"); u[:4] = 0.5
    sign = torch.where(torch.arange(W, device="cuda") % 2 == 0, 1.0, -1.0)
    q = (4.0 * sign[None, None, :, None] * u).expand(1, H, W, D).contiguous().to(torch.bfloat16)
    bounds = list(range(0, 1921, 24))                                      # 80 shots of 24 tokens
    off = torch.tensor([bounds], dtype=torch.int32, device="cuda")
    k = (0.05 * torch.randn((1, Hkv, N, D), generator=g, device="cuda"))
    for i in range(len(bounds) - 1):
        k[:, :, bounds[i]:bounds[i + 1], :] += (20.0 if i % 2 == 0 else -20.0) * (1 + 0.01 * i) * u
    k = k.to(torch.bfloat16)
    v = torch.zeros_like(k)
    scores, status = kv.prefill_scores(q, k, off, 1.0)
    torch.cuda.synchronize()
    assert status.cpu().tolist() == [0]
    ref = oracle_prefill(q[0], k[0], v[0], off[0].cpu().numpy(), N, 1.0)
    got = scores[0].cpu().numpy()
    assert np.all(np.isfinite(got))
    np.testing.assert_allclose(got, ref["scores"], rtol=1e-3, atol=1e-30)
    assert got[-1] > 1.0 and got[-2] > 1.0                                 # the last +u and -u shots dominate
