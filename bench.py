"""Benchmark of the ShotKV hot path on one MI355X.

A step = one pass of the whole hot path over one batch of synthetic input: prefill compression (chunk
plan, window-attention scores, per-shot reduction, selection, K/V compaction) of all 128 (layer, batch)
problems of the 32-layer x batch-4 x 32K-token Llama-3-8B-shaped workload, followed by one decode step
(attention over the compressed caches + token retention) for the same 128 (layer, sequence) caches.
Inputs are resident in HBM before the timed region.  The timed region carries no instrumentation; kernel
durations come from a separate pass of the same steps bracketed by caller-owned HIP events.  Prints ONE
JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload model32k]
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0      # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0

# HBM bytes the score kernel moved per launch (FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0 from two
# `rocprofv3 --pmc` runs of this file, see profiles/score_partials_mfma_model32k_counters.md).  Valid only
# for the kernel source it was measured on: reported as null once that file's hash differs.
SCORE_KERNEL_SOURCE = os.path.join(ROOT, "paper_2502_01941_amd", "csrc", "prefill_score_mfma.hip")
MEASURED_TRAFFIC = {"model32k": {"sha256": "864e57a17e23b5707280de8a5e16578af9d20837ac6324b9182bbe9136777c50",
                                 "bytes": 8.96e9}}

PREFILL_KINDS = ("plan", "score", "row_stats", "chunk_mass", "reduce_select", "compact")


def _measured_traffic(workload):
    rec = MEASURED_TRAFFIC.get(workload)
    if rec is None or not rec["sha256"]:
        return None
    with open(SCORE_KERNEL_SOURCE, "rb") as fh:
        if hashlib.sha256(fh.read()).hexdigest() != rec["sha256"]:
            return None
    return rec["bytes"]


def _kvb(shape):
    esize = 2 if str(shape.dtype).endswith("bfloat16") else 4
    return shape.n_kv_heads * shape.head_dim * esize


def _timed(torch, fn, iters, warm):
    """Average milliseconds of fn() over `iters` back-to-back calls on the current stream."""
    for i in range(warm):
        fn(i)
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    start.record()
    for i in range(iters):
        fn(warm + i)
    stop.record()
    torch.cuda.synchronize()
    return start.elapsed_time(stop) / iters


def _cpu_info():
    model = ""
    try:
        with open("/proc/cpuinfo") as fh:
            for line in fh:
                if line.startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    try:
        nproc = len(os.sched_getaffinity(0))
    except AttributeError:
        nproc = os.cpu_count() or 1
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:  # pragma: no cover
        threads = nproc
    return model, nproc, int(threads)


def _host(t):
    import torch
    return (t.float() if t.dtype == torch.bfloat16 else t).cpu().numpy()


def cpu_prefill_leg(shape, q, k, v, off, budget_s=12.0):
    """The CPU oracle as it stands on the first problems of the workload, on the bits the GPU run used (the
    device tensors copied to the host problem by problem).  Returns (problems done, seconds)."""
    from oracle import shotkv_oracle as orc
    total, done = 0.0, 0
    for p in range(shape.n_problems):
        qn, kn, vn, on = _host(q[p]), _host(k[p]), _host(v[p]), off[p].cpu().numpy()
        t0 = time.perf_counter()
        orc.prefill_compress(qn, kn, vn, on, shape.budget_tokens, shape.sm_scale)
        total += time.perf_counter() - t0
        done += 1
        if total > budget_s:
            break
    return done, total


def cpu_decode_leg(shp, st, inputs, budget_s=8.0):
    """Steady-state oracle decode steps (the pool is full: every step evicts) on the first sequences of a
    decode state, as the GPU run left it.  Returns (sequence-steps done, seconds)."""
    import numpy as np
    from oracle import shotkv_oracle as orc
    qs, ks, vs = inputs
    total, done = 0.0, 0
    for s in range(shp.n_seqs):
        kp, vp = _host(st["k_prefill"][s]).astype(np.float64), _host(st["v_prefill"][s]).astype(np.float64)
        kd, vd = _host(st["k_dec"][s]).copy(), _host(st["v_dec"][s]).copy()
        sp = st["slot_pos"][s].cpu().numpy().copy()
        qn, kn, vn = _host(qs[s]), _host(ks[s]), _host(vs[s])
        for step in range(4):
            t0 = time.perf_counter()
            r = orc.decode_step(kp, vp, int(st["prefill_count"][s]), kd, vd, sp, shp.decode_budget,
                                10 ** 6 + step, qn, kn, vn, shp.sm_scale)
            total += time.perf_counter() - t0
            assert r["status"] == 0
            done += 1
        if total > budget_s:
            break
    return done, total


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="model32k")
    ap.add_argument("--decode-steps", type=int, default=200)
    ap.add_argument("--kernel-steps", type=int, default=10, help="steps of the separate per-kernel timing pass")
    ap.add_argument("--kernel-warmup", type=int, default=5,
                    help="untimed steps at the start of that pass (the host-side pause before it lets the clocks "
                         "rise, and the first launches after a pause run into the power limit harder)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the other workloads and the decode legs")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (known traffic) for scaling profiler byte counters")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py measures one GPU's throughput; the library has no multi-GPU path (run with --gpus 1)",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2502_01941_amd import shotkv, workloads as wl

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    shotkv.load_library()
    torch.cuda.set_device(0)
    shape = wl.PREFILL_SHAPES[args.workload]
    seed = 0
    P, N, n, cap = shape.n_problems, shape.n_tokens, shape.n_shots, shape.budget_tokens
    kvb = _kvb(shape)

    def prefill_buffers(shp, k):
        ws = torch.empty(shotkv.prefill_workspace_bytes(shp.n_q_heads, shp.n_kv_heads, shp.head_dim, shp.window,
                                                        shp.dtype, shp.n_problems, shp.n_tokens, shp.n_shots,
                                                        shp.sm_scale), dtype=torch.uint8, device="cuda")
        out = shotkv._alloc_prefill_outputs(k, shp.n_problems, shp.n_kv_heads, shp.budget_tokens, shp.head_dim,
                                            shp.n_shots)
        return ws, out

    # ---- resident inputs and caller-owned buffers -------------------------------------------------
    q, k, v, off, bud = wl.prefill_batch(shape, "cuda", seed)
    ws, out = prefill_buffers(shape, k)
    dec_budget, n_slots = 1024, 1025
    k_dec = torch.zeros((P, shape.n_kv_heads, n_slots, shape.head_dim), dtype=shape.dtype, device="cuda")
    v_dec = torch.zeros_like(k_dec)
    slot_pos = torch.full((P, n_slots), -1, dtype=torch.int32, device="cuda")
    dstate = shotkv.DecodeState(out.k_out, out.v_out, out.kept_count, k_dec, v_dec, slot_pos, dec_budget,
                                shape.n_q_heads, shape.sm_scale)
    dshape = wl.DecodeShape("bench", P, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, cap, dec_budget,
                            0, shape.dtype)
    qn, kn, vn = wl.decode_inputs(dshape, 0, "cuda", seed)

    def prefill(i):
        shotkv.prefill_compress(q, k, v, off, bud, cap, shape.sm_scale, out=out, workspace=ws)

    def step(i):
        prefill(i)
        shotkv.decode_step(dstate, i, qn, kn, vn, want_scores=False)

    # ---- the timed region: W warm-up steps, then exactly K steps, nothing else on the stream --------
    ms_per_step = _timed(torch, step, args.steps, args.warmup)
    steps_done = args.warmup + args.steps
    assert int(out.status.abs().sum().item()) == 0 and int(dstate.status.abs().sum().item()) == 0
    kept_total = int(out.kept_count.sum().item())

    # ---- kernel durations: a separate pass of the same step, each kernel between caller-owned events
    timers = shotkv.KernelTimers()
    kinds = PREFILL_KINDS + ("decode_partial", "decode_finish")
    seen = {x: [] for x in kinds}
    with timers:
        for i in range(args.kernel_warmup + args.kernel_steps):
            step(steps_done + i)
            for x, ms in timers.read(kinds).items():
                if i >= args.kernel_warmup:
                    seen[x].append(ms)
    steps_done += args.kernel_warmup + args.kernel_steps
    kernels = {x: {"avg_ms": sum(seen[x]) / args.kernel_steps, "median_ms": statistics.median(seen[x]),
                   "min_ms": min(seen[x]), "launches": args.kernel_steps} for x in kinds}
    prefill_ms = _timed(torch, prefill, args.steps, 2)          # prefill compression alone, uninstrumented

    score_bytes = P * N * kvb                                   # K read once per launch
    compact_bytes = 4 * kept_total * kvb                        # K and V, read + write
    dec_tokens = kept_total + P * steps_done                    # live rows read by the last decode step
    kernels["score"]["algorithmic_gbps"] = score_bytes / kernels["score"]["avg_ms"] / 1e6
    kernels["compact"]["algorithmic_gbps"] = compact_bytes / kernels["compact"]["avg_ms"] / 1e6
    kernels["decode_partial"]["algorithmic_gbps"] = 2 * dec_tokens * kvb / kernels["decode_partial"]["avg_ms"] / 1e6
    algo_bytes_prefill = score_bytes + compact_bytes
    achieved = kernels["score"]["algorithmic_gbps"]
    result = {
        "metric": "prefill-compress tokens/s per layer (a step = prefill compression + 1 decode step)",
        "value": P * N / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if kvb == shape.n_kv_heads * shape.head_dim * 2 else "f32",
        "data": "synthetic",
        "config": {"workload": f"{shape.name}: {P} (layer,batch) problems x {N} tokens, {n} shots, "
                               f"{shape.n_q_heads}q/{shape.n_kv_heads}kv heads, head_dim {shape.head_dim}, "
                               f"window {shape.window}, budget {cap}; then 1 decode step over the "
                               f"{P} compressed caches",
                   "tokens_per_step": P * N, "kept_tokens": kept_total},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": _measured_traffic(shape.name),
                     "kernel": "score_partials_mfma_kernel", "algorithmic_bytes": score_bytes,
                     "timing": f"HIP events around the kernel in a separate pass of {args.kernel_steps} steps "
                               f"after {args.kernel_warmup} untimed ones"},
        "prefill": {"ms": prefill_ms, "tokens_per_s_per_layer": P * N / (prefill_ms * 1e-3),
                    "algorithmic_gbps": algo_bytes_prefill / prefill_ms / 1e6,
                    "hbm_frac": algo_bytes_prefill / prefill_ms / 1e6 / HBM_PEAK_GBPS,
                    "timing": f"{args.steps} uninstrumented prefill compressions back to back"},
        "kernels": kernels,
    }

    cpu_prefill = cpu_prefill_leg(shape, q, k, v, off) if not args.no_cpu_baseline else None
    del q, k, v, out, dstate, k_dec, v_dec, ws
    torch.cuda.empty_cache()

    # ---- decode step at the long-generation shape (16 sequences, 4096 + 1024 tokens) -------------
    d4 = wl.DECODE4K
    decode_cpu = None
    if not args.no_extras:
        def decode_leg(shp, iters, with_cpu=False):
            st = wl.decode_state(shp, "cuda", seed, resident=shp.decode_budget)
            state = shotkv.DecodeState(st["k_prefill"], st["v_prefill"], st["prefill_count"], st["k_dec"],
                                       st["v_dec"], st["slot_pos"], shp.decode_budget, shp.n_q_heads, shp.sm_scale)
            qs, ks, vs = wl.decode_inputs(shp, 0, "cuda", seed)
            us = _timed(torch, lambda i: shotkv.decode_step(state, shp.decode_budget + i, qs, ks, vs), iters, 20) * 1e3
            assert int(state.status.abs().sum().item()) == 0
            dbytes = shp.n_seqs * (shp.prefill_count + shp.decode_budget + 1) * 2 * _kvb(shp)
            cpu = cpu_decode_leg(shp, st, (qs, ks, vs)) if with_cpu else None
            return us, dbytes, cpu

        us, dbytes, decode_cpu = decode_leg(d4, args.decode_steps, not args.no_cpu_baseline)
        result["decode"] = {"workload": "decode4k: 16 sequences x (4096 prefill + 1024 decode) tokens, "
                                        "eviction every step", "step_us": us,
                            "algorithmic_gbps": dbytes / us / 1e3, "hbm_frac": dbytes / us / 1e3 / HBM_PEAK_GBPS,
                            "steps": args.decode_steps}
        d32 = wl.DecodeShape("decode4k_x32", 512, d4.n_q_heads, d4.n_kv_heads, d4.head_dim, d4.prefill_count,
                             d4.decode_budget, 0, d4.dtype)
        us32, dbytes32, _ = decode_leg(d32, 30)
        result["decode_32_layers"] = {"workload": "32 layers x 16 sequences of decode4k in one call (512 caches)",
                                      "step_us": us32, "us_per_layer": us32 / 32,
                                      "algorithmic_gbps": dbytes32 / us32 / 1e3,
                                      "hbm_frac": dbytes32 / us32 / 1e3 / HBM_PEAK_GBPS}
        torch.cuda.empty_cache()

        # ---- prefill compression alone on the other workload shapes ---------------------------------
        others = {}
        for name in ("layer8k", "skew128k", "sentences32k"):
            shp = wl.PREFILL_SHAPES[name]
            q2, k2, v2, off2, bud2 = wl.prefill_batch(shp, "cuda", seed)
            ws2, out2 = prefill_buffers(shp, k2)
            ms = _timed(torch, lambda i: shotkv.prefill_compress(q2, k2, v2, off2, bud2, shp.budget_tokens,
                                                                 shp.sm_scale, out=out2, workspace=ws2), 20, 3)
            kept2 = int(out2.kept_count.sum().item())
            assert int(out2.status.abs().sum().item()) == 0
            b = shp.n_problems * shp.n_tokens * _kvb(shp) + 4 * kept2 * _kvb(shp)
            others[name] = {"problems": shp.n_problems, "tokens": shp.n_tokens, "units": shp.n_shots,
                            "prefill_ms": ms, "tokens_per_s_per_layer": shp.n_problems * shp.n_tokens / (ms * 1e-3),
                            "algorithmic_gbps": b / ms / 1e6, "hbm_frac": b / ms / 1e6 / HBM_PEAK_GBPS}
            if name == "layer8k":
                # the same layer through the entry point that fuses scoring into the causal attention pass
                qa = torch.stack([wl.prefill_all_queries(shp, 0, q2[0], "cuda", seed)])
                attn = torch.empty((1, shp.n_q_heads, shp.n_tokens, shp.head_dim), dtype=torch.float32, device="cuda")
                ms_a = _timed(torch, lambda i: shotkv.prefill_attention_compress(
                    qa, k2, v2, off2, bud2, shp.budget_tokens, shp.window, shp.sm_scale, out=out2, attn_out=attn), 10, 2)
                flops = 4.0 * shp.n_tokens * shp.n_tokens / 2 * shp.head_dim * shp.n_q_heads
                others["layer8k_fused_attention"] = {
                    "ms": ms_a, "causal_tflops": flops / ms_a / 1e9,
                    "mfma_frac": flops / ms_a / 1e9 / MFMA_BF16_PEAK_TFLOPS,
                    "note": "causal attention forward (4*N^2/2*D*H flop) + Eq. 3 scores + selection + compaction; "
                            "saves the separate 2048*N-byte read of K per problem"}
                del qa, attn
            del q2, k2, v2, ws2, out2
            torch.cuda.empty_cache()
        # the fused entry point once more at 32K tokens (one problem of the model32k shape)
        shp = wl.PREFILL_SHAPES["model32k"]
        one = wl.PrefillShape("attn32k", 1, shp.n_q_heads, shp.n_kv_heads, shp.head_dim, shp.window, shp.n_tokens,
                              shp.n_shots, shp.dtype, shp.budget_tokens, tail_tokens=512)
        q2, k2, v2, off2, bud2 = wl.prefill_batch(one, "cuda", seed)
        _, out2 = prefill_buffers(one, k2)
        qa = torch.stack([wl.prefill_all_queries(one, 0, q2[0], "cuda", seed)])
        attn = torch.empty((1, one.n_q_heads, one.n_tokens, one.head_dim), dtype=torch.float32, device="cuda")
        ms_a = _timed(torch, lambda i: shotkv.prefill_attention_compress(
            qa, k2, v2, off2, bud2, one.budget_tokens, one.window, one.sm_scale, out=out2, attn_out=attn), 5, 2)
        flops = 4.0 * one.n_tokens * one.n_tokens / 2 * one.head_dim * one.n_q_heads
        others["attn32k_fused_attention"] = {"ms": ms_a, "causal_tflops": flops / ms_a / 1e9,
                                             "mfma_frac": flops / ms_a / 1e9 / MFMA_BF16_PEAK_TFLOPS}
        del qa, attn, q2, k2, v2, out2
        torch.cuda.empty_cache()
        result["other_workloads"] = others
        result["generic_paths"] = "fp32 / head_dim 64 inputs take untuned vector-ALU kernels (tests only; not measured here)"

    # What a plain streaming kernel reaches on this machine: torch's elementwise int32 x + 1 over 1 GiB (reads
    # 1 GiB, writes 1 GiB).  Context for the roofline fractions, and with --calibrate-copy the kernel of
    # known traffic that the profiler's byte counters are scaled by.
    src = torch.zeros(1 << 28, dtype=torch.int32, device="cuda")
    dst = torch.empty_like(src)
    copy_ms = _timed(torch, lambda i: torch.add(src, 1, out=dst), 10, 3)
    copy_gbps = 2 * (1 << 30) / (copy_ms * 1e-3) / 1e9
    result["achievable"] = {"copy_read_plus_write_gbps": copy_gbps, "kernel": "torch int32 add-scalar, 1 GiB in, 1 GiB out"}
    result["roofline"]["frac_of_copy"] = result["roofline"]["achieved"] / copy_gbps
    if args.calibrate_copy:
        result["calibration_kernel"] = {"op": "int32 add-scalar", "read_bytes": 1 << 30, "write_bytes": 1 << 30}
    del src, dst

    if not args.no_cpu_baseline:
        model, nproc, threads = _cpu_info()
        done, total = cpu_prefill
        base = {"value": done * shape.n_tokens / total, "unit": "tokens/s", "cores": threads, "kind": "oracle",
                "sample": f"prefill compression of the first {done} of {shape.n_problems} problems of {shape.name} "
                          f"(numpy float64, {total:.1f} s, on the device tensors copied to the host)",
                "nproc": nproc, "cpu_model": model, "blas_threads": threads}
        if decode_cpu is not None:
            d_done, d_total = decode_cpu
            base["decode_step_us_per_layer"] = d_total / d_done * d4.n_seqs * 1e6
            base["sample"] += (f"; decode leg: {d_done} steady-state sequence-steps of {d4.name} in {d_total:.1f} s, "
                               f"scaled to one step of all {d4.n_seqs} sequences")
        result["cpu_baseline"] = base
    print(json.dumps(result))


if __name__ == "__main__":
    main()
