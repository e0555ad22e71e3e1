"""Thin ctypes binding over libshotkv.so (the C ABI declared in include/shotkv.h).

Argument marshalling only: every step of the method runs in the library's HIP kernels.  PyTorch is
used for device memory and for the current HIP stream.  There is no fallback: if the library has not
been built (python -m paper_2502_01941_amd.build) loading fails with an error.
"""
from __future__ import annotations

import ctypes
import dataclasses
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# SHOTKV_LIBRARY overrides the path (e.g. to load a differently tuned build of the same sources)
LIB_PATH = os.environ.get("SHOTKV_LIBRARY") or os.path.join(_HERE, "libshotkv.so")

BF16, F32 = 0, 1
SELECT_PREFIX, SELECT_FIRST_FIT = 0, 1
HEADS_PER_LAYER, HEADS_PER_KV_HEAD = 0, 1
ST_OK, ST_BAD_OFFSETS, ST_BUDGET_TOO_SMALL, ST_NO_FREE_SLOT = 0, -1, -2, -3
INT32_MAX = 2 ** 31 - 1
E_SCRATCH = -6
STATIC_SCRATCH_BYTES = 8 << 20

EXPORTS = (
    "shotkv_strerror", "shotkv_abi_version", "shotkv_prefill_workspace_bytes",
    "shotkv_prefill_compress", "shotkv_prefill_scores", "shotkv_select_and_compact",
    "shotkv_prefill_attention_workspace_bytes", "shotkv_prefill_attention_compress",
    "shotkv_decode_workspace_bytes", "shotkv_decode_step", "shotkv_decode_step_static",
)

KERNEL_KINDS = ("plan", "score", "row_stats", "chunk_mass", "reduce_select", "compact",
                "decode_partial", "decode_finish", "pack_vt", "attention")


class ShotKVError(RuntimeError):
    pass


class _Config(ctypes.Structure):
    _fields_ = [("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("window", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("sm_scale", ctypes.c_float), ("select_mode", ctypes.c_int32),
                ("head_mode", ctypes.c_int32), ("timing_events", ctypes.c_void_p)]


class _DecodeState(ctypes.Structure):
    _fields_ = [("k_prefill", ctypes.c_void_p), ("v_prefill", ctypes.c_void_p),
                ("prefill_count", ctypes.c_void_p), ("k_dec", ctypes.c_void_p),
                ("v_dec", ctypes.c_void_p), ("slot_pos", ctypes.c_void_p), ("cap", ctypes.c_int32),
                ("n_slots", ctypes.c_int32), ("decode_budget", ctypes.c_int32)]


_lib = None


def load_library() -> ctypes.CDLL:
    """Load libshotkv.so and declare the prototypes.  Raises if the library is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ShotKVError(f"{LIB_PATH} not found: build it with `python -m paper_2502_01941_amd.build`")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    cfgp = ctypes.POINTER(_Config)
    lib.shotkv_strerror.restype = ctypes.c_char_p
    lib.shotkv_strerror.argtypes = [ctypes.c_int]
    lib.shotkv_abi_version.restype = i32
    lib.shotkv_abi_version.argtypes = []
    lib.shotkv_prefill_workspace_bytes.restype = sz
    lib.shotkv_prefill_workspace_bytes.argtypes = [cfgp, i32, i32, i32]
    lib.shotkv_prefill_compress.restype = ctypes.c_int
    lib.shotkv_prefill_compress.argtypes = [cfgp, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, i32, vp, vp,
                                            vp, vp, vp, vp, sz, vp]
    lib.shotkv_prefill_scores.restype = ctypes.c_int
    lib.shotkv_prefill_scores.argtypes = [cfgp, i32, i32, i32, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.shotkv_select_and_compact.restype = ctypes.c_int
    lib.shotkv_select_and_compact.argtypes = [cfgp, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, i32, vp,
                                              vp, vp, vp, vp, sz, vp]
    lib.shotkv_prefill_attention_workspace_bytes.restype = sz
    lib.shotkv_prefill_attention_workspace_bytes.argtypes = [cfgp, i32, i32, i32]
    lib.shotkv_prefill_attention_compress.restype = ctypes.c_int
    lib.shotkv_prefill_attention_compress.argtypes = [cfgp, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, i32,
                                                      vp, vp, vp, vp, vp, vp, sz, vp]
    lib.shotkv_decode_workspace_bytes.restype = sz
    lib.shotkv_decode_workspace_bytes.argtypes = [cfgp, i32, i32, i32]
    lib.shotkv_decode_step.restype = ctypes.c_int
    lib.shotkv_decode_step.argtypes = [cfgp, i32, ctypes.POINTER(_DecodeState), i32, vp, vp, vp, vp, vp,
                                       vp, vp, vp, sz, vp]
    lib.shotkv_decode_step_static.restype = ctypes.c_int
    lib.shotkv_decode_step_static.argtypes = [cfgp, i32, ctypes.POINTER(_DecodeState), i32, vp, vp, vp, vp, vp,
                                              vp, vp, vp]
    _lib = lib
    return lib


def _check(rc: int, what: str):
    if rc != 0:
        raise ShotKVError(f"{what}: {load_library().shotkv_strerror(rc).decode()} ({rc})")


def _dtype_code(dt: torch.dtype) -> int:
    if dt == torch.bfloat16:
        return BF16
    if dt == torch.float32:
        return F32
    raise ShotKVError(f"unsupported dtype {dt}")


def _ptr(t, dtype=None, shape=None, name="tensor"):
    if t is None:
        return None
    if not t.is_cuda:
        raise ShotKVError(f"{name} must live on the GPU")
    if not t.is_contiguous():
        raise ShotKVError(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise ShotKVError(f"{name} must be {dtype}, got {t.dtype}")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ShotKVError(f"{name} must have shape {tuple(shape)}, got {tuple(t.shape)}")
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


_timers = None      # the KernelTimers that configs made from now on point at, or None


def _config(H, H_kv, D, W, dtype, sm_scale, select_mode, head_mode=HEADS_PER_LAYER):
    return _Config(H, H_kv, D, W, _dtype_code(dtype), float(sm_scale), int(select_mode), int(head_mode),
                   _timers.address if _timers is not None else None)


class KernelTimers:
    """Caller-owned HIP events for shotkv_config.timing_events (benchmarks only): one start/stop pair per
    kernel kind.  Use as a context manager around calls; read() waits and returns {kind: ms} for the kinds
    whose kernels ran in the last call."""

    def __init__(self):
        n = len(KERNEL_KINDS)
        self.events = [torch.cuda.Event(enable_timing=True) for _ in range(2 * n)]
        for e in self.events:       # a first record creates the underlying event
            e.record()
        torch.cuda.synchronize()
        self._handles = (ctypes.c_void_p * (2 * n))(*[e.cuda_event for e in self.events])
        self.address = ctypes.cast(self._handles, ctypes.c_void_p)

    def __enter__(self):
        global _timers
        self._before, _timers = _timers, self
        return self

    def __exit__(self, *exc):
        global _timers
        _timers = self._before

    def read(self, kinds):
        torch.cuda.synchronize()
        return {k: self.events[2 * KERNEL_KINDS.index(k)].elapsed_time(self.events[2 * KERNEL_KINDS.index(k) + 1])
                for k in kinds}


def _per(head_mode, H_kv):
    """Leading shape of per-problem outputs: (P,) per layer, (P, H_kv) per KV head."""
    return (H_kv,) if head_mode == HEADS_PER_KV_HEAD else ()


def prefill_workspace_bytes(H, H_kv, D, W, dtype, P, n_tokens, n_shots, sm_scale=1.0,
                            select_mode=SELECT_PREFIX, head_mode=HEADS_PER_LAYER) -> int:
    cfg = _config(H, H_kv, D, W, dtype, sm_scale, select_mode, head_mode)
    n = load_library().shotkv_prefill_workspace_bytes(ctypes.byref(cfg), P, n_tokens, n_shots)
    if n == 0:
        raise ShotKVError("unsupported prefill shape")
    return int(n)


@dataclasses.dataclass
class PrefillResult:
    k_out: torch.Tensor           # [P, H_kv, cap, D]
    v_out: torch.Tensor
    kept_positions: torch.Tensor  # [P, cap] int32         (per-KV-head mode: [P, H_kv, cap])
    kept_count: torch.Tensor      # [P] int32              ([P, H_kv])
    shot_scores: torch.Tensor     # [P, n] float32         ([P, H_kv, n])
    shot_selected: torch.Tensor   # [P, n] uint8           ([P, H_kv, n])
    status: torch.Tensor          # [P] int32              ([P, H_kv])


def _alloc_prefill_outputs(k, P, H_kv, cap, D, n, with_scores=True, head_mode=HEADS_PER_LAYER):
    dev = k.device
    lead = (P,) + _per(head_mode, H_kv)
    return PrefillResult(
        k_out=torch.empty((P, H_kv, cap, D), dtype=k.dtype, device=dev),
        v_out=torch.empty((P, H_kv, cap, D), dtype=k.dtype, device=dev),
        kept_positions=torch.empty(lead + (cap,), dtype=torch.int32, device=dev),
        kept_count=torch.empty(lead, dtype=torch.int32, device=dev),
        shot_scores=torch.empty(lead + (n,), dtype=torch.float32, device=dev) if with_scores else None,
        shot_selected=torch.empty(lead + (n,), dtype=torch.uint8, device=dev),
        status=torch.empty(lead, dtype=torch.int32, device=dev),
    )


def prefill_compress(q_obs, k, v, shot_offsets, budget_tokens, cap, sm_scale,
                     select_mode=SELECT_PREFIX, out: PrefillResult | None = None, workspace=None,
                     head_mode=HEADS_PER_LAYER):
    """shotkv_prefill_compress.  q_obs [P,H,W,D], k/v [P,H_kv,N,D], shot_offsets [P,n+1] int32,
    budget_tokens [P] int32 (all on the GPU).  Returns a PrefillResult; nothing is synchronised."""
    P, H, W, D = q_obs.shape
    _, H_kv, N, _ = k.shape
    n = shot_offsets.shape[1] - 1
    cfg = _config(H, H_kv, D, W, k.dtype, sm_scale, select_mode, head_mode)
    lib = load_library()
    lead = (P,) + _per(head_mode, H_kv)
    if out is None:
        out = _alloc_prefill_outputs(k, P, H_kv, cap, D, n, head_mode=head_mode)
    if workspace is None:
        workspace = torch.empty(prefill_workspace_bytes(H, H_kv, D, W, k.dtype, P, N, n, sm_scale,
                                                        select_mode, head_mode),
                                dtype=torch.uint8, device=k.device)
    rc = lib.shotkv_prefill_compress(
        ctypes.byref(cfg), P, N, n,
        _ptr(q_obs, k.dtype, (P, H, W, D), "q_obs"), _ptr(k, None, (P, H_kv, N, D), "k"),
        _ptr(v, k.dtype, (P, H_kv, N, D), "v"),
        _ptr(shot_offsets, torch.int32, (P, n + 1), "shot_offsets"),
        _ptr(budget_tokens, torch.int32, (P,), "budget_tokens"),
        _ptr(out.k_out, k.dtype, (P, H_kv, cap, D), "k_out"),
        _ptr(out.v_out, k.dtype, (P, H_kv, cap, D), "v_out"), cap,
        _ptr(out.kept_positions, torch.int32, lead + (cap,), "kept_positions"),
        _ptr(out.kept_count, torch.int32, lead, "kept_count"),
        _ptr(out.shot_scores, torch.float32, lead + (n,), "shot_scores"),
        _ptr(out.shot_selected, torch.uint8, lead + (n,), "shot_selected"),
        _ptr(out.status, torch.int32, lead, "status"),
        _ptr(workspace, torch.uint8, None, "workspace"), workspace.numel(), _stream())
    _check(rc, "shotkv_prefill_compress")
    return out


def prefill_attention_compress(q, k, v, shot_offsets, budget_tokens, cap, window, sm_scale,
                               select_mode=SELECT_PREFIX, out: PrefillResult | None = None, workspace=None,
                               attn_out=None, head_mode=HEADS_PER_LAYER):
    """shotkv_prefill_attention_compress.  q [P,H,N,D] (all query rows), k/v [P,H_kv,N,D], window = W.
    Returns (attn_out [P,H,N,D] float32, PrefillResult); nothing is synchronised."""
    P, H, N, D = q.shape
    _, H_kv, _, _ = k.shape
    n = shot_offsets.shape[1] - 1
    cfg = _config(H, H_kv, D, window, k.dtype, sm_scale, select_mode, head_mode)
    lib = load_library()
    lead = (P,) + _per(head_mode, H_kv)
    if out is None:
        out = _alloc_prefill_outputs(k, P, H_kv, cap, D, n, head_mode=head_mode)
    if attn_out is None:
        attn_out = torch.empty((P, H, N, D), dtype=torch.float32, device=k.device)
    if workspace is None:
        nbytes = lib.shotkv_prefill_attention_workspace_bytes(ctypes.byref(cfg), P, N, n)
        if nbytes == 0:
            raise ShotKVError("unsupported shape for the fused attention entry point")
        workspace = torch.empty(int(nbytes), dtype=torch.uint8, device=k.device)
    rc = lib.shotkv_prefill_attention_compress(
        ctypes.byref(cfg), P, N, n, _ptr(q, k.dtype, (P, H, N, D), "q"), _ptr(k, None, (P, H_kv, N, D), "k"),
        _ptr(v, k.dtype, (P, H_kv, N, D), "v"), _ptr(shot_offsets, torch.int32, (P, n + 1), "shot_offsets"),
        _ptr(budget_tokens, torch.int32, (P,), "budget_tokens"),
        _ptr(attn_out, torch.float32, (P, H, N, D), "attn_out"),
        _ptr(out.k_out, k.dtype, (P, H_kv, cap, D), "k_out"), _ptr(out.v_out, k.dtype, (P, H_kv, cap, D), "v_out"),
        cap, _ptr(out.kept_positions, torch.int32, lead + (cap,), "kept_positions"),
        _ptr(out.kept_count, torch.int32, lead, "kept_count"),
        _ptr(out.shot_scores, torch.float32, lead + (n,), "shot_scores"),
        _ptr(out.shot_selected, torch.uint8, lead + (n,), "shot_selected"), _ptr(out.status, torch.int32, lead, "status"),
        _ptr(workspace, torch.uint8, None, "workspace"), workspace.numel(), _stream())
    _check(rc, "shotkv_prefill_attention_compress")
    return attn_out, out


def prefill_scores(q_obs, k, shot_offsets, sm_scale, workspace=None, head_mode=HEADS_PER_LAYER):
    """shotkv_prefill_scores.  Returns (shot_scores [P,n] float32, status [P] int32); both gain an H_kv
    dimension after P in per-KV-head mode."""
    P, H, W, D = q_obs.shape
    _, H_kv, N, _ = k.shape
    n = shot_offsets.shape[1] - 1
    cfg = _config(H, H_kv, D, W, k.dtype, sm_scale, SELECT_PREFIX, head_mode)
    lib = load_library()
    lead = (P,) + _per(head_mode, H_kv)
    scores = torch.empty(lead + (n,), dtype=torch.float32, device=k.device)
    status = torch.empty(lead, dtype=torch.int32, device=k.device)
    if workspace is None:
        workspace = torch.empty(prefill_workspace_bytes(H, H_kv, D, W, k.dtype, P, N, n, sm_scale,
                                                        SELECT_PREFIX, head_mode),
                                dtype=torch.uint8, device=k.device)
    rc = lib.shotkv_prefill_scores(
        ctypes.byref(cfg), P, N, n, _ptr(q_obs, k.dtype, (P, H, W, D), "q_obs"),
        _ptr(k, None, (P, H_kv, N, D), "k"), _ptr(shot_offsets, torch.int32, (P, n + 1), "shot_offsets"),
        _ptr(scores), _ptr(status), _ptr(workspace, torch.uint8, None, "workspace"), workspace.numel(),
        _stream())
    _check(rc, "shotkv_prefill_scores")
    return scores, status


def select_and_compact(shot_scores, k, v, shot_offsets, budget_tokens, cap, H, W,
                       select_mode=SELECT_PREFIX, workspace=None, head_mode=HEADS_PER_LAYER):
    """shotkv_select_and_compact from caller-supplied scores [P,n] float32 ([P,H_kv,n] in per-KV-head
    mode).  Returns a PrefillResult whose shot_scores is the input tensor."""
    P, H_kv, N, D = k.shape
    n = shot_offsets.shape[1] - 1
    cfg = _config(H, H_kv, D, W, k.dtype, 1.0, select_mode, head_mode)
    lib = load_library()
    lead = (P,) + _per(head_mode, H_kv)
    out = _alloc_prefill_outputs(k, P, H_kv, cap, D, n, with_scores=False, head_mode=head_mode)
    out.shot_scores = shot_scores
    if workspace is None:
        workspace = torch.empty(prefill_workspace_bytes(H, H_kv, D, W, k.dtype, P, N, n, 1.0, select_mode,
                                                        head_mode),
                                dtype=torch.uint8, device=k.device)
    rc = lib.shotkv_select_and_compact(
        ctypes.byref(cfg), P, N, n, _ptr(shot_scores, torch.float32, lead + (n,), "shot_scores"),
        _ptr(k, None, (P, H_kv, N, D), "k"), _ptr(v, k.dtype, (P, H_kv, N, D), "v"),
        _ptr(shot_offsets, torch.int32, (P, n + 1), "shot_offsets"),
        _ptr(budget_tokens, torch.int32, (P,), "budget_tokens"), _ptr(out.k_out), _ptr(out.v_out), cap,
        _ptr(out.kept_positions), _ptr(out.kept_count), _ptr(out.shot_selected), _ptr(out.status),
        _ptr(workspace, torch.uint8, None, "workspace"), workspace.numel(), _stream())
    _check(rc, "shotkv_select_and_compact")
    return out


class DecodeState:
    """Caller-owned decode buffers of one layer (see shotkv_decode_state in include/shotkv.h)."""

    def __init__(self, k_prefill, v_prefill, prefill_count, k_dec, v_dec, slot_pos, decode_budget,
                 n_q_heads, sm_scale, head_mode=HEADS_PER_LAYER):
        S, H_kv, cap, D = k_prefill.shape
        n_slots = k_dec.shape[2]
        self.S, self.H_kv, self.cap, self.D, self.n_slots = S, H_kv, cap, D, n_slots
        self.H = n_q_heads
        self.dtype = k_prefill.dtype
        self.sm_scale = float(sm_scale)
        self.decode_budget = int(decode_budget)
        self.k_prefill, self.v_prefill, self.prefill_count = k_prefill, v_prefill, prefill_count
        self.k_dec, self.v_dec, self.slot_pos = k_dec, v_dec, slot_pos
        self.cfg = _config(self.H, H_kv, D, 1, self.dtype, sm_scale, SELECT_PREFIX, head_mode)
        lead = (S,) + _per(head_mode, H_kv)
        self.c_state = _DecodeState(
            _ptr(k_prefill, self.dtype, None, "k_prefill"), _ptr(v_prefill, self.dtype, (S, H_kv, cap, D), "v_prefill"),
            _ptr(prefill_count, torch.int32, lead, "prefill_count"),
            _ptr(k_dec, self.dtype, (S, H_kv, n_slots, D), "k_dec"),
            _ptr(v_dec, self.dtype, (S, H_kv, n_slots, D), "v_dec"),
            _ptr(slot_pos, torch.int32, lead + (n_slots,), "slot_pos"), cap, n_slots, self.decode_budget)
        nbytes = load_library().shotkv_decode_workspace_bytes(ctypes.byref(self.cfg), S, cap, n_slots)
        if nbytes == 0:
            raise ShotKVError("unsupported decode shape")
        dev = k_prefill.device
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        self.out = torch.empty((S, self.H, D), dtype=torch.float32, device=dev)
        self.token_scores = torch.empty(lead + (n_slots,), dtype=torch.float32, device=dev)
        self.evicted_pos = torch.empty(lead, dtype=torch.int32, device=dev)
        self.status = torch.empty(lead, dtype=torch.int32, device=dev)


def decode_step(state: DecodeState, step_index: int, q_new, k_new, v_new, want_scores=True):
    """shotkv_decode_step on `state` (updated in place).  q_new [S,H,D], k_new/v_new [S,H_kv,D].
    Results land in state.out / token_scores / evicted_pos / status; nothing is synchronised."""
    S, H, H_kv, D = state.S, state.H, state.H_kv, state.D
    state.cfg.timing_events = _timers.address if _timers is not None else None
    rc = load_library().shotkv_decode_step(
        ctypes.byref(state.cfg), S, ctypes.byref(state.c_state), int(step_index),
        _ptr(q_new, state.dtype, (S, H, D), "q_new"), _ptr(k_new, state.dtype, (S, H_kv, D), "k_new"),
        _ptr(v_new, state.dtype, (S, H_kv, D), "v_new"), _ptr(state.out),
        _ptr(state.token_scores) if want_scores else None, _ptr(state.evicted_pos), _ptr(state.status),
        _ptr(state.workspace), state.workspace.numel(), _stream())
    _check(rc, "shotkv_decode_step")
    return state.out


def decode_step_static(state: DecodeState, step_index: int, q_new, k_new, v_new, want_scores=True):
    """shotkv_decode_step_static: the same step on the library's own static scratch buffer (state.workspace
    is not used).  Raises ShotKVError (SHOTKV_E_SCRATCH) when the shape needs more than STATIC_SCRATCH_BYTES."""
    S, H, H_kv, D = state.S, state.H, state.H_kv, state.D
    rc = load_library().shotkv_decode_step_static(
        ctypes.byref(state.cfg), S, ctypes.byref(state.c_state), int(step_index),
        _ptr(q_new, state.dtype, (S, H, D), "q_new"), _ptr(k_new, state.dtype, (S, H_kv, D), "k_new"),
        _ptr(v_new, state.dtype, (S, H_kv, D), "v_new"), _ptr(state.out),
        _ptr(state.token_scores) if want_scores else None, _ptr(state.evicted_pos), _ptr(state.status),
        _stream())
    _check(rc, "shotkv_decode_step_static")
    return state.out
