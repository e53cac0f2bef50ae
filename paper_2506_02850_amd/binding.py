"""Thin ctypes binding of libmetok.so: same names as the C calls, argument marshalling only.

PyTorch is used for device memory and the current stream; every step of the method runs in
the HIP kernels.  There is no CPU fallback: importing this module without the compiled library,
or calling it without a GPU, raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, List, Optional, Sequence

import torch  # must be imported before the library so that both share one HIP runtime

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmetok.so")

METOK_OK = 0
F32, BF16 = 0, 1
SIM_FLAT, SIM_TOKEN_MEAN, SIM_POOLED = 0, 1, 2
SCORE_CAUSAL_ALL, SCORE_VISUAL_ONLY = 0, 1
EVENT_MEAN, EVENT_MAX = 0, 1
POOL_FLOOR, POOL_CEIL = 0, 1

EXPORTS = [
    "metok_last_error", "metok_version",
    "metok_segment_events_workspace_bytes", "metok_segment_events",
    "metok_compress_encoder_tokens_workspace_bytes", "metok_compress_encoder_tokens",
    "metok_segment_compress_workspace_bytes", "metok_segment_compress",
    "metok_segment_compress_batched_workspace_bytes", "metok_segment_compress_batched",
    "metok_retention_quotas", "metok_account",
    "metok_prefill_prune_workspace_bytes", "metok_prefill_prune",
    "metok_prefill_prune_batched_workspace_bytes", "metok_prefill_prune_batched",
    "metok_kv_compact", "metok_kv_compact_paged", "metok_calib_copy",
    "metok_preset", "metok_compress_encoder_tokens_capacity_rows",
    "metok_static_scratch_bytes", "metok_prefill_prune_static",
    "metok_kv_compact_workspace_bytes", "metok_debug_set_move_spin_limit", "metok_trace_kernel",
    "metok_kv_relink_paged_workspace_bytes", "metok_kv_relink_paged",
]


class AccountStruct(ctypes.Structure):
    _fields_ = [("tokens_encoder", ctypes.c_int64), ("tokens_llm", ctypes.c_int64), ("tokens_key", ctypes.c_int64),
                ("tokens_non", ctypes.c_int64), ("level_tokens", ctypes.c_int64 * 4),
                ("prefill_token_layers", ctypes.c_int64), ("kv_token_layers_full", ctypes.c_int64),
                ("kv_token_layers_stage2", ctypes.c_int64), ("kv_token_layers_stage3", ctypes.c_int64)]


class ParamsStruct(ctypes.Structure):
    _fields_ = [("frames", ctypes.c_int32), ("n_layers", ctypes.c_int32), ("k", ctypes.c_int32), ("s1", ctypes.c_int32),
                ("s2", ctypes.c_int32), ("layers_h", ctypes.c_int32 * 3), ("alpha", ctypes.c_double),
                ("beta", ctypes.c_double), ("r", ctypes.c_double)]


MODEL_LLAVA_OV_0_5B, MODEL_LLAVA_OV_7B, MODEL_LONGVA_7B, MODEL_VILA_13B = 0, 1, 2, 3


class MetokError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"metok error {code}: {text}")
        self.code = code


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2506_02850_amd.build` "
                          "(there is no fallback implementation)")
    lib = ctypes.CDLL(LIB_PATH)
    c = ctypes
    vp, i32, i64, sz, dbl = c.c_void_p, c.c_int, c.c_int64, c.c_size_t, c.c_double
    lib.metok_last_error.restype = c.c_char_p
    lib.metok_last_error.argtypes = []
    lib.metok_version.restype = i32
    lib.metok_segment_events_workspace_bytes.restype = sz
    lib.metok_segment_events_workspace_bytes.argtypes = [i32, i32, i32, i32]
    lib.metok_segment_events.restype = i32
    lib.metok_segment_events.argtypes = [vp, i32, i32, i32, i32, vp, i32, i32, vp, vp, vp, vp, vp, sz, vp]
    lib.metok_compress_encoder_tokens_workspace_bytes.restype = sz
    lib.metok_compress_encoder_tokens_workspace_bytes.argtypes = [i32, i32, i32, i32, i32]
    lib.metok_compress_encoder_tokens.restype = i32
    lib.metok_compress_encoder_tokens.argtypes = [vp, i32, i32, i32, i32, i32, vp, vp, vp, i32, dbl, dbl, i32, i32,
                                                  i32, i32, vp, i64, i32, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.metok_segment_compress_workspace_bytes.restype = sz
    lib.metok_segment_compress_workspace_bytes.argtypes = [i32, i32, i32, i32, i32]
    lib.metok_segment_compress.restype = i32
    lib.metok_segment_compress_batched_workspace_bytes.restype = sz
    lib.metok_segment_compress_batched_workspace_bytes.argtypes = [i32, i32, i32, i32, i32, i32]
    lib.metok_segment_compress_batched.restype = i32
    lib.metok_segment_compress_batched.argtypes = [i32] + [vp, i32, i32, i32, i32, i32, vp, i32, i32, dbl, dbl, i32, i32, i32, i32,
                                                            vp, vp, vp, vp, i64, i32, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.metok_segment_compress.argtypes = [vp, i32, i32, i32, i32, i32, vp, i32, i32, dbl, dbl, i32, i32, i32, i32,
                                           vp, vp, vp, vp, i64, i32, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.metok_retention_quotas.restype = i32
    lib.metok_retention_quotas.argtypes = [i32, dbl, dbl, i64, i64, c.POINTER(c.c_int32)]
    lib.metok_account.restype = i32
    lib.metok_account.argtypes = [c.POINTER(c.c_int32), c.POINTER(c.c_uint8), i32, i32, i32, dbl, dbl, i32, i32, i32, dbl,
                                  c.POINTER(c.c_int32), i32, i64, c.POINTER(AccountStruct)]
    lib.metok_prefill_prune_workspace_bytes.restype = sz
    lib.metok_prefill_prune_workspace_bytes.argtypes = [i64, i32, i32, i32, i32, i32, i32]
    lib.metok_prefill_prune.restype = i32
    lib.metok_prefill_prune.argtypes = [vp, i64, i32, i32, vp, vp, i32, i32, i32, i32, i32, i32, i32, vp, vp, vp, i32,
                                        i32, c.POINTER(c.c_int32), vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.metok_prefill_prune_batched_workspace_bytes.restype = sz
    lib.metok_prefill_prune_batched_workspace_bytes.argtypes = [i32, i64, i32, i32, i32, i32, i32, i32]
    lib.metok_prefill_prune_batched.restype = i32
    lib.metok_prefill_prune_batched.argtypes = [i32, vp, i64, i32, i32, vp, vp, i32, i32, i32, i32, i32, i32, i32, vp, vp, vp, i32,
                                                i32, c.POINTER(c.c_int32), vp, i64, vp, vp, i64, vp, i64, vp, vp, vp, i64, vp, sz, vp]
    lib.metok_kv_compact.restype = i32
    lib.metok_kv_compact_workspace_bytes.restype = sz
    lib.metok_kv_compact_workspace_bytes.argtypes = [i32, i32, i32, i64, i32, i32]
    lib.metok_trace_kernel.restype = i32
    lib.metok_trace_kernel.argtypes = [i32, vp, vp]
    lib.metok_debug_set_move_spin_limit.restype = i32
    lib.metok_debug_set_move_spin_limit.argtypes = [i32]
    lib.metok_kv_compact.argtypes = [c.POINTER(vp), c.POINTER(vp), i32, i32, i32, i64, i32, i32, c.POINTER(vp),
                                     c.POINTER(c.c_int32), vp, vp, sz, vp]
    lib.metok_kv_compact_paged.restype = i32
    lib.metok_kv_compact_paged.argtypes = [c.POINTER(vp), c.POINTER(vp), i32, i32, i32, i64, i32, i32, i32, vp, i32,
                                           c.POINTER(vp), c.POINTER(c.c_int32), vp, vp, sz, vp]
    lib.metok_calib_copy.restype = i32
    lib.metok_calib_copy.argtypes = [vp, vp, sz, vp]
    lib.metok_kv_relink_paged_workspace_bytes.restype = sz
    lib.metok_kv_relink_paged_workspace_bytes.argtypes = [i32, i32, i32, i32, i32, i32, i32]
    lib.metok_kv_relink_paged.restype = i32
    lib.metok_kv_relink_paged.argtypes = [c.POINTER(vp), c.POINTER(vp), i32, i32, i32, i64, i32, i32, i32, vp, i64, i32,
                                          c.POINTER(c.c_int32), c.POINTER(vp), c.POINTER(c.c_int32), vp, vp, vp, vp, vp, vp, sz, vp]
    lib.metok_preset.restype = i32
    lib.metok_preset.argtypes = [i32, c.POINTER(ParamsStruct)]
    lib.metok_compress_encoder_tokens_capacity_rows.restype = i64
    lib.metok_compress_encoder_tokens_capacity_rows.argtypes = [i32, i32, i32, i32, i32, i32]
    lib.metok_static_scratch_bytes.restype = sz
    lib.metok_static_scratch_bytes.argtypes = []
    lib.metok_prefill_prune_static.restype = i32
    lib.metok_prefill_prune_static.argtypes = lib.metok_prefill_prune.argtypes[:-3] + [vp]
    return lib


_lib = _load()


def lib() -> ctypes.CDLL:
    return _lib


def _check(rc: int) -> None:
    if rc != METOK_OK:
        raise MetokError(rc, _lib.metok_last_error().decode())


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.float32:
        return F32
    raise TypeError(f"metok supports float32 and bfloat16 tensors, got {t.dtype}")


def _torch_dtype(code: int) -> torch.dtype:
    return torch.bfloat16 if code == BF16 else torch.float32


def _dev(t: Optional[torch.Tensor], name: str) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name} must live on the GPU (there is no CPU path)")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _workspace(nbytes: int, device) -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def metok_last_error() -> str:
    return _lib.metok_last_error().decode()


def metok_version() -> int:
    return int(_lib.metok_version())


# -------------------------------------------------------------------------------------------------
def _out(out: Optional[Dict[str, torch.Tensor]], name: str, shape, dtype, dev) -> torch.Tensor:
    """A caller-provided output tensor (checked) or a fresh one."""
    if out is not None and name in out and out[name] is not None:
        t = out[name]
        shape = tuple(shape) if isinstance(shape, (tuple, list)) else (shape,)
        if t.dtype != dtype or tuple(t.shape) != shape:
            raise ValueError(f"out[{name!r}] must be {dtype} of shape {shape}, got {t.dtype} {tuple(t.shape)}")
        return t
    return torch.empty(shape, dtype=dtype, device=dev)


def metok_segment_events(feats: torch.Tensor, k: int, text_emb: Optional[torch.Tensor] = None,
                         sim_mode: int = SIM_FLAT, workspace: Optional[torch.Tensor] = None,
                         out: Optional[Dict[str, torch.Tensor]] = None) -> Dict[str, torch.Tensor]:
    """feats [T, N, d] -> sim [T-1], event_start [k+1], frame_event [T] (+ frame_score [T] if text_emb).
    `out` may carry preallocated tensors under the same names."""
    T, N, d = feats.shape
    dt = _dtype_code(feats)
    dev = feats.device
    need = _lib.metok_segment_events_workspace_bytes(T, N, d, dt)
    ws = workspace if workspace is not None else _workspace(need, dev)
    sim = _out(out, "sim", max(T - 1, 0), torch.float32, dev)
    event_start = _out(out, "event_start", k + 1, torch.int32, dev)
    frame_event = _out(out, "frame_event", T, torch.int32, dev)
    frame_score = _out(out, "frame_score", T, torch.float32, dev) if text_emb is not None else None
    _check(_lib.metok_segment_events(_dev(feats, "feats"), dt, T, N, d, _dev(text_emb, "text_emb"), k, sim_mode,
                                     _dev(sim, "sim"), _dev(event_start, "event_start"), _dev(frame_event, "frame_event"),
                                     _dev(frame_score, "frame_score"), _dev(ws, "workspace"), ws.numel(), _stream()))
    res = dict(sim=sim, event_start=event_start, frame_event=frame_event)
    if frame_score is not None:
        res["frame_score"] = frame_score
    return res


def metok_compress_encoder_tokens_capacity_rows(T: int, grid_h: int, grid_w: int, s1: int, s2: int,
                                                pool_edge: int = POOL_FLOOR) -> int:
    rows = int(_lib.metok_compress_encoder_tokens_capacity_rows(int(T), int(grid_h), int(grid_w), int(s1), int(s2), int(pool_edge)))
    if rows < 0:
        raise ValueError("metok_compress_encoder_tokens_capacity_rows: arguments out of range")
    return rows


def metok_preset(model: int) -> Dict[str, object]:
    out = ParamsStruct()
    _check(_lib.metok_preset(int(model), ctypes.byref(out)))
    return dict(frames=out.frames, n_layers=out.n_layers, k=out.k, s1=out.s1, s2=out.s2,
                layers_h=[int(x) for x in out.layers_h], alpha=out.alpha, beta=out.beta, r=out.r)


def metok_compress_encoder_tokens(feats: torch.Tensor, grid_h: int, grid_w: int, event_start: torch.Tensor,
                                  alpha: float, beta: float, s1: int, s2: int,
                                  text_emb: Optional[torch.Tensor] = None,
                                  frame_score: Optional[torch.Tensor] = None,
                                  event_reduce: int = EVENT_MEAN, pool_edge: int = POOL_FLOOR,
                                  out_dtype: Optional[torch.dtype] = None,
                                  out_tokens: Optional[torch.Tensor] = None,
                                  workspace: Optional[torch.Tensor] = None,
                                  out: Optional[Dict[str, torch.Tensor]] = None) -> Dict[str, torch.Tensor]:
    """Key events / key frames and adaptive pooling.  Returns out_tokens (capacity rows; the first
    frame_offsets[T] are valid) plus frame_offsets, token_event, event_is_key, frame_is_key, frame_stride,
    event_score, frame_score -- all on the device; nothing is synchronised."""
    T, N, d = feats.shape
    if N != grid_h * grid_w:
        raise ValueError("feats.shape[1] must equal grid_h * grid_w")
    dt = _dtype_code(feats)
    dev = feats.device
    k = event_start.numel() - 1
    odt = out_dtype if out_dtype is not None else feats.dtype
    cap = metok_compress_encoder_tokens_capacity_rows(T, grid_h, grid_w, s1, s2, pool_edge)
    if out_tokens is None and out is not None:
        out_tokens = out.get("out_tokens")
    if out_tokens is None:
        out_tokens = torch.empty((cap, d), dtype=odt, device=dev)
    need = _lib.metok_compress_encoder_tokens_workspace_bytes(T, grid_h, grid_w, d, dt)
    ws = workspace if workspace is not None else _workspace(need, dev)
    frame_offsets = _out(out, "frame_offsets", T + 1, torch.int32, dev)
    token_event = _out(out, "token_event", out_tokens.shape[0], torch.int32, dev)
    event_is_key = _out(out, "event_is_key", k, torch.uint8, dev)
    frame_is_key = _out(out, "frame_is_key", T, torch.uint8, dev)
    frame_stride = _out(out, "frame_stride", T, torch.int32, dev)
    event_score = _out(out, "event_score", k, torch.float32, dev)
    frame_score_out = _out(out, "frame_score", T, torch.float32, dev)
    _check(_lib.metok_compress_encoder_tokens(
        _dev(feats, "feats"), dt, T, grid_h, grid_w, d, _dev(text_emb, "text_emb"), _dev(frame_score, "frame_score"),
        _dev(event_start, "event_start"), k, float(alpha), float(beta), int(s1), int(s2), event_reduce, pool_edge,
        _dev(out_tokens, "out_tokens"), out_tokens.shape[0], _dtype_code(out_tokens),
        _dev(frame_offsets, "frame_offsets"), _dev(token_event, "token_event"), _dev(event_is_key, "event_is_key"),
        _dev(frame_is_key, "frame_is_key"), _dev(frame_stride, "frame_stride"), _dev(event_score, "event_score"),
        _dev(frame_score_out, "frame_score_out"), _dev(ws, "workspace"), ws.numel(), _stream()))
    return dict(out_tokens=out_tokens, frame_offsets=frame_offsets, token_event=token_event,
                event_is_key=event_is_key, frame_is_key=frame_is_key, frame_stride=frame_stride,
                event_score=event_score, frame_score=frame_score_out)


def metok_segment_compress(feats: torch.Tensor, grid_h: int, grid_w: int, k: int, text_emb: torch.Tensor,
                           alpha: float, beta: float, s1: int, s2: int,
                           sim_mode: int = SIM_FLAT, event_reduce: int = EVENT_MEAN, pool_edge: int = POOL_FLOOR,
                           out_dtype: Optional[torch.dtype] = None, workspace: Optional[torch.Tensor] = None,
                           out: Optional[Dict[str, torch.Tensor]] = None) -> Dict[str, torch.Tensor]:
    """Stage 1 in one call: the outputs of metok_segment_events and metok_compress_encoder_tokens together
    (one pass over feats when all frames are pooled with stride 2 on an even grid, else two)."""
    T, N, d = feats.shape
    if N != grid_h * grid_w:
        raise ValueError("feats.shape[1] must equal grid_h * grid_w")
    dt = _dtype_code(feats)
    dev = feats.device
    odt = out_dtype if out_dtype is not None else feats.dtype
    cap = metok_compress_encoder_tokens_capacity_rows(T, grid_h, grid_w, s1, s2, pool_edge)
    out_tokens = out.get("out_tokens") if out is not None else None
    if out_tokens is None:
        out_tokens = torch.empty((cap, d), dtype=odt, device=dev)
    need = _lib.metok_segment_compress_workspace_bytes(T, grid_h, grid_w, d, dt)
    ws = workspace if workspace is not None else _workspace(need, dev)
    sim = _out(out, "sim", max(T - 1, 0), torch.float32, dev)
    event_start = _out(out, "event_start", k + 1, torch.int32, dev)
    frame_event = _out(out, "frame_event", T, torch.int32, dev)
    frame_offsets = _out(out, "frame_offsets", T + 1, torch.int32, dev)
    token_event = _out(out, "token_event", out_tokens.shape[0], torch.int32, dev)
    event_is_key = _out(out, "event_is_key", k, torch.uint8, dev)
    frame_is_key = _out(out, "frame_is_key", T, torch.uint8, dev)
    frame_stride = _out(out, "frame_stride", T, torch.int32, dev)
    event_score = _out(out, "event_score", k, torch.float32, dev)
    frame_score = _out(out, "frame_score", T, torch.float32, dev)
    _check(_lib.metok_segment_compress(
        _dev(feats, "feats"), dt, T, grid_h, grid_w, d, _dev(text_emb, "text_emb"), int(k), int(sim_mode),
        float(alpha), float(beta), int(s1), int(s2), event_reduce, pool_edge,
        _dev(sim, "sim"), _dev(event_start, "event_start"), _dev(frame_event, "frame_event"),
        _dev(out_tokens, "out_tokens"), out_tokens.shape[0], _dtype_code(out_tokens),
        _dev(frame_offsets, "frame_offsets"), _dev(token_event, "token_event"), _dev(event_is_key, "event_is_key"),
        _dev(frame_is_key, "frame_is_key"), _dev(frame_stride, "frame_stride"), _dev(event_score, "event_score"),
        _dev(frame_score, "frame_score"), _dev(ws, "workspace"), ws.numel(), _stream()))
    return dict(sim=sim, event_start=event_start, frame_event=frame_event, out_tokens=out_tokens,
                frame_offsets=frame_offsets, token_event=token_event, event_is_key=event_is_key,
                frame_is_key=frame_is_key, frame_stride=frame_stride, event_score=event_score, frame_score=frame_score)


def metok_segment_compress_batched(feats: torch.Tensor, grid_h: int, grid_w: int, k: int, text_emb: torch.Tensor,
                                   alpha: float, beta: float, s1: int, s2: int,
                                   sim_mode: int = SIM_FLAT, event_reduce: int = EVENT_MEAN, pool_edge: int = POOL_FLOOR,
                                   out_dtype: Optional[torch.dtype] = None, workspace: Optional[torch.Tensor] = None,
                                   out: Optional[Dict[str, torch.Tensor]] = None) -> Dict[str, torch.Tensor]:
    """Stage 1 in one call for a batch of videos: feats [B, T, N, d], text_emb [B, d]; every output of
    metok_segment_compress with a leading batch dimension."""
    B, T, N, d = feats.shape
    if N != grid_h * grid_w:
        raise ValueError("feats.shape[2] must equal grid_h * grid_w")
    if tuple(text_emb.shape) != (B, d):
        raise ValueError("text_emb must be [B, d]")
    dt = _dtype_code(feats)
    dev = feats.device
    odt = out_dtype if out_dtype is not None else feats.dtype
    cap = metok_compress_encoder_tokens_capacity_rows(T, grid_h, grid_w, s1, s2, pool_edge)
    out_tokens = out.get("out_tokens") if out is not None else None
    if out_tokens is None:
        out_tokens = torch.empty((B, cap, d), dtype=odt, device=dev)
    elif out_tokens.dim() != 3 or out_tokens.shape[0] != B or out_tokens.shape[2] != d:
        raise ValueError("out['out_tokens'] must be [B, capacity rows, d]")
    rows = out_tokens.shape[1]
    need = _lib.metok_segment_compress_batched_workspace_bytes(B, T, grid_h, grid_w, d, dt)
    ws = workspace if workspace is not None else _workspace(need, dev)
    sim = _out(out, "sim", (B, max(T - 1, 0)), torch.float32, dev)
    event_start = _out(out, "event_start", (B, k + 1), torch.int32, dev)
    frame_event = _out(out, "frame_event", (B, T), torch.int32, dev)
    frame_offsets = _out(out, "frame_offsets", (B, T + 1), torch.int32, dev)
    token_event = _out(out, "token_event", (B, rows), torch.int32, dev)
    event_is_key = _out(out, "event_is_key", (B, k), torch.uint8, dev)
    frame_is_key = _out(out, "frame_is_key", (B, T), torch.uint8, dev)
    frame_stride = _out(out, "frame_stride", (B, T), torch.int32, dev)
    event_score = _out(out, "event_score", (B, k), torch.float32, dev)
    frame_score = _out(out, "frame_score", (B, T), torch.float32, dev)
    _check(_lib.metok_segment_compress_batched(
        B, _dev(feats, "feats"), dt, T, grid_h, grid_w, d, _dev(text_emb, "text_emb"), int(k), int(sim_mode),
        float(alpha), float(beta), int(s1), int(s2), event_reduce, pool_edge,
        _dev(sim, "sim"), _dev(event_start, "event_start"), _dev(frame_event, "frame_event"),
        _dev(out_tokens, "out_tokens"), rows, _dtype_code(out_tokens),
        _dev(frame_offsets, "frame_offsets"), _dev(token_event, "token_event"), _dev(event_is_key, "event_is_key"),
        _dev(frame_is_key, "frame_is_key"), _dev(frame_stride, "frame_stride"), _dev(event_score, "event_score"),
        _dev(frame_score, "frame_score"), _dev(ws, "workspace"), ws.numel(), _stream()))
    return dict(sim=sim, event_start=event_start, frame_event=frame_event, out_tokens=out_tokens,
                frame_offsets=frame_offsets, token_event=token_event, event_is_key=event_is_key,
                frame_is_key=frame_is_key, frame_stride=frame_stride, event_score=event_score, frame_score=frame_score)


def metok_retention_quotas(level: int, r: float, alpha: float, n_key_orig: int, n_non_orig: int) -> List[int]:
    out = (ctypes.c_int32 * 2)()
    _check(_lib.metok_retention_quotas(level, float(r), float(alpha), int(n_key_orig), int(n_non_orig), out))
    return [int(out[0]), int(out[1])]


def metok_account(event_len: Sequence[int], event_is_key: Sequence[int], grid_h: int, grid_w: int, alpha: float,
                  beta: float, s1: int, s2: int, pool_edge: int, r: float, layers_h: Sequence[int], n_layers: int,
                  n_text: int) -> Dict[str, object]:
    """Host-only bookkeeping: token counts after each stage and (token, layer) counts of prefill and cache."""
    k = len(event_len)
    if len(event_is_key) != k or len(layers_h) != 3:
        raise ValueError("event_is_key must match event_len and layers_h must have three entries")
    lens = (ctypes.c_int32 * k)(*[int(x) for x in event_len])
    keys = (ctypes.c_uint8 * k)(*[1 if x else 0 for x in event_is_key])
    lh = (ctypes.c_int32 * 3)(*[int(x) for x in layers_h])
    out = AccountStruct()
    _check(_lib.metok_account(lens, keys, k, int(grid_h), int(grid_w), float(alpha), float(beta), int(s1), int(s2),
                              int(pool_edge), float(r), lh, int(n_layers), int(n_text), ctypes.byref(out)))
    res = {name: getattr(out, name) for name, _ in AccountStruct._fields_}
    res["level_tokens"] = [int(x) for x in out.level_tokens]
    return res


def metok_prefill_prune(hidden: torch.Tensor, vis_start: int, n_vis: int, token_seg: torch.Tensor,
                        seg_quota: Sequence[int],
                        q_text: Optional[torch.Tensor] = None, k_all: Optional[torch.Tensor] = None,
                        token_event: Optional[torch.Tensor] = None, event_weight: Optional[torch.Tensor] = None,
                        orig_idx: Optional[torch.Tensor] = None, scores: Optional[torch.Tensor] = None,
                        hidden_out: Optional[torch.Tensor] = None,
                        workspace: Optional[torch.Tensor] = None,
                        out: Optional[Dict[str, torch.Tensor]] = None,
                        score_mode: int = 0, static_scratch: bool = False) -> Dict[str, torch.Tensor]:
    """One pruning level.  With q_text/k_all the attention scores are computed; otherwise `scores` is used as given.
    static_scratch=True calls metok_prefill_prune_static (no workspace argument)."""
    S, D = hidden.shape
    dt = _dtype_code(hidden)
    dev = hidden.device
    n_seg = len(seg_quota)
    total = int(sum(int(q) for q in seg_quota))
    quota_arr = (ctypes.c_int32 * n_seg)(*[int(q) for q in seg_quota])
    if q_text is not None:
        if k_all is None:
            raise ValueError("k_all is required with q_text")
        Hq, Tq, dh = q_text.shape
        Hkv = k_all.shape[0]
        if k_all.shape[1] != S or k_all.shape[2] != dh or _dtype_code(q_text) != dt or _dtype_code(k_all) != dt:
            raise ValueError("k_all must be [Hkv, S, dh] with the dtype of hidden and q_text")
        scores = _out(out, "scores", n_vis, torch.float32, dev)
    else:
        if scores is None:
            raise ValueError("either q_text/k_all or scores must be given")
        Hq = Hkv = dh = Tq = 0
    if static_scratch:
        ws = None
    else:
        need = _lib.metok_prefill_prune_workspace_bytes(S, Hq, Hkv, dh, Tq, n_vis, dt)
        ws = workspace if workspace is not None else _workspace(need, dev)
    kept_idx = _out(out, "kept_idx", total, torch.int32, dev)
    out_rows = S - n_vis + total
    if hidden_out is None and out is not None:
        hidden_out = out.get("hidden_out")
    if hidden_out is None:
        hidden_out = torch.empty((out_rows, D), dtype=hidden.dtype, device=dev)
    elif tuple(hidden_out.shape) != (out_rows, D) or hidden_out.dtype != hidden.dtype:
        raise ValueError(f"hidden_out must be {hidden.dtype} of shape {(out_rows, D)}")
    token_seg_out = _out(out, "token_seg_out", total, torch.int32, dev)
    token_event_out = _out(out, "token_event_out", total, torch.int32, dev) if token_event is not None else None
    orig_idx_out = _out(out, "orig_idx_out", total, torch.int32, dev)
    n_events = int(event_weight.numel()) if event_weight is not None else 0
    args = [_dev(hidden, "hidden"), S, D, dt, _dev(q_text, "q_text"), _dev(k_all, "k_all"), Hq, Hkv, dh, Tq,
            int(score_mode), int(vis_start), int(n_vis), _dev(token_seg, "token_seg"), _dev(token_event, "token_event"),
            _dev(event_weight, "event_weight"), n_events, n_seg, quota_arr, _dev(orig_idx, "orig_idx"),
            _dev(scores, "scores"), _dev(kept_idx, "kept_idx"), _dev(hidden_out, "hidden_out"),
            _dev(token_seg_out, "token_seg_out"), _dev(token_event_out, "token_event_out"),
            _dev(orig_idx_out, "orig_idx_out")]
    if static_scratch:
        _check(_lib.metok_prefill_prune_static(*args, _stream()))
    else:
        _check(_lib.metok_prefill_prune(*args, _dev(ws, "workspace"), ws.numel(), _stream()))
    res = dict(scores=scores, kept_idx=kept_idx, hidden_out=hidden_out, token_seg_out=token_seg_out,
               orig_idx_out=orig_idx_out)
    if token_event_out is not None:
        res["token_event_out"] = token_event_out
    return res


def metok_prefill_prune_batched(hidden: torch.Tensor, vis_start: int, n_vis: int, token_seg: torch.Tensor,
                                seg_quota: Sequence[Sequence[int]],
                                q_text: Optional[torch.Tensor] = None, k_all: Optional[torch.Tensor] = None,
                                token_event: Optional[torch.Tensor] = None, event_weight: Optional[torch.Tensor] = None,
                                orig_idx: Optional[torch.Tensor] = None, scores: Optional[torch.Tensor] = None,
                                hidden_out: Optional[torch.Tensor] = None,
                                workspace: Optional[torch.Tensor] = None,
                                out: Optional[Dict[str, torch.Tensor]] = None,
                                score_mode: int = 0, keep_stride: Optional[int] = None,
                                out_row_stride: Optional[int] = None) -> Dict[str, torch.Tensor]:
    """One pruning level of a batch of videos of one shape: every tensor of metok_prefill_prune with a leading batch
    dimension, seg_quota one list per video.  Returns the per-video kept counts as `n_keep` (a Python list) beside the
    padded outputs ([B, keep_stride] index lists, [B, out_row_stride, D] hidden states)."""
    B, S, D = hidden.shape
    dt = _dtype_code(hidden)
    dev = hidden.device
    if len(seg_quota) != B:
        raise ValueError("seg_quota needs one list per video")
    n_seg = len(seg_quota[0])
    if any(len(q) != n_seg for q in seg_quota):
        raise ValueError("every video needs the same number of retention classes")
    n_keep = [int(sum(int(x) for x in q)) for q in seg_quota]
    quota_arr = (ctypes.c_int32 * (B * n_seg))(*[int(x) for q in seg_quota for x in q])
    if q_text is not None:
        if k_all is None:
            raise ValueError("k_all is required with q_text")
        _, Hq, Tq, dh = q_text.shape
        Hkv = k_all.shape[1]
        if (q_text.shape[0] != B or k_all.shape[0] != B or k_all.shape[2] != S or k_all.shape[3] != dh
                or _dtype_code(q_text) != dt or _dtype_code(k_all) != dt):
            raise ValueError("q_text must be [B, Hq, Tq, dh] and k_all [B, Hkv, S, dh] with the dtype of hidden")
        scores = _out(out, "scores", (B, n_vis), torch.float32, dev)
    else:
        if scores is None:
            raise ValueError("either q_text/k_all or scores must be given")
        Hq = Hkv = dh = Tq = 0
    if orig_idx is not None and (orig_idx.dim() != 2 or orig_idx.shape[0] != B or orig_idx.shape[1] < n_vis):
        raise ValueError("orig_idx must be int32 [B, stride >= n_vis]")
    for name, t, shape in (("token_seg", token_seg, (B, n_vis)), ("token_event", token_event, (B, n_vis)),
                           ("scores", scores, (B, n_vis))):
        if t is not None and tuple(t.shape) != shape:
            raise ValueError(f"{name} must have the shape {shape}")
    need = _lib.metok_prefill_prune_batched_workspace_bytes(B, S, Hq, Hkv, dh, Tq, n_vis, dt)
    ws = workspace if workspace is not None else _workspace(need, dev)
    in_place = hidden_out is hidden
    keep_stride = max(n_keep) if keep_stride is None else int(keep_stride)
    if out_row_stride is None:
        out_row_stride = S if in_place else S - n_vis + max(n_keep)
    kept_idx = _out(out, "kept_idx", (B, keep_stride), torch.int32, dev)
    if hidden_out is None and out is not None:
        hidden_out = out.get("hidden_out")
    if hidden_out is None:
        hidden_out = torch.empty((B, out_row_stride, D), dtype=hidden.dtype, device=dev)
    elif tuple(hidden_out.shape) != (B, out_row_stride, D) or hidden_out.dtype != hidden.dtype:
        raise ValueError(f"hidden_out must be {hidden.dtype} of shape {(B, out_row_stride, D)}")
    token_seg_out = _out(out, "token_seg_out", (B, keep_stride), torch.int32, dev)
    token_event_out = _out(out, "token_event_out", (B, keep_stride), torch.int32, dev) if token_event is not None else None
    # orig_idx_out may be wider than the other lists (the leading columns of stage 3's [B, kept + text] index lists)
    orig_idx_out = out.get("orig_idx_out") if out is not None else None
    if orig_idx_out is None:
        orig_idx_out = torch.empty((B, keep_stride), dtype=torch.int32, device=dev)
    elif orig_idx_out.dtype != torch.int32 or orig_idx_out.dim() != 2 or orig_idx_out.shape[0] != B:
        raise ValueError("out['orig_idx_out'] must be int32 [B, stride]")
    n_events = int(event_weight.shape[1]) if event_weight is not None else 0
    if event_weight is not None and event_weight.shape[0] != B:
        raise ValueError("event_weight must be [B, n_events]")
    _check(_lib.metok_prefill_prune_batched(
        B, _dev(hidden, "hidden"), S, D, dt, _dev(q_text, "q_text"), _dev(k_all, "k_all"), Hq, Hkv, dh, Tq,
        int(score_mode), int(vis_start), int(n_vis), _dev(token_seg, "token_seg"), _dev(token_event, "token_event"),
        _dev(event_weight, "event_weight"), n_events, n_seg, quota_arr, _dev(orig_idx, "orig_idx"),
        orig_idx.shape[1] if orig_idx is not None else 0,
        _dev(scores, "scores"), _dev(kept_idx, "kept_idx"), keep_stride, _dev(hidden_out, "hidden_out"), out_row_stride,
        _dev(token_seg_out, "token_seg_out"), _dev(token_event_out, "token_event_out"),
        _dev(orig_idx_out, "orig_idx_out"), orig_idx_out.shape[1], _dev(ws, "workspace"), ws.numel(), _stream()))
    res = dict(scores=scores, kept_idx=kept_idx, hidden_out=hidden_out, token_seg_out=token_seg_out,
               orig_idx_out=orig_idx_out, n_keep=n_keep)
    if token_event_out is not None:
        res["token_event_out"] = token_event_out
    return res


def _layer_tables(k_layers, v_layers, idx, shape, B):
    """ctypes pointer tables of the per-layer K / V buffers and index lists, plus the per-layer kept counts."""
    L = len(k_layers)
    if len(v_layers) != L or len(idx) != L:
        raise ValueError("K buffers, V buffers and idx must have one entry per layer")
    dev = k_layers[0].device
    vp = ctypes.c_void_p
    karr, varr, iarr = (vp * L)(), (vp * L)(), (vp * L)()
    nk = (ctypes.c_int32 * L)()
    for l in range(L):
        if tuple(k_layers[l].shape) != shape or tuple(v_layers[l].shape) != shape:
            raise ValueError(f"every layer must have the shape {shape}")
        karr[l] = _dev(k_layers[l], "K buffer")
        varr[l] = _dev(v_layers[l], "V buffer")
        if idx[l] is None:
            iarr[l] = None
            nk[l] = 0
        else:
            if idx[l].dtype != torch.int32 or idx[l].dim() != 2 or idx[l].shape[0] != B:
                raise ValueError("idx[l] must be int32 [B, n_keep]")
            # an empty list (drop every row) still needs a non-NULL pointer: NULL means "leave the layer alone"
            iarr[l] = _dev(idx[l], "idx") if idx[l].numel() else _dev(new_len_dummy(dev), "idx")
            nk[l] = idx[l].shape[1]
    return L, karr, varr, iarr, nk


def metok_kv_compact_workspace_bytes(L: int, B: int, Hkv: int, S_cap: int, dh: int, dtype_code: int) -> int:
    return int(_lib.metok_kv_compact_workspace_bytes(int(L), int(B), int(Hkv), int(S_cap), int(dh), int(dtype_code)))


def metok_kv_compact(k_layers: Sequence[torch.Tensor], v_layers: Sequence[torch.Tensor],
                     idx: Sequence[Optional[torch.Tensor]], new_len: Optional[torch.Tensor] = None,
                     workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """In-place compaction of per-layer K/V caches [B, Hkv, S_cap, dh] to idx[l] [B, n_keep_l] (None = untouched).
    `workspace` (uint8, metok_kv_compact_workspace_bytes) is allocated here when not given; after the call its
    first int32 word is 0 unless a bounded wait inside the kernel expired."""
    B, Hkv, S_cap, dh = k_layers[0].shape
    L, karr, varr, iarr, nk = _layer_tables(k_layers, v_layers, idx, (B, Hkv, S_cap, dh), B)
    dev = k_layers[0].device
    dt = _dtype_code(k_layers[0])
    if new_len is None:
        new_len = torch.empty(L, dtype=torch.int32, device=dev)
    ws = workspace if workspace is not None else _workspace(_lib.metok_kv_compact_workspace_bytes(L, B, Hkv, S_cap, dh, dt), dev)
    _check(_lib.metok_kv_compact(karr, varr, L, B, Hkv, S_cap, dh, dt, iarr, nk,
                                 _dev(new_len, "new_len"), _dev(ws, "workspace"), ws.numel(), _stream()))
    return new_len


def metok_kv_compact_paged(k_pools: Sequence[torch.Tensor], v_pools: Sequence[torch.Tensor], page_table: torch.Tensor,
                           idx: Sequence[Optional[torch.Tensor]], new_len: Optional[torch.Tensor] = None,
                           workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """In-place compaction of paged per-layer K/V pools [n_pages, Hkv, page_size, dh] through page_table [B, pages_per_seq]
    to the logical rows idx[l] [B, n_keep_l] (None = untouched)."""
    n_pages, Hkv, page_size, dh = k_pools[0].shape
    if page_table.dtype != torch.int32 or page_table.dim() != 2:
        raise ValueError("page_table must be int32 [B, pages_per_seq]")
    B, pages_per_seq = page_table.shape
    L, karr, varr, iarr, nk = _layer_tables(k_pools, v_pools, idx, (n_pages, Hkv, page_size, dh), B)
    dev = k_pools[0].device
    dt = _dtype_code(k_pools[0])
    if new_len is None:
        new_len = torch.empty(L, dtype=torch.int32, device=dev)
    ws = workspace if workspace is not None else _workspace(
        _lib.metok_kv_compact_workspace_bytes(L, B, Hkv, pages_per_seq * page_size, dh, dt), dev)
    _check(_lib.metok_kv_compact_paged(karr, varr, L, B, Hkv, n_pages, page_size, dh, dt,
                                       _dev(page_table, "page_table"), pages_per_seq, iarr, nk, _dev(new_len, "new_len"),
                                       _dev(ws, "workspace"), ws.numel(), _stream()))
    return new_len


def metok_kv_relink_paged(k_pools: Sequence[torch.Tensor], v_pools: Sequence[torch.Tensor], page_table: torch.Tensor,
                          idx: Sequence[Optional[torch.Tensor]], len_in: Optional[Sequence[int]] = None,
                          workspace: Optional[torch.Tensor] = None) -> Dict[str, torch.Tensor]:
    """Compaction of paged per-layer K/V pools [n_pages, Hkv, page_size, dh] by relinking whole pages and copying the rest.
    page_table is [B, pages_per_seq] (shared by the layers) or [L, B, pages_per_seq]; returns page_table_out [L, B, pages],
    free_pages [L, B, pages], n_free [L, B], rows_copied [L, B], new_len [L] and the workspace."""
    n_pages, Hkv, page_size, dh = k_pools[0].shape
    if page_table.dtype != torch.int32 or page_table.dim() not in (2, 3):
        raise ValueError("page_table must be int32 [B, pages_per_seq] or [L, B, pages_per_seq]")
    B, pages_per_seq = page_table.shape[-2:]
    L, karr, varr, iarr, nk = _layer_tables(k_pools, v_pools, idx, (n_pages, Hkv, page_size, dh), B)
    if page_table.dim() == 3 and page_table.shape[0] != L:
        raise ValueError("a per-layer page_table needs one table per layer")
    stride = 0 if page_table.dim() == 2 else B * pages_per_seq
    dev = k_pools[0].device
    dt = _dtype_code(k_pools[0])
    i32 = torch.int32
    out = dict(page_table_out=torch.empty((L, B, pages_per_seq), dtype=i32, device=dev),
               free_pages=torch.empty((L, B, pages_per_seq), dtype=i32, device=dev),
               n_free=torch.empty((L, B), dtype=i32, device=dev), rows_copied=torch.empty((L, B), dtype=i32, device=dev),
               new_len=torch.empty(L, dtype=i32, device=dev))
    ws = workspace if workspace is not None else _workspace(
        _lib.metok_kv_relink_paged_workspace_bytes(L, B, Hkv, page_size, pages_per_seq, dh, dt), dev)
    lens = None if len_in is None else (ctypes.c_int32 * L)(*[int(x) for x in len_in])
    _check(_lib.metok_kv_relink_paged(karr, varr, L, B, Hkv, n_pages, page_size, dh, dt, _dev(page_table, "page_table"), stride,
                                      pages_per_seq, lens, iarr, nk, _dev(out["page_table_out"], "page_table_out"),
                                      _dev(out["free_pages"], "free_pages"), _dev(out["n_free"], "n_free"),
                                      _dev(out["rows_copied"], "rows_copied"), _dev(out["new_len"], "new_len"),
                                      _dev(ws, "workspace"), ws.numel(), _stream()))
    out["workspace"] = ws
    return out


def metok_debug_set_move_spin_limit(polls: int) -> None:
    _check(_lib.metok_debug_set_move_spin_limit(int(polls)))


_DUMMY = {}


def new_len_dummy(dev) -> torch.Tensor:
    key = str(dev)
    if key not in _DUMMY:
        _DUMMY[key] = torch.zeros(4, dtype=torch.int32, device=dev)
    return _DUMMY[key]


def metok_prefill_prune_static(*a, **kw) -> Dict[str, torch.Tensor]:
    """metok_prefill_prune on the library's static scratch array (nothing is allocated for the workspace)."""
    return metok_prefill_prune(*a, static_scratch=True, **kw)


def metok_static_scratch_bytes() -> int:
    return int(_lib.metok_static_scratch_bytes())


def metok_calib_copy(dst: torch.Tensor, src: torch.Tensor) -> None:
    nbytes = src.numel() * src.element_size()
    _check(_lib.metok_calib_copy(_dev(dst, "dst"), _dev(src, "src"), nbytes, _stream()))
