"""ctypes binding of librestkv.so: argument marshalling only.

Function names and arguments mirror ``include/restkv.h``.  Tensors are torch
tensors on the GPU; torch is used for device memory and the current stream,
nothing else -- every step of the path runs in the library's HIP kernels.
There is no CPU fallback: a missing library raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
# RESTKV_LIB names another build of the same library (the host-sanitized one of the CPU tests)
LIB_PATH = os.environ.get("RESTKV_LIB") or os.path.join(_PKG, "librestkv.so")

RESTKV_F32 = 0
RESTKV_BF16 = 1
# ablation variants (restkv_params.variant, see include/restkv.h)
RESTKV_IND_ATTENTION = 1
RESTKV_IND_VALUE_NORM = 2
RESTKV_GROUP_MAX = 1 << 2
RESTKV_TEMPORAL_MEAN = 1 << 4
RESTKV_TEMPORAL_INV_EMA = 2 << 4
RESTKV_POOL_MAX = 1 << 6


class RestkvParams(ctypes.Structure):
    _fields_ = [
        ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
        ("seq_len", ctypes.c_int32), ("window", ctypes.c_int32), ("budget", ctypes.c_int32),
        ("dtype", ctypes.c_int32), ("causal", ctypes.c_int32), ("scale", ctypes.c_float),
        ("ema_alpha", ctypes.c_float), ("base_window", ctypes.c_int32), ("adaptive", ctypes.c_int32),
        ("beta", ctypes.c_float), ("variant", ctypes.c_int32),
        ("q_stride_h", ctypes.c_int64), ("q_stride_t", ctypes.c_int64),
        ("kv_stride_h", ctypes.c_int64), ("kv_stride_t", ctypes.c_int64), ("ld_score", ctypes.c_int64),
    ]


class RestkvError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        super().__init__(f"{what}: {strerror(code)} (code {code})")


_lib = None


def lib() -> ctypes.CDLL:
    """Loads the HIP library; fails loudly when it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'`"
                              " (there is no CPU fallback)")
        L = ctypes.CDLL(LIB_PATH)
        P = ctypes.POINTER(RestkvParams)
        vp, sz, i64 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int64
        L.restkv_workspace_bytes.restype = sz
        L.restkv_workspace_bytes.argtypes = [P]
        L.restkv_prepare_wo.argtypes = [P, vp, i64, vp, vp]
        L.restkv_score.argtypes = [P, vp, vp, vp, vp, vp, vp, sz, vp]
        L.restkv_score_from_attention.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.restkv_score_from_attention.restype = ctypes.c_int
        L.restkv_smooth.argtypes = [P, vp, vp, vp, vp, vp, vp, sz, vp]
        L.restkv_score_smooth.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.restkv_select.argtypes = [P, vp, vp, vp, sz, vp]
        L.restkv_smooth_b.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.restkv_select_b.argtypes = [P, vp, vp, vp, vp, sz, vp]
        L.restkv_select_static.argtypes = [P, vp, vp, vp]
        L.restkv_select_static.restype = ctypes.c_int
        L.restkv_select_static_capacity.restype = sz
        L.restkv_select_static_capacity.argtypes = []
        L.restkv_compact.argtypes = [P, vp, vp, vp, vp, vp, vp]
        L.restkv_strerror.restype = ctypes.c_char_p
        L.restkv_strerror.argtypes = [ctypes.c_int]
        L.restkv_timing_read.argtypes = [vp, vp, ctypes.c_int]
        L.restkv_timing_enable.argtypes = [ctypes.c_int]
        L.restkv_stage_name.restype = ctypes.c_char_p
        L.restkv_stage_name.argtypes = [ctypes.c_int]
        L.restkv_debug_force_fp32.argtypes = [ctypes.c_int]
        L.restkv_debug_force_fp32.restype = ctypes.c_int
        L.restkv_stream_reference.argtypes = [vp, sz, vp, sz, vp]
        L.restkv_stream_reference.restype = ctypes.c_int
        for f in ("restkv_timing_enable", "restkv_timing_read", "restkv_prepare_wo", "restkv_score", "restkv_smooth", "restkv_select",
                  "restkv_compact", "restkv_version", "restkv_score_smooth", "restkv_smooth_b", "restkv_select_b"):
            getattr(L, f).restype = ctypes.c_int
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().restkv_strerror(int(code)).decode()


def make_params(*, n_q_heads, n_kv_heads, head_dim, seq_len, window, budget, dtype,
                causal=True, scale=0.0, ema_alpha=0.3, base_window=5, adaptive=True, beta=2000.0,
                q_stride_h=0, q_stride_t=0, kv_stride_h=0, kv_stride_t=0, ld_score=0, variant=0) -> RestkvParams:
    dt = {torch.float32: RESTKV_F32, torch.bfloat16: RESTKV_BF16, "f32": RESTKV_F32,
          "bf16": RESTKV_BF16}.get(dtype, dtype)
    return RestkvParams(n_q_heads, n_kv_heads, head_dim, seq_len, window, budget, int(dt),
                        int(bool(causal)), float(scale), float(ema_alpha), int(base_window),
                        int(bool(adaptive)), float(beta), int(variant), q_stride_h, q_stride_t, kv_stride_h,
                        kv_stride_t, ld_score)


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream=None):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _chk(rc: int, what: str):
    if rc != 0:
        raise RestkvError(rc, what)


def restkv_workspace_bytes(p: RestkvParams) -> int:
    return int(lib().restkv_workspace_bytes(ctypes.byref(p)))


def alloc_workspace(p: RestkvParams, device="cuda") -> torch.Tensor:
    n = restkv_workspace_bytes(p)
    if n == 0:
        raise RestkvError(-1, "restkv_workspace_bytes")
    return torch.empty(n + 256, dtype=torch.uint8, device=device)


def _ws(ws: Optional[torch.Tensor]):
    if ws is None:
        return None, 0
    off = (-ws.data_ptr()) % 256
    return ctypes.c_void_p(ws.data_ptr() + off), ws.numel() - off


def restkv_prepare_wo(p, w_o: torch.Tensor, gram: torch.Tensor, stream=None):
    _chk(lib().restkv_prepare_wo(ctypes.byref(p), _ptr(w_o), w_o.shape[1], _ptr(gram), _stream(stream)),
         "restkv_prepare_wo")


def restkv_score(p, q, k, v, gram, score, workspace, stream=None):
    wp, wn = _ws(workspace)
    _chk(lib().restkv_score(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(gram), _ptr(score),
                            wp, wn, _stream(stream)), "restkv_score")


def restkv_score_from_attention(p, q, k, v, gram, attn_out, lse, score, workspace, stream=None):
    wp, wn = _ws(workspace)
    _chk(lib().restkv_score_from_attention(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(gram), _ptr(attn_out),
                                           _ptr(lse), _ptr(score), wp, wn, _stream(stream)),
         "restkv_score_from_attention")


def restkv_smooth(p, score, ema, final, aws_info, aws_d, workspace, stream=None):
    wp, wn = _ws(workspace)
    _chk(lib().restkv_smooth(ctypes.byref(p), _ptr(score), _ptr(ema), _ptr(final), _ptr(aws_info),
                             _ptr(aws_d), wp, wn, _stream(stream)), "restkv_smooth")


def restkv_score_smooth(p, q, k, v, gram, score, ema, final, aws_info, aws_d, workspace, stream=None):
    wp, wn = _ws(workspace)
    _chk(lib().restkv_score_smooth(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(gram), _ptr(score),
                                   _ptr(ema), _ptr(final), _ptr(aws_info), _ptr(aws_d), wp, wn,
                                   _stream(stream)), "restkv_score_smooth")


def restkv_smooth_b(p, score, head_budget, ema, final, aws_info, aws_d, workspace, stream=None):
    wp, wn = _ws(workspace)
    _chk(lib().restkv_smooth_b(ctypes.byref(p), _ptr(score), _ptr(head_budget), _ptr(ema), _ptr(final),
                               _ptr(aws_info), _ptr(aws_d), wp, wn, _stream(stream)), "restkv_smooth_b")


def restkv_select_b(p, final, head_budget, idx, workspace, stream=None):
    wp, wn = _ws(workspace)
    _chk(lib().restkv_select_b(ctypes.byref(p), _ptr(final), _ptr(head_budget), _ptr(idx), wp, wn,
                               _stream(stream)), "restkv_select_b")


def restkv_select(p, final, idx, workspace, stream=None):
    wp, wn = _ws(workspace)
    _chk(lib().restkv_select(ctypes.byref(p), _ptr(final), _ptr(idx), wp, wn, _stream(stream)),
         "restkv_select")


def restkv_select_static(p, final, idx, stream=None):
    _chk(lib().restkv_select_static(ctypes.byref(p), _ptr(final), _ptr(idx), _stream(stream)),
         "restkv_select_static")


def restkv_select_static_capacity() -> int:
    return int(lib().restkv_select_static_capacity())


def restkv_compact(p, k, v, idx, k_out, v_out, stream=None):
    _chk(lib().restkv_compact(ctypes.byref(p), _ptr(k), _ptr(v), _ptr(idx), _ptr(k_out), _ptr(v_out),
                              _stream(stream)), "restkv_compact")


N_STAGES = 10


def restkv_timing_enable(on):
    """True / False, or a collection of stage names to time only those (see restkv_timing_read)."""
    if isinstance(on, (bool, int)):
        mask = -1 if on else 0
    else:
        names = [lib().restkv_stage_name(s).decode() for s in range(N_STAGES)]
        mask = 0
        for name in on:
            mask |= 1 << names.index(name)
    _chk(lib().restkv_timing_enable(mask), "restkv_timing_enable")


def restkv_timing_read():
    """{stage name: (total ms, launches)} since the last read; waits for the recorded events."""
    ms = (ctypes.c_double * N_STAGES)()
    cnt = (ctypes.c_int64 * N_STAGES)()
    _chk(lib().restkv_timing_read(ms, cnt, N_STAGES), "restkv_timing_read")
    return {lib().restkv_stage_name(s).decode(): (ms[s], cnt[s]) for s in range(N_STAGES)}


def restkv_debug_force_fp32(on: bool):
    _chk(lib().restkv_debug_force_fp32(int(bool(on))), "restkv_debug_force_fp32")


def restkv_stream_reference(src: Optional[torch.Tensor], read_bytes: int, dst: Optional[torch.Tensor],
                            write_bytes: int, stream=None):
    """Plain streaming kernel with a given read / write byte mix (a measurement aid)."""
    _chk(lib().restkv_stream_reference(_ptr(src), int(read_bytes), _ptr(dst), int(write_bytes), _stream(stream)),
         "restkv_stream_reference")


def restkv_version() -> int:
    return int(lib().restkv_version())


@dataclass
class LayerBuffers:
    """Device buffers of one layer's pass (allocated once, reused across layers)."""
    score: torch.Tensor
    ema: torch.Tensor
    final: torch.Tensor
    aws_info: torch.Tensor
    aws_d: torch.Tensor
    idx: torch.Tensor
    k_out: torch.Tensor
    v_out: torch.Tensor
    workspace: torch.Tensor


def alloc_layer_buffers(p: RestkvParams, dtype: torch.dtype, device="cuda") -> LayerBuffers:
    Hkv, W, B, d = p.n_kv_heads, p.window, p.budget, p.head_dim
    ld = p.ld_score if p.ld_score else p.seq_len - p.window
    f32 = dict(dtype=torch.float32, device=device)
    return LayerBuffers(
        score=torch.empty((Hkv, W, ld), **f32), ema=torch.empty((Hkv, ld), **f32),
        final=torch.empty((Hkv, ld), **f32),
        aws_info=torch.empty((Hkv, 2), dtype=torch.int32, device=device),
        aws_d=torch.empty((Hkv, 2), dtype=torch.float64, device=device),
        idx=torch.empty((Hkv, B), dtype=torch.int32, device=device),
        k_out=torch.empty((Hkv, B, d), dtype=dtype, device=device),
        v_out=torch.empty((Hkv, B, d), dtype=dtype, device=device),
        workspace=alloc_workspace(p, device))


def evict_layer(p: RestkvParams, q, k, v, gram, buf: LayerBuffers, stream=None, fused=False):
    """The calls of one layer, back to back on one stream (no host synchronisation); with
    fused=True the score and the smoothing run as the one fused call."""
    if fused:
        restkv_score_smooth(p, q, k, v, gram, buf.score, buf.ema, buf.final, buf.aws_info, buf.aws_d,
                            buf.workspace, stream)
    else:
        restkv_score(p, q, k, v, gram, buf.score, buf.workspace, stream)
        restkv_smooth(p, buf.score, buf.ema, buf.final, buf.aws_info, buf.aws_d, buf.workspace, stream)
    restkv_select(p, buf.final, buf.idx, buf.workspace, stream)
    restkv_compact(p, k, v, buf.idx, buf.k_out, buf.v_out, stream)
