"""ctypes binding of libsquat.so -- same names and argument order as include/squat.h.

Argument marshalling only: every step of the path runs in the library's HIP
kernels.  PyTorch is used for device memory and the current stream.  There is
no CPU fallback: if the library is missing or no GPU is present the calls raise.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

F32, F16, BF16 = 0, 1, 2
_DT = {torch.float32: F32, torch.float16: F16, torch.bfloat16: BF16}
_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libsquat.so")
_lib = None

SYMBOLS = ("squat_version", "squat_strerror", "squat_build_subspace_workspace",
           "squat_build_subspace", "squat_refresh_subspace_workspace", "squat_refresh_subspace",
           "squat_prepare_workspace", "squat_prepare", "squat_prepare_ex", "squat_prepare_noalloc",
           "squat_quantize_keys", "squat_quantize_keys_plan", "squat_dequantize_keys",
           "squat_quantize_keys_per_channel", "squat_dequantize_keys_per_channel", "squat_key_scores", "squat_key_scores_per_channel", "squat_key_scores_rope",
           "squat_key_scores_rope_per_channel",
           "squat_cache_arena_bytes", "squat_cache_create", "squat_cache_destroy", "squat_cache_reset",
           "squat_cache_state", "squat_cache_get_buffers", "squat_cache_prefill", "squat_cache_append",
           "squat_cache_key_scores", "squat_cache_key_scores_rope")


class CacheConfig(ctypes.Structure):
    _fields_ = [("n_batch", ctypes.c_int64), ("n_kv_heads", ctypes.c_int), ("q_per_kv", ctypes.c_int),
                ("d", ctypes.c_int), ("bits", ctypes.c_int), ("group", ctypes.c_int), ("g", ctypes.c_int),
                ("residual", ctypes.c_int), ("max_tokens", ctypes.c_int64), ("kv_dtype", ctypes.c_int),
                ("quantize_values", ctypes.c_int), ("key_per_channel", ctypes.c_int)]


class CacheBuffers(ctypes.Structure):
    _fields_ = [("key_codes", ctypes.c_void_p), ("key_scale", ctypes.c_void_p), ("key_zero", ctypes.c_void_p),
                ("key_residual", ctypes.c_void_p), ("value_codes", ctypes.c_void_p),
                ("value_scale", ctypes.c_void_p), ("value_zero", ctypes.c_void_p),
                ("value_residual", ctypes.c_void_p)]


class CacheCounts(ctypes.Structure):
    _fields_ = [("n_tokens", ctypes.c_int64), ("keys_quantized", ctypes.c_int64), ("keys_residual", ctypes.c_int),
                ("values_quantized", ctypes.c_int64), ("values_residual", ctypes.c_int),
                ("value_ring_head", ctypes.c_int)]


class QuantizePlan(ctypes.Structure):
    _fields_ = [("problems", ctypes.c_int64), ("workgroups_per_problem", ctypes.c_int),
                ("wavefronts_per_workgroup", ctypes.c_int), ("tiles_per_problem", ctypes.c_int64)]


class SquatError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %s (%d)" % (where, strerror(status), status))


def lib() -> ctypes.CDLL:
    """Loads libsquat.so (built in-tree by paper_2503_24358_amd.build); raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError("libsquat.so not found at %s: run `python -m paper_2503_24358_amd.build` "
                           "(there is no fallback path)" % _LIB_PATH)
    L = ctypes.CDLL(_LIB_PATH)
    i64, i32, vp, sz, f32 = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_float
    L.squat_version.restype = i32
    L.squat_version.argtypes = []
    L.squat_strerror.restype = ctypes.c_char_p
    L.squat_strerror.argtypes = [i32]
    L.squat_build_subspace_workspace.restype = sz
    L.squat_build_subspace_workspace.argtypes = [i64, i32, i32, i32, i32]
    L.squat_build_subspace.restype = i32
    L.squat_build_subspace.argtypes = [vp, i32, i64, i32, i32, i32, i64, i64, i32, vp, vp, vp, vp, sz, vp]
    L.squat_refresh_subspace_workspace.restype = sz
    L.squat_refresh_subspace_workspace.argtypes = [i64, i32, i32, i32, i32]
    L.squat_refresh_subspace.restype = i32
    L.squat_refresh_subspace.argtypes = [vp, i32, i64, i32, i32, i32, i64, i64, i32, vp, i32, i32, vp, i32, vp, vp, vp,
                                         vp, sz, vp]
    L.squat_prepare_workspace.restype = sz
    L.squat_prepare_workspace.argtypes = [i32, i32, i32, i32]
    L.squat_prepare.restype = i32
    L.squat_prepare.argtypes = [vp, i32, i32, i32, f32, i32, vp, vp, sz, vp]
    L.squat_prepare_ex.restype = i32
    L.squat_prepare_ex.argtypes = [vp, i32, i32, i32, f32, i32, ctypes.c_uint, vp, vp, sz, vp]
    L.squat_prepare_noalloc.restype = i32
    L.squat_prepare_noalloc.argtypes = [vp, i32, i32, i32, f32, i32, vp, vp]
    L.squat_quantize_keys.restype = i32
    L.squat_quantize_keys.argtypes = [vp, i32, i64, i32, i64, i32, i64, i64, i64, vp, i64, i32, i32, i32,
                                      vp, vp, vp, vp]
    L.squat_quantize_keys_plan.restype = i32
    L.squat_quantize_keys_plan.argtypes = [i32, i64, i32, i64, i32, i64, i32, i32, i32, i32,
                                           ctypes.POINTER(QuantizePlan)]
    L.squat_dequantize_keys.restype = i32
    L.squat_dequantize_keys.argtypes = [vp, vp, vp, i64, i32, i64, i32, i32, i32, vp, i32, i64, i64, i64, vp]
    L.squat_quantize_keys_per_channel.restype = i32
    L.squat_quantize_keys_per_channel.argtypes = L.squat_quantize_keys.argtypes
    L.squat_dequantize_keys_per_channel.restype = i32
    L.squat_dequantize_keys_per_channel.argtypes = L.squat_dequantize_keys.argtypes
    L.squat_key_scores.restype = i32
    L.squat_key_scores.argtypes = [vp, vp, vp, i64, i32, i64, i32, i32, i32, vp, i32, i32, i64, i64, f32, vp,
                                   i64, i64, vp]
    cfgp = ctypes.POINTER(CacheConfig)
    L.squat_cache_arena_bytes.restype = sz
    L.squat_cache_arena_bytes.argtypes = [cfgp]
    L.squat_cache_create.restype = i32
    L.squat_cache_create.argtypes = [cfgp, vp, sz, vp, ctypes.POINTER(vp)]
    L.squat_cache_destroy.restype = None
    L.squat_cache_destroy.argtypes = [vp]
    L.squat_cache_reset.restype = i32
    L.squat_cache_reset.argtypes = [vp]
    L.squat_cache_state.restype = i32
    L.squat_cache_state.argtypes = [vp, ctypes.POINTER(CacheCounts)]
    L.squat_cache_get_buffers.restype = i32
    L.squat_cache_get_buffers.argtypes = [vp, ctypes.POINTER(CacheBuffers)]
    L.squat_cache_prefill.restype = i32
    L.squat_cache_prefill.argtypes = [vp, vp, vp, i64, i64, i64, i64, vp]
    L.squat_cache_append.restype = i32
    L.squat_cache_append.argtypes = [vp, vp, vp, i64, i64, vp]
    L.squat_key_scores_rope.restype = i32
    L.squat_key_scores_rope.argtypes = [vp, vp, vp, i64, i32, i64, i32, i32, i32, vp, i64, vp, i32, i32, i64, i64, f32, vp,
                                        i64, i64, vp]
    L.squat_key_scores_rope_per_channel.restype = i32
    L.squat_key_scores_rope_per_channel.argtypes = [vp, vp, vp, i64, i32, i64, i32, i32, i32, vp, i64, vp, i32, i32, i64, i64, f32, vp,
                                        i64, i64, vp]
    L.squat_key_scores_per_channel.restype = i32
    L.squat_key_scores_per_channel.argtypes = list(L.squat_key_scores.argtypes)
    L.squat_cache_key_scores.restype = i32
    L.squat_cache_key_scores.argtypes = [vp, vp, i32, i64, i64, f32, vp, i64, i64, vp]
    L.squat_cache_key_scores_rope.restype = i32
    L.squat_cache_key_scores_rope.argtypes = [vp, vp, i32, i64, i64, vp, i64, f32, vp, i64, i64, vp]
    _lib = L
    return L


def version() -> int:
    return int(lib().squat_version())


def strerror(status: int) -> str:
    return lib().squat_strerror(int(status)).decode()


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _need_cuda(*ts):
    for t in ts:
        if t is not None and not t.is_cuda:
            raise ValueError("libsquat takes device tensors only")


def _ws(nbytes: int, device) -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def build_subspace_workspace(n_tokens: int, n_kv_heads: int, q_per_kv: int, d: int, r: int) -> int:
    return int(lib().squat_build_subspace_workspace(n_tokens, n_kv_heads, q_per_kv, d, r))


def build_subspace(q: torch.Tensor, q_per_kv: int, r: int, *, want_eig: bool = True, want_gram: bool = False,
                   qhat=None, eig=None, gram=None, ws=None, stream=None):
    """squat_build_subspace.  q: [n_kv_heads*q_per_kv, n_tokens, d] (last dim contiguous).
    Returns (qhat [n_kv, r, d] f32, eig [n_kv, r] f32 or None, gram [n_kv, d, d] f32 or None)."""
    _need_cuda(q)
    hq, n, d = q.shape
    if q.stride(2) != 1 or hq % q_per_kv:
        raise ValueError("q must be [heads, tokens, d] with unit channel stride")
    n_kv = hq // q_per_kv
    dev = q.device
    if qhat is None:
        qhat = torch.empty((n_kv, r, d), dtype=torch.float32, device=dev)
    if eig is None and want_eig:
        eig = torch.empty((n_kv, r), dtype=torch.float32, device=dev)
    if gram is None and want_gram:
        gram = torch.empty((n_kv, d, d), dtype=torch.float32, device=dev)
    if ws is None:
        ws = _ws(build_subspace_workspace(n, n_kv, q_per_kv, d, r), dev)
    rc = lib().squat_build_subspace(_ptr(q), _DT[q.dtype], n, n_kv, q_per_kv, d, q.stride(0), q.stride(1), r,
                                    _ptr(qhat) if r > 0 else None, _ptr(eig), _ptr(gram), _ptr(ws), ws.numel(),
                                    _stream(stream))
    if rc:
        raise SquatError(rc, "squat_build_subspace")
    return qhat, eig, gram


def refresh_subspace(gram_state: torch.Tensor, q_per_kv: int, r: int, iterations: int, *, q_new=None,
                     accumulate: bool = True, qhat_prev=None, qhat=None, eig=None, residual=None, ws=None, stream=None):
    """squat_refresh_subspace.  gram_state: float64 [n_kv_heads, d, d] (updated in place); q_new:
    [n_kv_heads*q_per_kv, n_new, d] or None; qhat_prev: float32 [n_kv_heads, r_prev, d] or None (cold start).
    Returns (qhat [n_kv, r, d] f32, eig [n_kv, r] f32, residual [n_kv] f32)."""
    _need_cuda(gram_state, q_new, qhat_prev)
    n_kv, d, _ = gram_state.shape
    if gram_state.dtype != torch.float64 or not gram_state.is_contiguous():
        raise ValueError("gram_state must be dense float64 [n_kv_heads, d, d]")
    dev = gram_state.device
    n_new, sh, st, dt = 0, 0, 0, BF16
    if q_new is not None:
        hq, n_new, _ = q_new.shape
        if q_new.stride(2) != 1 or hq != n_kv * q_per_kv:
            raise ValueError("q_new must be [n_kv_heads*q_per_kv, tokens, d] with unit channel stride")
        sh, st, dt = q_new.stride(0), q_new.stride(1), _DT[q_new.dtype]
    r_prev = 0
    if qhat_prev is not None:
        if qhat_prev.dtype != torch.float32 or not qhat_prev.is_contiguous() or qhat_prev.shape[0] != n_kv:
            raise ValueError("qhat_prev must be dense float32 [n_kv_heads, r_prev, d]")
        r_prev = qhat_prev.shape[1]
    if qhat is None:
        qhat = torch.empty((n_kv, r, d), dtype=torch.float32, device=dev)
    if eig is None:
        eig = torch.empty((n_kv, r), dtype=torch.float32, device=dev)
    if residual is None:
        residual = torch.empty((n_kv,), dtype=torch.float32, device=dev)
    if ws is None:
        ws = _ws(lib().squat_refresh_subspace_workspace(n_new, n_kv, q_per_kv, d, r), dev)
    rc = lib().squat_refresh_subspace(_ptr(q_new) if n_new else None, dt, n_new, n_kv, q_per_kv, d, sh, st,
                                      int(bool(accumulate)), _ptr(gram_state), r, int(iterations),
                                      _ptr(qhat_prev) if r_prev else None, r_prev, _ptr(qhat) if r > 0 else None,
                                      _ptr(eig), _ptr(residual), _ptr(ws), ws.numel(), _stream(stream))
    if rc:
        raise SquatError(rc, "squat_refresh_subspace")
    return qhat, eig, residual


def prepare_workspace(n_heads: int, d: int, r: int, g: int) -> int:
    return int(lib().squat_prepare_workspace(n_heads, d, r, g))


PREPARE_FULL_PRECISION = 1


def prepare(qhat: torch.Tensor, lam: float, g: int, *, update=None, ws=None, stream=None,
            full_precision: bool = False) -> torch.Tensor:
    """squat_prepare (squat_prepare_ex with SQUAT_PREPARE_FULL_PRECISION when full_precision is set).
    qhat: [n_heads, r, d] f32 dense -> update [n_heads, d, d] f32."""
    _need_cuda(qhat)
    if qhat.dtype != torch.float32 or not qhat.is_contiguous():
        raise ValueError("qhat must be dense float32")
    h, r, d = qhat.shape
    if update is None:
        update = torch.empty((h, d, d), dtype=torch.float32, device=qhat.device)
    if ws is None:
        ws = _ws(prepare_workspace(h, d, r, g), qhat.device)
    if full_precision:
        rc = lib().squat_prepare_ex(_ptr(qhat) if r > 0 else None, h, d, r, float(lam), g, PREPARE_FULL_PRECISION,
                                    _ptr(update), _ptr(ws), ws.numel(), _stream(stream))
    else:
        rc = lib().squat_prepare(_ptr(qhat) if r > 0 else None, h, d, r, float(lam), g, _ptr(update), _ptr(ws),
                                 ws.numel(), _stream(stream))
    if rc:
        raise SquatError(rc, "squat_prepare")
    return update


def prepare_noalloc(qhat: torch.Tensor, lam: float, g: int, update: torch.Tensor, stream=None) -> torch.Tensor:
    """squat_prepare_noalloc: squat_prepare on the library's static scratch; `update` [n_heads, d, d] f32 is
    the caller's (this binding allocates nothing either)."""
    _need_cuda(qhat, update)
    if qhat.dtype != torch.float32 or not qhat.is_contiguous():
        raise ValueError("qhat must be dense float32")
    h, r, d = qhat.shape
    if update.dtype != torch.float32 or not update.is_contiguous() or tuple(update.shape) != (h, d, d):
        raise ValueError("update must be dense float32 [n_heads, d, d]")
    rc = lib().squat_prepare_noalloc(_ptr(qhat) if r > 0 else None, h, d, r, float(lam), g, _ptr(update),
                                     _stream(stream))
    if rc:
        raise SquatError(rc, "squat_prepare_noalloc")
    return update


def quantize_keys(k: torch.Tensor, update: Optional[torch.Tensor], bits: int, group: int, g: int, *,
                  codes=None, scale=None, zero=None, stream=None):
    """squat_quantize_keys.  k: [n_batch, n_heads, n_tokens, d]; update: [n_heads, d, d] f32 shared
    across the batch, or [n_batch, n_heads, d, d], or None (plain round-to-nearest).
    Returns (codes uint32 viewed as int32 [B,H,n,d*bits/32], scale f16 [B,H,n,d/group], zero f16)."""
    _need_cuda(k, update)
    b, h, n, d = k.shape
    if k.stride(3) != 1:
        raise ValueError("k must have unit channel stride")
    dev = k.device
    usb = 0
    if update is not None:
        if update.dtype != torch.float32 or not update.is_contiguous():
            raise ValueError("update must be dense float32")
        if update.dim() == 4:
            usb = update.stride(0)
    if codes is None:
        codes = torch.empty((b, h, n, d * bits // 32), dtype=torch.int32, device=dev)
    if scale is None:
        scale = torch.empty((b, h, n, d // group), dtype=torch.float16, device=dev)
    if zero is None:
        zero = torch.empty((b, h, n, d // group), dtype=torch.float16, device=dev)
    rc = lib().squat_quantize_keys(_ptr(k), _DT[k.dtype], b, h, n, d, k.stride(0), k.stride(1), k.stride(2),
                                   _ptr(update), usb, bits, group, g, _ptr(codes), _ptr(scale), _ptr(zero),
                                   _stream(stream))
    if rc:
        raise SquatError(rc, "squat_quantize_keys")
    return codes, scale, zero


def quantize_keys_plan(k_dtype, n_batch: int, n_heads: int, n_tokens: int, has_update: bool, update_stride_batch: int,
                       bits: int, group: int, g: int, per_channel: bool = False) -> QuantizePlan:
    """squat_quantize_keys_plan: the launch shape the quantize call would use (host-only query)."""
    out = QuantizePlan()
    rc = lib().squat_quantize_keys_plan(_DT[k_dtype], n_batch, n_heads, n_tokens, int(bool(has_update)),
                                        update_stride_batch, bits, group, g, int(bool(per_channel)), ctypes.byref(out))
    if rc:
        raise SquatError(rc, "squat_quantize_keys_plan")
    return out


def dequantize_keys(codes: torch.Tensor, scale: torch.Tensor, zero: torch.Tensor, bits: int, group: int,
                    out_dtype=torch.bfloat16, *, out=None, stream=None) -> torch.Tensor:
    """squat_dequantize_keys.  Dense codes/scale/zero as written by quantize_keys -> k [B,H,n,d]."""
    _need_cuda(codes, scale, zero)
    b, h, n, w = codes.shape
    d = w * 32 // bits
    if not (codes.is_contiguous() and scale.is_contiguous() and zero.is_contiguous()):
        raise ValueError("codes/scale/zero must be dense")
    if out is None:
        out = torch.empty((b, h, n, d), dtype=out_dtype, device=codes.device)
    rc = lib().squat_dequantize_keys(_ptr(codes), _ptr(scale), _ptr(zero), b, h, n, d, bits, group, _ptr(out),
                                     _DT[out.dtype], out.stride(0), out.stride(1), out.stride(2), _stream(stream))
    if rc:
        raise SquatError(rc, "squat_dequantize_keys")
    return out


def quantize_keys_per_channel(k: torch.Tensor, update: Optional[torch.Tensor], bits: int, group: int, g: int, *,
                              codes=None, scale=None, zero=None, stream=None):
    """squat_quantize_keys_per_channel.  k: [n_batch, n_heads, n_tokens, d], n_tokens a multiple of
    group (= 32); update as for quantize_keys.
    Returns (codes uint32 viewed as int32 [B,H,n/32,d,bits], scale f16 [B,H,n/32,d], zero f16)."""
    _need_cuda(k, update)
    b, h, n, d = k.shape
    if k.stride(3) != 1:
        raise ValueError("k must have unit channel stride")
    if group <= 0 or n % group:
        raise ValueError("n_tokens must be a multiple of group")
    dev = k.device
    usb = 0
    if update is not None:
        if update.dtype != torch.float32 or not update.is_contiguous():
            raise ValueError("update must be dense float32")
        if update.dim() == 4:
            usb = update.stride(0)
    if codes is None:
        codes = torch.empty((b, h, n // 32, d, bits), dtype=torch.int32, device=dev)
    if scale is None:
        scale = torch.empty((b, h, n // group, d), dtype=torch.float16, device=dev)
    if zero is None:
        zero = torch.empty((b, h, n // group, d), dtype=torch.float16, device=dev)
    rc = lib().squat_quantize_keys_per_channel(_ptr(k), _DT[k.dtype], b, h, n, d, k.stride(0), k.stride(1),
                                               k.stride(2), _ptr(update), usb, bits, group, g, _ptr(codes),
                                               _ptr(scale), _ptr(zero), _stream(stream))
    if rc:
        raise SquatError(rc, "squat_quantize_keys_per_channel")
    return codes, scale, zero


def dequantize_keys_per_channel(codes: torch.Tensor, scale: torch.Tensor, zero: torch.Tensor, bits: int,
                                group: int, out_dtype=torch.bfloat16, *, out=None, stream=None) -> torch.Tensor:
    """squat_dequantize_keys_per_channel.  Dense codes [B,H,n/32,d,bits], scale/zero [B,H,n/group,d]
    as written by quantize_keys_per_channel -> k [B,H,n,d]."""
    _need_cuda(codes, scale, zero)
    b, h, tiles, d, w = codes.shape
    if w != bits:
        raise ValueError("codes must be [B, H, n/32, d, bits]")
    if not (codes.is_contiguous() and scale.is_contiguous() and zero.is_contiguous()):
        raise ValueError("codes/scale/zero must be dense")
    n = tiles * 32
    if out is None:
        out = torch.empty((b, h, n, d), dtype=out_dtype, device=codes.device)
    rc = lib().squat_dequantize_keys_per_channel(_ptr(codes), _ptr(scale), _ptr(zero), b, h, n, d, bits, group,
                                                 _ptr(out), _DT[out.dtype], out.stride(0), out.stride(1),
                                                 out.stride(2), _stream(stream))
    if rc:
        raise SquatError(rc, "squat_dequantize_keys_per_channel")
    return out


def key_scores(q: torch.Tensor, codes: torch.Tensor, scale: torch.Tensor, zero: torch.Tensor, bits: int,
               group: int, q_per_kv: int, out_scale: float = 1.0, *, out=None, stream=None) -> torch.Tensor:
    """squat_key_scores.  q: [B, n_kv_heads*q_per_kv, d]; codes/scale/zero as written by quantize_keys
    ([B, n_kv_heads, n, ...], dense) -> scores float32 [B, n_kv_heads*q_per_kv, n] (or into `out`, whose
    last dimension may be longer than n: the logits land in its first n columns)."""
    _need_cuda(q, codes, scale, zero)
    b, h, n, w = codes.shape
    d = w * 32 // bits
    if q.dim() != 3 or q.shape[0] != b or q.shape[1] != h * q_per_kv or q.shape[2] != d or q.stride(2) != 1:
        raise ValueError("q must be [B, n_kv_heads*q_per_kv, d] with unit channel stride")
    if not (codes.is_contiguous() and scale.is_contiguous() and zero.is_contiguous()):
        raise ValueError("codes/scale/zero must be dense")
    if out is None:
        out = torch.empty((b, h * q_per_kv, n), dtype=torch.float32, device=codes.device)
    if out.dtype != torch.float32 or out.stride(2) != 1 or out.shape[0] != b or out.shape[1] != h * q_per_kv:
        raise ValueError("out must be float32 [B, n_q_heads, >= n] with unit token stride")
    rc = lib().squat_key_scores(_ptr(codes), _ptr(scale), _ptr(zero), b, h, n, d, bits, group, _ptr(q), _DT[q.dtype],
                                q_per_kv, q.stride(0), q.stride(1), float(out_scale), _ptr(out), out.stride(0),
                                out.stride(1), _stream(stream))
    if rc:
        raise SquatError(rc, "squat_key_scores")
    return out


def key_scores_rope(q: torch.Tensor, codes: torch.Tensor, scale: torch.Tensor, zero: torch.Tensor, bits: int,
                    group: int, q_per_kv: int, inv_freq: torch.Tensor, pos0: int = 0, out_scale: float = 1.0, out=None,
                    stream=None) -> torch.Tensor:
    """squat_key_scores_rope: logits against keys stored before the rotary embedding.  Arguments as for
    key_scores plus inv_freq (float32 [64], device) and the position of token 0."""
    b, h, n, _ = codes.shape
    d = 128
    if inv_freq.dtype != torch.float32 or inv_freq.numel() != 64 or not inv_freq.is_contiguous():
        raise ValueError("inv_freq must be 64 dense float32 values")
    _need_cuda(q, codes, inv_freq)
    if q.dim() != 3 or q.shape[0] != b or q.shape[1] != h * q_per_kv or q.shape[2] != d or q.stride(2) != 1:
        raise ValueError("q must be [B, n_kv_heads*q_per_kv, d] with unit channel stride")
    if not (codes.is_contiguous() and scale.is_contiguous() and zero.is_contiguous()):
        raise ValueError("codes/scale/zero must be dense")
    if out is None:
        out = torch.empty((b, h * q_per_kv, n), dtype=torch.float32, device=codes.device)
    if out.dtype != torch.float32 or out.stride(2) != 1 or out.shape[0] != b or out.shape[1] != h * q_per_kv:
        raise ValueError("out must be float32 [B, n_q_heads, >= n] with unit token stride")
    rc = lib().squat_key_scores_rope(_ptr(codes), _ptr(scale), _ptr(zero), b, h, n, d, bits, group, _ptr(inv_freq),
                                     int(pos0), _ptr(q), _DT[q.dtype], q_per_kv, q.stride(0), q.stride(1),
                                     float(out_scale), _ptr(out), out.stride(0), out.stride(1), _stream(stream))
    if rc:
        raise SquatError(rc, "squat_key_scores_rope")
    return out


def key_scores_rope_per_channel(q: torch.Tensor, codes: torch.Tensor, scale: torch.Tensor, zero: torch.Tensor,
                                bits: int, q_per_kv: int, inv_freq: torch.Tensor, pos0: int = 0,
                                out_scale: float = 1.0, out=None, stream=None) -> torch.Tensor:
    """squat_key_scores_rope_per_channel: logits against keys stored before the rotary embedding in the
    per-channel layout (codes [B, H, n/32, d, bits] int32, scale/zero [B, H, n/32, d] float16).  inv_freq:
    float32 [64] on the device; pos0: position of token 0."""
    b, h, tiles, d, nw = codes.shape
    n = tiles * 32
    if nw != bits or scale.shape != (b, h, tiles, d) or zero.shape != scale.shape:
        raise ValueError("codes [B,H,n/32,d,bits], scale/zero [B,H,n/32,d] expected")
    if inv_freq.dtype != torch.float32 or inv_freq.numel() != 64 or not inv_freq.is_contiguous():
        raise ValueError("inv_freq must be 64 dense float32 values")
    _need_cuda(q, codes, inv_freq)
    if q.dim() != 3 or q.shape[0] != b or q.shape[1] != h * q_per_kv or q.shape[2] != d or q.stride(2) != 1:
        raise ValueError("q must be [B, n_kv_heads*q_per_kv, d] with unit channel stride")
    if not (codes.is_contiguous() and scale.is_contiguous() and zero.is_contiguous()):
        raise ValueError("codes/scale/zero must be dense")
    if out is None:
        out = torch.empty((b, h * q_per_kv, n), dtype=torch.float32, device=codes.device)
    if out.dtype != torch.float32 or out.stride(2) != 1 or out.shape[0] != b or out.shape[1] != h * q_per_kv:
        raise ValueError("out must be float32 [B, n_q_heads, >= n] with unit token stride")
    rc = lib().squat_key_scores_rope_per_channel(_ptr(codes), _ptr(scale), _ptr(zero), b, h, n, d, bits, 32,
                                                 _ptr(inv_freq), int(pos0), _ptr(q), _DT[q.dtype], q_per_kv,
                                                 q.stride(0), q.stride(1), float(out_scale), _ptr(out),
                                                 out.stride(0), out.stride(1), _stream(stream))
    if rc:
        raise SquatError(rc, "squat_key_scores_rope_per_channel")
    return out


def key_scores_per_channel(q: torch.Tensor, codes: torch.Tensor, scale: torch.Tensor, zero: torch.Tensor, bits: int,
                           q_per_kv: int, out_scale: float = 1.0, out=None, stream=None) -> torch.Tensor:
    """squat_key_scores_per_channel.  q: [B, n_kv_heads*q_per_kv, d]; codes [B, H, n/32, d, bits] int32,
    scale/zero [B, H, n/32, d] float16 as written by quantize_keys_per_channel.  Returns float32
    [B, n_kv_heads*q_per_kv, n] (or fills `out`)."""
    b, h, tiles, d, nw = codes.shape
    n = tiles * 32
    if nw != bits or scale.shape != (b, h, tiles, d) or zero.shape != scale.shape:
        raise ValueError("codes [B,H,n/32,d,bits], scale/zero [B,H,n/32,d] expected")
    if q.dim() != 3 or q.shape[0] != b or q.shape[1] != h * q_per_kv or q.shape[2] != d or q.stride(2) != 1:
        raise ValueError("q must be [B, n_kv_heads*q_per_kv, d] with unit channel stride")
    if not (codes.is_contiguous() and scale.is_contiguous() and zero.is_contiguous()):
        raise ValueError("codes/scale/zero must be dense")
    if out is None:
        out = torch.empty((b, h * q_per_kv, n), dtype=torch.float32, device=codes.device)
    if out.dtype != torch.float32 or out.stride(2) != 1 or out.shape[0] != b or out.shape[1] != h * q_per_kv:
        raise ValueError("out must be float32 [B, n_q_heads, >= n] with unit token stride")
    rc = lib().squat_key_scores_per_channel(_ptr(codes), _ptr(scale), _ptr(zero), b, h, n, d, bits, 32, _ptr(q),
                                            _DT[q.dtype], q_per_kv, q.stride(0), q.stride(1), float(out_scale),
                                            _ptr(out), out.stride(0), out.stride(1), _stream(stream))
    if rc:
        raise SquatError(rc, "squat_key_scores_per_channel")
    return out


class Cache:
    """squat_cache_*: the residual-buffer bookkeeping around the stateless calls.  The arena (one uint8
    device tensor) and the update matrix are kept alive by this object; the store tensors returned by
    `stores()` are views into the arena."""

    def __init__(self, n_batch: int, n_kv_heads: int, q_per_kv: int, bits: int, group: int, g: int, residual: int,
                 max_tokens: int, kv_dtype=torch.bfloat16, update: Optional[torch.Tensor] = None,
                 quantize_values: bool = False, device="cuda", d: int = 128, key_per_channel: bool = False):
        self.cfg = CacheConfig(n_batch, n_kv_heads, q_per_kv, d, bits, group, g, residual, max_tokens,
                               _DT[kv_dtype], int(quantize_values), int(key_per_channel))
        self.kv_dtype = kv_dtype
        nbytes = int(lib().squat_cache_arena_bytes(ctypes.byref(self.cfg)))
        if nbytes == 0:
            raise SquatError(-2, "squat_cache_arena_bytes")
        self.arena = torch.empty(nbytes, dtype=torch.uint8, device=device)
        if update is not None and (update.dtype != torch.float32 or not update.is_contiguous()):
            raise ValueError("update must be dense float32")
        self.update = update
        handle = ctypes.c_void_p()
        rc = lib().squat_cache_create(ctypes.byref(self.cfg), _ptr(self.arena), nbytes, _ptr(update), ctypes.byref(handle))
        if rc:
            raise SquatError(rc, "squat_cache_create")
        self._h = handle

    def __del__(self):
        h = getattr(self, "_h", None)
        if h:
            lib().squat_cache_destroy(h)
            self._h = None

    def counts(self) -> CacheCounts:
        out = CacheCounts()
        rc = lib().squat_cache_state(self._h, ctypes.byref(out))
        if rc:
            raise SquatError(rc, "squat_cache_state")
        return out

    def reset(self):
        lib().squat_cache_reset(self._h)

    def _view(self, ptr, shape, dtype):
        off = ptr - self.arena.data_ptr()
        n = 1
        for x in shape:
            n *= x
        nb = n * torch.empty((), dtype=dtype).element_size()
        return self.arena[off:off + nb].view(dtype).view(shape)

    def stores(self) -> dict:
        """Views of the arena: codes int32 [B,H,max,d*bits/32], scale/zero f16 [B,H,max,d/group] (per-channel
        keys: [B,H,max/32,d,bits] and [B,H,max/32,d]), residual
        buffers [B,H,R,d] in the kv dtype (values only when configured)."""
        b = CacheBuffers()
        rc = lib().squat_cache_get_buffers(self._h, ctypes.byref(b))
        if rc:
            raise SquatError(rc, "squat_cache_get_buffers")
        c = self.cfg
        B, H, M, R, d = c.n_batch, c.n_kv_heads, c.max_tokens, c.residual, c.d
        kc, km = (B, H, M, d * c.bits // 32), (B, H, M, d // c.group)
        if c.key_per_channel:
            kc, km = (B, H, M // 32, d, c.bits), (B, H, M // 32, d)
        out = {"key_codes": self._view(b.key_codes, kc, torch.int32),
               "key_scale": self._view(b.key_scale, km, torch.float16),
               "key_zero": self._view(b.key_zero, km, torch.float16),
               "key_residual": self._view(b.key_residual, (B, H, R, d), self.kv_dtype)}
        if c.quantize_values:
            out.update({"value_codes": self._view(b.value_codes, (B, H, M, d * c.bits // 32), torch.int32),
                        "value_scale": self._view(b.value_scale, (B, H, M, d // c.group), torch.float16),
                        "value_zero": self._view(b.value_zero, (B, H, M, d // c.group), torch.float16),
                        "value_residual": self._view(b.value_residual, (B, H, R, d), self.kv_dtype)})
        return out

    def prefill(self, k: torch.Tensor, v: Optional[torch.Tensor] = None, stream=None):
        """k, v: [B, H, n, d] in the kv dtype (same strides)."""
        _need_cuda(k, v)
        if v is not None and v.stride() != k.stride():
            raise ValueError("k and v must share their strides")
        rc = lib().squat_cache_prefill(self._h, _ptr(k), _ptr(v), k.shape[2], k.stride(0), k.stride(1), k.stride(2),
                                       _stream(stream))
        if rc:
            raise SquatError(rc, "squat_cache_prefill")

    def append(self, k: torch.Tensor, v: Optional[torch.Tensor] = None, stream=None):
        """k, v: [B, H, d], one decoded token per sequence."""
        _need_cuda(k, v)
        if v is not None and v.stride() != k.stride():
            raise ValueError("k and v must share their strides")
        rc = lib().squat_cache_append(self._h, _ptr(k), _ptr(v), k.stride(0), k.stride(1), _stream(stream))
        if rc:
            raise SquatError(rc, "squat_cache_append")

    def key_scores(self, q: torch.Tensor, out_scale: float = 1.0, out=None, stream=None) -> torch.Tensor:
        """q: [B, H*q_per_kv, d] -> logits float32 [B, H*q_per_kv, keys cached] (quantized keys first)."""
        _need_cuda(q)
        cnt = self.counts()
        n = cnt.keys_quantized + cnt.keys_residual
        if out is None:
            out = torch.empty((q.shape[0], q.shape[1], n), dtype=torch.float32, device=q.device)
        rc = lib().squat_cache_key_scores(self._h, _ptr(q), _DT[q.dtype], q.stride(0), q.stride(1), float(out_scale),
                                          _ptr(out), out.stride(0), out.stride(1), _stream(stream))
        if rc:
            raise SquatError(rc, "squat_cache_key_scores")
        return out

    def key_scores_rope(self, q: torch.Tensor, inv_freq: torch.Tensor, pos0: int = 0, out_scale: float = 1.0, out=None,
                        stream=None) -> torch.Tensor:
        """Logits against a cache of pre-RoPE keys: cache token t is rotated to position pos0 + t first.
        inv_freq: [d/2] float32 on the device."""
        _need_cuda(q, inv_freq)
        if inv_freq.dtype != torch.float32 or not inv_freq.is_contiguous():
            raise ValueError("inv_freq must be dense float32")
        cnt = self.counts()
        n = cnt.keys_quantized + cnt.keys_residual
        if out is None:
            out = torch.empty((q.shape[0], q.shape[1], n), dtype=torch.float32, device=q.device)
        rc = lib().squat_cache_key_scores_rope(self._h, _ptr(q), _DT[q.dtype], q.stride(0), q.stride(1),
                                               _ptr(inv_freq), int(pos0), float(out_scale), _ptr(out),
                                               out.stride(0), out.stride(1), _stream(stream))
        if rc:
            raise SquatError(rc, "squat_cache_key_scores_rope")
        return out
