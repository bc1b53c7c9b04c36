"""Thin binding over liblss_attn.so: same names as the C ABI (include/lss_attn.h).

Argument marshalling only -- every step of the path runs in the HIP kernels.  torch
supplies device memory and the stream; nothing here computes.  If the library has
not been built, the first call raises (there is no fallback path).
"""
from __future__ import annotations

import ctypes
from pathlib import Path

import torch

_PKG = Path(__file__).resolve().parent
LIB_PATH = _PKG / "liblss_attn.so"
_lib = None

LSS_OK = 0
STATUS_NAMES = {0: "LSS_OK", -1: "LSS_ERR_NULL", -2: "LSS_ERR_SHAPE", -3: "LSS_ERR_UNSUPPORTED_D",
                -4: "LSS_ERR_ALIGN", -5: "LSS_ERR_RANGE", -6: "LSS_ERR_WORKSPACE", -7: "LSS_ERR_LAUNCH"}

EXPORTS = ["lss_version", "lss_last_error", "lss_workspace_bytes", "lss_set_workspace",
           "lss_segment_attn_fwd", "lss_segment_attn_bwd", "lss_segment_attn_fwd_f32",
           "lss_segment_attn_bwd_f32", "lss_segment_attn_fwd_dropout", "lss_segment_attn_bwd_dropout",
           "lss_segment_attn_fwd_ex", "lss_segment_attn_bwd_ex", "lss_segment_attn_bwd_noalloc", "lss_reduce_partials", "lss_project_qkv", "lss_project_bwd",
           "lss_project_bwd_ex", "lss_project_bwd_weight_scratch_bytes", "lss_project_bwd_weight",
           "lss_embed_pe_fwd", "lss_embed_pe_bwd", "lss_residual_dropout_add", "lss_layernorm_fwd", "lss_layernorm_bwd_scratch_bytes",
           "lss_layernorm_bwd", "lss_linear_fwd", "lss_linear_bwd_input", "lss_linear_bwd_weight_scratch_bytes", "lss_linear_bwd_weight",
           "lss_linear_gelu_fwd",
           "lss_linear_bwd_input_gelu", "lss_gelu_fwd", "lss_gelu_bwd"]

LSS_FLAG_SKIP_MASKED_TAIL = 1


class LssError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"{STATUS_NAMES.get(code, code)}: {msg}")
        self.code = code


def load():
    """Load the built library (once).  Raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not LIB_PATH.exists():
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2311_02382_amd.build` "
                           "(there is no fallback implementation)")
    lib = ctypes.CDLL(str(LIB_PATH))
    i64, vp, ci, sz = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    lib.lss_version.restype = ci
    lib.lss_last_error.restype = ctypes.c_char_p
    lib.lss_workspace_bytes.argtypes = [i64, i64, i64, i64, i64, ci]
    lib.lss_workspace_bytes.restype = sz
    lib.lss_set_workspace.argtypes = [vp, sz]
    lib.lss_set_workspace.restype = ci
    fwd = [vp, vp, vp, i64, i64, i64, i64, i64, i64, ci, vp, vp, vp]
    bwd = [vp, vp, vp, i64, i64, i64, i64, i64, i64, ci, vp, vp, vp, vp, vp, vp, vp]
    for name, args in (("lss_segment_attn_fwd", fwd), ("lss_segment_attn_fwd_f32", fwd),
                       ("lss_segment_attn_bwd", bwd), ("lss_segment_attn_bwd_f32", bwd),
                       ("lss_segment_attn_bwd_noalloc", bwd)):
        getattr(lib, name).argtypes = args
        getattr(lib, name).restype = ci
    f64, u64 = ctypes.c_double, ctypes.c_uint64
    lib.lss_segment_attn_fwd_dropout.argtypes = [vp, vp, vp, i64, i64, i64, i64, i64, i64, ci, f64, u64, ci, vp, vp, vp]
    lib.lss_segment_attn_bwd_dropout.argtypes = [vp, vp, vp, i64, i64, i64, i64, i64, i64, ci, f64, u64, ci,
                                                 vp, vp, vp, vp, vp, vp, vp]
    lib.lss_segment_attn_fwd_dropout.restype = ci
    lib.lss_segment_attn_bwd_dropout.restype = ci
    cu = ctypes.c_uint
    lib.lss_segment_attn_fwd_ex.argtypes = [vp, vp, vp, i64, i64, i64, i64, i64, i64, ci, f64, u64, ci, cu, vp, sz, vp, vp, vp]
    lib.lss_segment_attn_bwd_ex.argtypes = [vp, vp, vp, i64, i64, i64, i64, i64, i64, ci, f64, u64, ci, cu, vp, sz,
                                            vp, vp, vp, vp, vp, vp, vp]
    lib.lss_segment_attn_fwd_ex.restype = ci
    lib.lss_segment_attn_bwd_ex.restype = ci
    lib.lss_reduce_partials.argtypes = [vp, ci, vp, i64, i64, i64, i64, vp, vp]
    lib.lss_reduce_partials.restype = ci
    lib.lss_project_qkv.argtypes = [vp, vp, vp, i64, i64, i64, i64, i64, i64, vp, vp, vp, vp]
    lib.lss_project_qkv.restype = ci
    lib.lss_project_bwd.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i64, i64, i64, vp, vp, vp]
    lib.lss_project_bwd.restype = ci
    lib.lss_project_bwd_ex.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i64, i64, i64, cu, vp, vp, vp]
    lib.lss_project_bwd_ex.restype = ci
    lib.lss_project_bwd_weight_scratch_bytes.argtypes = [i64, i64, i64, i64, i64]
    lib.lss_project_bwd_weight_scratch_bytes.restype = sz
    lib.lss_project_bwd_weight.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, i64, i64, i64, vp, vp, vp, sz, vp]
    lib.lss_project_bwd_weight.restype = ci
    lib.lss_embed_pe_fwd.argtypes = [vp, vp, i64, i64, i64, i64, i64, vp, vp]
    lib.lss_embed_pe_bwd.argtypes = [vp, i64, i64, i64, vp, vp]
    lib.lss_residual_dropout_add.argtypes = [vp, vp, i64, i64, i64, i64, f64, u64, vp, vp]
    lib.lss_residual_dropout_add.restype = ci
    lib.lss_layernorm_fwd.argtypes = [vp, vp, vp, f64, i64, i64, vp, vp, vp, vp]
    lib.lss_layernorm_bwd_scratch_bytes.argtypes = [i64, i64]
    lib.lss_layernorm_bwd_scratch_bytes.restype = sz
    lib.lss_layernorm_bwd.argtypes = [vp, vp, vp, vp, vp, i64, i64, vp, vp, vp, vp, sz, vp]
    lib.lss_linear_fwd.argtypes = [vp, vp, i64, i64, i64, vp, vp]
    lib.lss_linear_bwd_input.argtypes = [vp, vp, i64, i64, i64, vp, vp]
    lib.lss_linear_bwd_weight_scratch_bytes.argtypes = [i64, i64, i64]
    lib.lss_linear_bwd_weight_scratch_bytes.restype = sz
    lib.lss_linear_bwd_weight.argtypes = [vp, vp, i64, i64, i64, vp, vp, sz, vp]
    lib.lss_linear_bwd_weight.restype = ci
    lib.lss_linear_gelu_fwd.argtypes = [vp, vp, i64, i64, i64, vp, vp, vp]
    lib.lss_linear_bwd_input_gelu.argtypes = [vp, vp, vp, i64, i64, i64, vp, vp]
    lib.lss_gelu_fwd.argtypes = [vp, i64, vp, vp]
    lib.lss_gelu_bwd.argtypes = [vp, vp, i64, vp, vp]
    for name in ("lss_embed_pe_fwd", "lss_embed_pe_bwd", "lss_residual_dropout_add", "lss_layernorm_fwd", "lss_layernorm_bwd", "lss_linear_fwd",
                 "lss_linear_bwd_input", "lss_linear_gelu_fwd", "lss_linear_bwd_input_gelu", "lss_gelu_fwd", "lss_gelu_bwd"):
        getattr(lib, name).restype = ci
    _lib = lib
    return lib


def _check(rc: int):
    if rc != LSS_OK:
        raise LssError(rc, load().lss_last_error().decode())


def lss_version() -> int:
    return int(load().lss_version())


def lss_last_error() -> str:
    return load().lss_last_error().decode()


def lss_workspace_bytes(l_s, l_x, B, H, d, elem_bytes=2) -> int:
    return int(load().lss_workspace_bytes(l_s, l_x, B, H, d, elem_bytes))


_ws = {}        # device index -> uint8 tensor currently handed to the library
# Outgrown buffers are kept alive, because kernels in flight may still use them and nothing here
# synchronises.  A buffer at least doubles when it grows, so together they stay below the current one.
_ws_retired = []


def lss_set_workspace(buf) -> None:
    """Hand the library a device buffer (a uint8 torch tensor) as scratch; None clears it."""
    if buf is None:
        _check(load().lss_set_workspace(None, 0))
        return
    _check(load().lss_set_workspace(buf.data_ptr(), buf.numel() * buf.element_size()))


def _ensure_workspace(l_s, l_x, B, H, d, elem_bytes, device):
    need = lss_workspace_bytes(l_s, l_x, B, H, d, elem_bytes)
    idx = device.index if device.index is not None else torch.cuda.current_device()
    cur = _ws.get(idx)
    if cur is None or cur.numel() < need:
        if cur is not None:
            _ws_retired.append(cur)
        grown = 2 * cur.numel() if cur is not None else 1 << 20
        cur = torch.empty(max(need, grown), dtype=torch.uint8, device=device)
        _ws[idx] = cur
    lss_set_workspace(cur)


def _stream_ptr(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _dims(q_seg, k, v):
    if q_seg.dim() != 4 or k.dim() != 4 or k.shape != v.shape:
        raise ValueError("q_seg, k, v must be [B, L, H, d] with k.shape == v.shape")
    B, l_s, H, d = q_seg.shape
    if k.shape[0] != B or k.shape[2] != H or k.shape[3] != d:
        raise ValueError("q_seg and k disagree on B, H or d")
    for t in (q_seg, k, v):
        if not t.is_cuda or not t.is_contiguous():
            raise ValueError("tensors must be contiguous device tensors")
    if not (q_seg.dtype == k.dtype == v.dtype) or q_seg.dtype not in (torch.bfloat16, torch.float32):
        raise ValueError("q_seg, k, v must share dtype bfloat16 or float32")
    return B, l_s, k.shape[1], H, d


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr())


def _own_workspace(workspace, need):
    """(pointer, bytes) of a caller's scratch tensor for the *_ex entry points."""
    if not workspace.is_cuda or not workspace.is_contiguous():
        raise ValueError("workspace must be a contiguous device tensor")
    nbytes = workspace.numel() * workspace.element_size()
    if nbytes < need:
        raise ValueError(f"workspace of {nbytes} bytes, need {need}")
    return _ptr(workspace), nbytes


def lss_segment_attn_fwd(q_seg, k, v, seg_offset, causal=True, out=None, lse=None, stream=None,
                         p_drop=None, seed=0, workspace=None):
    """Forward of one segment; dispatches on dtype (bf16 -> lss_segment_attn_fwd, f32 -> _f32), calls
    lss_segment_attn_fwd_dropout when p_drop is given, and lss_segment_attn_fwd_ex when `workspace` (a
    device tensor of lss_workspace_bytes() bytes used by this call alone) is given.

    Returns (out [B,l_s,H,d] in the input dtype, lse [B,H,l_s] float32).
    """
    B, l_s, l_x, H, d = _dims(q_seg, k, v)
    if out is None:
        out = torch.empty_like(q_seg)
    if lse is None:
        lse = torch.empty((B, H, l_s), dtype=torch.float32, device=q_seg.device)
    f32 = q_seg.dtype == torch.float32
    if workspace is not None:
        wp, wn = _own_workspace(workspace, lss_workspace_bytes(l_s, l_x, B, H, d, 4 if f32 else 2))
        _check(load().lss_segment_attn_fwd_ex(_ptr(q_seg), _ptr(k), _ptr(v), int(seg_offset), l_s, l_x, B, H, d,
                                              int(bool(causal)), float(p_drop or 0.0), int(seed) & (2 ** 64 - 1),
                                              4 if f32 else 2, 0, wp, wn, _ptr(out), _ptr(lse), _stream_ptr(stream)))
        return out, lse
    _ensure_workspace(l_s, l_x, B, H, d, 4 if f32 else 2, q_seg.device)
    if p_drop is not None:
        _check(load().lss_segment_attn_fwd_dropout(_ptr(q_seg), _ptr(k), _ptr(v), int(seg_offset), l_s, l_x, B, H, d,
                                                   int(bool(causal)), float(p_drop), int(seed) & (2 ** 64 - 1),
                                                   4 if f32 else 2, _ptr(out), _ptr(lse), _stream_ptr(stream)))
        return out, lse
    fn = load().lss_segment_attn_fwd_f32 if f32 else load().lss_segment_attn_fwd
    _check(fn(_ptr(q_seg), _ptr(k), _ptr(v), int(seg_offset), l_s, l_x, B, H, d, int(bool(causal)),
              _ptr(out), _ptr(lse), _stream_ptr(stream)))
    return out, lse


def lss_segment_attn_bwd(q_seg, k, v, seg_offset, out, lse, d_out, causal=True,
                         dq=None, dk_partial=None, dv_partial=None, stream=None, p_drop=None, seed=0,
                         skip_masked_tail=False, workspace=None):
    """Backward of one segment.  Returns (dq, dk_partial, dv_partial); partials are float32 [B,l_x,H,d].

    skip_masked_tail (LSS_FLAG_SKIP_MASKED_TAIL) or `workspace` select lss_segment_attn_bwd_ex."""
    B, l_s, l_x, H, d = _dims(q_seg, k, v)
    for t in (out, d_out):
        if t.shape != q_seg.shape or t.dtype != q_seg.dtype or not t.is_contiguous():
            raise ValueError("out and d_out must match q_seg in shape and dtype and be contiguous")
    if lse.shape != (B, H, l_s) or lse.dtype != torch.float32 or not lse.is_contiguous():
        raise ValueError("lse must be contiguous float32 [B, H, l_s]")
    if dq is None:
        dq = torch.empty_like(q_seg)
    if dk_partial is None:
        dk_partial = torch.empty(k.shape, dtype=torch.float32, device=k.device)
    if dv_partial is None:
        dv_partial = torch.empty(k.shape, dtype=torch.float32, device=k.device)
    f32 = q_seg.dtype == torch.float32
    if workspace is None:
        _ensure_workspace(l_s, l_x, B, H, d, 4 if f32 else 2, q_seg.device)
    if skip_masked_tail or workspace is not None:
        wp, wn = (None, 0) if workspace is None else \
            _own_workspace(workspace, lss_workspace_bytes(l_s, l_x, B, H, d, 4 if f32 else 2))
        _check(load().lss_segment_attn_bwd_ex(_ptr(q_seg), _ptr(k), _ptr(v), int(seg_offset), l_s, l_x, B, H, d,
                                              int(bool(causal)), float(p_drop or 0.0), int(seed) & (2 ** 64 - 1),
                                              4 if f32 else 2, LSS_FLAG_SKIP_MASKED_TAIL if skip_masked_tail else 0,
                                              wp, wn, _ptr(out), _ptr(lse), _ptr(d_out), _ptr(dq),
                                              _ptr(dk_partial), _ptr(dv_partial), _stream_ptr(stream)))
        return dq, dk_partial, dv_partial
    if p_drop is not None:
        _check(load().lss_segment_attn_bwd_dropout(_ptr(q_seg), _ptr(k), _ptr(v), int(seg_offset), l_s, l_x, B, H, d,
                                                   int(bool(causal)), float(p_drop), int(seed) & (2 ** 64 - 1),
                                                   4 if f32 else 2, _ptr(out), _ptr(lse), _ptr(d_out), _ptr(dq),
                                                   _ptr(dk_partial), _ptr(dv_partial), _stream_ptr(stream)))
        return dq, dk_partial, dv_partial
    fn = load().lss_segment_attn_bwd_f32 if f32 else load().lss_segment_attn_bwd
    _check(fn(_ptr(q_seg), _ptr(k), _ptr(v), int(seg_offset), l_s, l_x, B, H, d, int(bool(causal)),
              _ptr(out), _ptr(lse), _ptr(d_out), _ptr(dq), _ptr(dk_partial), _ptr(dv_partial),
              _stream_ptr(stream)))
    return dq, dk_partial, dv_partial


LSS_NOALLOC_SCRATCH_BYTES = 64 << 20


def lss_segment_attn_bwd_noalloc(q_seg, k, v, seg_offset, out, lse, d_out, causal, dq, dk_partial, dv_partial, stream=None):
    """lss_segment_attn_bwd with the library's built-in scratch buffer (bf16 only): the call itself allocates
    nothing, so every output must be passed in."""
    B, l_s, l_x, H, d = _dims(q_seg, k, v)
    if q_seg.dtype != torch.bfloat16:
        raise ValueError("bf16 only")
    for t in (out, d_out, dq):
        if t.shape != q_seg.shape or t.dtype != q_seg.dtype or not t.is_contiguous():
            raise ValueError("out, d_out and dq must match q_seg in shape and dtype and be contiguous")
    if lse.shape != (B, H, l_s) or lse.dtype != torch.float32 or not lse.is_contiguous():
        raise ValueError("lse must be contiguous float32 [B, H, l_s]")
    for t in (dk_partial, dv_partial):
        if t.shape != k.shape or t.dtype != torch.float32 or not t.is_contiguous():
            raise ValueError("partials must be contiguous float32 [B, l_x, H, d]")
    _check(load().lss_segment_attn_bwd_noalloc(_ptr(q_seg), _ptr(k), _ptr(v), int(seg_offset), l_s, l_x, B, H, d,
                                               int(bool(causal)), _ptr(out), _ptr(lse), _ptr(d_out), _ptr(dq),
                                               _ptr(dk_partial), _ptr(dv_partial), _stream_ptr(stream)))
    return dq, dk_partial, dv_partial


def lss_reduce_partials(parts, rows_valid=None, out=None, stream=None):
    """out = parts[0] + parts[1] + ... in list order; rows >= rows_valid[i] of parts[i] count as 0."""
    parts = list(parts)
    if not parts:
        raise ValueError("need at least one partial")
    B, l_x, H, d = parts[0].shape
    for p in parts:
        if p.shape != parts[0].shape or p.dtype != torch.float32 or not p.is_cuda or not p.is_contiguous():
            raise ValueError("partials must be contiguous float32 device tensors of one shape")
    if out is None:
        out = torch.empty_like(parts[0])
    arr = (ctypes.c_void_p * len(parts))(*[p.data_ptr() for p in parts])
    rv = None
    if rows_valid is not None:
        if len(rows_valid) != len(parts):
            raise ValueError("rows_valid must have one entry per partial")
        rv = (ctypes.c_int64 * len(parts))(*[int(x) for x in rows_valid])
    _check(load().lss_reduce_partials(arr, len(parts), rv, l_x, B, H, d, _ptr(out), _stream_ptr(stream)))
    return out


def lss_project_qkv(x, w_q, w_kv, seg_offset, l_s, H, q_seg=None, k=None, v=None, stream=None):
    """Q_i = x_i W_q, K = x W_k, V = x W_v.  x [B,l_x,E] bf16, w_q [E,E], w_kv [E,2E] = [W_k | W_v].

    Returns (q_seg [B,l_s,H,d], k [B,l_x,H,d], v [B,l_x,H,d]) in bf16.
    """
    if x.dim() != 3 or x.dtype != torch.bfloat16:
        raise ValueError("x must be bf16 [B, l_x, E]")
    B, l_x, E = x.shape
    if E % H:
        raise ValueError("E must be a multiple of H")
    d = E // H
    if tuple(w_q.shape) != (E, E) or tuple(w_kv.shape) != (E, 2 * E):
        raise ValueError("w_q must be [E, E] and w_kv [E, 2E]")
    if q_seg is None:
        q_seg = torch.empty((B, l_s, H, d), dtype=torch.bfloat16, device=x.device)
    if k is None:
        k = torch.empty((B, l_x, H, d), dtype=torch.bfloat16, device=x.device)
    if v is None:
        v = torch.empty((B, l_x, H, d), dtype=torch.bfloat16, device=x.device)
    if tuple(q_seg.shape) != (B, l_s, H, d) or tuple(k.shape) != (B, l_x, H, d) or tuple(v.shape) != (B, l_x, H, d):
        raise ValueError("output shapes disagree with x, l_s and H")
    for t in (x, w_q, w_kv, q_seg, k, v):
        if not t.is_cuda or not t.is_contiguous() or t.dtype != torch.bfloat16:
            raise ValueError("tensors must be contiguous bf16 device tensors")
    _check(load().lss_project_qkv(_ptr(x), _ptr(w_q), _ptr(w_kv), int(seg_offset), int(l_s), l_x, B, H, d,
                                  _ptr(q_seg), _ptr(k), _ptr(v), _stream_ptr(stream)))
    return q_seg, k, v


def lss_project_bwd(dq, dk_partial, dv_partial, w_q, w_kv, rows_valid=None, dx_q=None, dx_partial=None, stream=None,
                    skip_masked_tail=False):
    """dx_q = dQ_i W_q^T [B,l_s,E] and dx_partial = dK_part W_k^T + dV_part W_v^T [B,l_x,E], both float32.

    skip_masked_tail selects lss_project_bwd_ex with LSS_FLAG_SKIP_MASKED_TAIL."""
    if dq.dim() != 4 or dk_partial.dim() != 4 or dk_partial.shape != dv_partial.shape:
        raise ValueError("dq must be [B,l_s,H,d]; partials [B,l_x,H,d]")
    B, l_s, H, d = dq.shape
    l_x, E = dk_partial.shape[1], H * d
    if tuple(dk_partial.shape) != (B, l_x, H, d) or tuple(w_q.shape) != (E, E) or tuple(w_kv.shape) != (E, 2 * E):
        raise ValueError("shapes disagree")
    if rows_valid is None:
        rows_valid = l_x
    if dx_q is None:
        dx_q = torch.empty((B, l_s, E), dtype=torch.float32, device=dq.device)
    if dx_partial is None:
        dx_partial = torch.empty((B, l_x, E), dtype=torch.float32, device=dq.device)
    if tuple(dx_q.shape) != (B, l_s, E) or tuple(dx_partial.shape) != (B, l_x, E):
        raise ValueError("output shapes disagree")
    for t, dt in ((dq, torch.bfloat16), (w_q, torch.bfloat16), (w_kv, torch.bfloat16), (dk_partial, torch.float32),
                  (dv_partial, torch.float32), (dx_q, torch.float32), (dx_partial, torch.float32)):
        if not t.is_cuda or not t.is_contiguous() or t.dtype != dt:
            raise ValueError("tensors must be contiguous device tensors of the documented types")
    if skip_masked_tail:
        _check(load().lss_project_bwd_ex(_ptr(dq), _ptr(dk_partial), _ptr(dv_partial), _ptr(w_q), _ptr(w_kv), l_s, l_x,
                                         int(rows_valid), B, H, d, LSS_FLAG_SKIP_MASKED_TAIL, _ptr(dx_q), _ptr(dx_partial),
                                         _stream_ptr(stream)))
        return dx_q, dx_partial
    _check(load().lss_project_bwd(_ptr(dq), _ptr(dk_partial), _ptr(dv_partial), _ptr(w_q), _ptr(w_kv), l_s, l_x,
                                  int(rows_valid), B, H, d, _ptr(dx_q), _ptr(dx_partial), _stream_ptr(stream)))
    return dx_q, dx_partial


def lss_project_bwd_weight_scratch_bytes(l_s, l_x, B, H, d):
    return int(load().lss_project_bwd_weight_scratch_bytes(int(l_s), int(l_x), int(B), int(H), int(d)))


def lss_project_bwd_weight(x, dq, dk_partial, dv_partial, seg_offset, rows_valid=None, dw_q=None, dw_kv=None,
                           scratch=None, stream=None):
    """One segment's share of dW_q [E,E] = sum_b x_i^T dQ_i and dW_kv [E,2E] = sum_b x^T [dK_part | dV_part], float32."""
    if x.dim() != 3 or dq.dim() != 4 or dk_partial.dim() != 4 or dk_partial.shape != dv_partial.shape:
        raise ValueError("x must be [B,l_x,E]; dq [B,l_s,H,d]; partials [B,l_x,H,d]")
    B, l_s, H, d = dq.shape
    l_x, E = x.shape[1], H * d
    if tuple(x.shape) != (B, l_x, E) or tuple(dk_partial.shape) != (B, l_x, H, d):
        raise ValueError("shapes disagree")
    if rows_valid is None:
        rows_valid = l_x
    for t, dt in ((x, torch.bfloat16), (dq, torch.bfloat16), (dk_partial, torch.float32), (dv_partial, torch.float32)):
        if not t.is_cuda or not t.is_contiguous() or t.dtype != dt:
            raise ValueError("tensors must be contiguous device tensors of the documented types")
    if dw_q is None:
        dw_q = torch.empty((E, E), dtype=torch.float32, device=x.device)
    if dw_kv is None:
        dw_kv = torch.empty((E, 2 * E), dtype=torch.float32, device=x.device)
    if tuple(dw_q.shape) != (E, E) or tuple(dw_kv.shape) != (E, 2 * E) or dw_q.dtype != torch.float32 or dw_kv.dtype != torch.float32:
        raise ValueError("dw_q must be float32 [E, E] and dw_kv float32 [E, 2E]")
    if scratch is None:
        scratch = torch.empty((max(16, lss_project_bwd_weight_scratch_bytes(l_s, l_x, B, H, d)),), dtype=torch.uint8, device=x.device)
    _check(load().lss_project_bwd_weight(_ptr(x), _ptr(dq), _ptr(dk_partial), _ptr(dv_partial), int(seg_offset), l_s, l_x,
                                         int(rows_valid), B, H, d, _ptr(dw_q), _ptr(dw_kv), _ptr(scratch), scratch.numel(),
                                         _stream_ptr(stream)))
    return dw_q, dw_kv


def _dev(t, dtype, what):
    if not t.is_cuda or not t.is_contiguous() or t.dtype != dtype:
        raise ValueError(f"{what} must be a contiguous {dtype} device tensor")


def _out(t, shape, dtype, like):
    if t is None:
        return torch.empty(shape, dtype=dtype, device=like.device)
    if tuple(t.shape) != tuple(shape):
        raise ValueError(f"output has shape {tuple(t.shape)}, expected {tuple(shape)}")
    _dev(t, dtype, "output")
    return t


def lss_embed_pe_fwd(tok, pe_table, seg_offset, x=None, stream=None):
    """x[b, r] = tok[b, r] + pe_table[seg_offset + r].  tok [B,l_s,E] bf16, pe_table [l_x,E] bf16."""
    if tok.dim() != 3 or pe_table.dim() != 2 or pe_table.shape[1] != tok.shape[2]:
        raise ValueError("tok must be [B, l_s, E] and pe_table [l_x, E]")
    B, l_s, E = tok.shape
    _dev(tok, torch.bfloat16, "tok"); _dev(pe_table, torch.bfloat16, "pe_table")
    x = _out(x, (B, l_s, E), torch.bfloat16, tok)
    _check(load().lss_embed_pe_fwd(_ptr(tok), _ptr(pe_table), int(seg_offset), l_s, pe_table.shape[0], B, E, _ptr(x),
                                   _stream_ptr(stream)))
    return x


def lss_embed_pe_bwd(dx, dpe_rows=None, stream=None):
    """dpe_rows[r] = sum_b dx[b, r], float32 [l_s, E]: the gradient of the segment's rows of the table."""
    if dx.dim() != 3:
        raise ValueError("dx must be [B, l_s, E]")
    B, l_s, E = dx.shape
    _dev(dx, torch.bfloat16, "dx")
    dpe_rows = _out(dpe_rows, (l_s, E), torch.float32, dx)
    _check(load().lss_embed_pe_bwd(_ptr(dx), l_s, B, E, _ptr(dpe_rows), _stream_ptr(stream)))
    return dpe_rows


def lss_residual_dropout_add(x, delta, seg_offset, p_drop=0.0, seed=0, out=None, stream=None):
    """out = x + dropout(delta) on a segment's rows [B, l_s, E] bf16; x may be None (zeros)."""
    if delta.dim() != 3 or (x is not None and x.shape != delta.shape):
        raise ValueError("delta must be [B, l_s, E] and x, if given, of the same shape")
    B, l_s, E = delta.shape
    _dev(delta, torch.bfloat16, "delta")
    if x is not None:
        _dev(x, torch.bfloat16, "x")
    out = _out(out, delta.shape, torch.bfloat16, delta)
    _check(load().lss_residual_dropout_add(_ptr(x) if x is not None else None, _ptr(delta), int(seg_offset), l_s, B, E,
                                           float(p_drop), int(seed), _ptr(out), _stream_ptr(stream)))
    return out


def lss_layernorm_fwd(x, gamma, beta, eps=1e-5, y=None, mean=None, rstd=None, stream=None):
    """Row-wise layer normalisation of x [..., E] bf16; returns (y bf16, mean, rstd float32 [rows])."""
    E = x.shape[-1]
    rows = x.numel() // E if E else 0
    _dev(x, torch.bfloat16, "x"); _dev(gamma, torch.float32, "gamma"); _dev(beta, torch.float32, "beta")
    if gamma.numel() != E or beta.numel() != E:
        raise ValueError("gamma and beta must have E elements")
    y = _out(y, x.shape, torch.bfloat16, x)
    mean = _out(mean, (rows,), torch.float32, x)
    rstd = _out(rstd, (rows,), torch.float32, x)
    _check(load().lss_layernorm_fwd(_ptr(x), _ptr(gamma), _ptr(beta), float(eps), rows, E, _ptr(y), _ptr(mean), _ptr(rstd),
                                    _stream_ptr(stream)))
    return y, mean, rstd


def lss_layernorm_bwd_scratch_bytes(rows, E):
    return int(load().lss_layernorm_bwd_scratch_bytes(int(rows), int(E)))


def lss_layernorm_bwd(x, gamma, mean, rstd, dy, dx=None, dgamma=None, dbeta=None, scratch=None, stream=None):
    """Backward of lss_layernorm_fwd: returns (dx bf16, dgamma, dbeta float32 [E]).

    `scratch` is a uint8 device tensor of at least lss_layernorm_bwd_scratch_bytes(rows, E) bytes
    (allocated here if absent).
    """
    E = x.shape[-1]
    rows = x.numel() // E if E else 0
    for t, dt, nm in ((x, torch.bfloat16, "x"), (dy, torch.bfloat16, "dy"), (gamma, torch.float32, "gamma"),
                      (mean, torch.float32, "mean"), (rstd, torch.float32, "rstd")):
        _dev(t, dt, nm)
    if dy.shape != x.shape or gamma.numel() != E or mean.numel() != rows or rstd.numel() != rows:
        raise ValueError("shapes disagree")
    dx = _out(dx, x.shape, torch.bfloat16, x)
    dgamma = _out(dgamma, (E,), torch.float32, x)
    dbeta = _out(dbeta, (E,), torch.float32, x)
    need = lss_layernorm_bwd_scratch_bytes(rows, E)
    if scratch is None:
        scratch = torch.empty((max(need, 16),), dtype=torch.uint8, device=x.device)
    _dev(scratch, torch.uint8, "scratch")
    _check(load().lss_layernorm_bwd(_ptr(x), _ptr(gamma), _ptr(mean), _ptr(rstd), _ptr(dy), rows, E, _ptr(dx), _ptr(dgamma),
                                    _ptr(dbeta), _ptr(scratch), scratch.numel(), _stream_ptr(stream)))
    return dx, dgamma, dbeta


def lss_linear_fwd(a, w, c=None, stream=None):
    """c = a w.  a [..., K] bf16, w [K, N] bf16 -> c [..., N] bf16."""
    K, N = w.shape
    if a.shape[-1] != K:
        raise ValueError("a's last dimension must equal w's rows")
    _dev(a, torch.bfloat16, "a"); _dev(w, torch.bfloat16, "w")
    rows = a.numel() // K
    c = _out(c, (*a.shape[:-1], N), torch.bfloat16, a)
    _check(load().lss_linear_fwd(_ptr(a), _ptr(w), rows, K, N, _ptr(c), _stream_ptr(stream)))
    return c


def lss_linear_bwd_input(dc, w, da=None, stream=None):
    """da = dc w^T.  dc [..., N] bf16, w [K, N] bf16 -> da [..., K] bf16."""
    K, N = w.shape
    if dc.shape[-1] != N:
        raise ValueError("dc's last dimension must equal w's columns")
    _dev(dc, torch.bfloat16, "dc"); _dev(w, torch.bfloat16, "w")
    rows = dc.numel() // N
    da = _out(da, (*dc.shape[:-1], K), torch.bfloat16, dc)
    _check(load().lss_linear_bwd_input(_ptr(dc), _ptr(w), rows, K, N, _ptr(da), _stream_ptr(stream)))
    return da


def lss_linear_bwd_weight_scratch_bytes(rows, K, N):
    return int(load().lss_linear_bwd_weight_scratch_bytes(int(rows), int(K), int(N)))


def lss_linear_bwd_weight(a, dc, dw=None, scratch=None, stream=None):
    """dw = a^T dc over every row.  a [..., K], dc [..., N] bf16 -> dw [K, N] float32.

    `scratch` is a uint8 device tensor of at least lss_linear_bwd_weight_scratch_bytes(rows, K, N)
    bytes (allocated here if absent)."""
    K, N = a.shape[-1], dc.shape[-1]
    if a.shape[:-1] != dc.shape[:-1]:
        raise ValueError("a and dc must have the same rows")
    _dev(a, torch.bfloat16, "a"); _dev(dc, torch.bfloat16, "dc")
    rows = a.numel() // K if K else 0
    dw = _out(dw, (K, N), torch.float32, a)
    need = lss_linear_bwd_weight_scratch_bytes(rows, K, N)
    if scratch is None:
        scratch = torch.empty((max(need, 16),), dtype=torch.uint8, device=a.device)
    _dev(scratch, torch.uint8, "scratch")
    _check(load().lss_linear_bwd_weight(_ptr(a), _ptr(dc), rows, K, N, _ptr(dw), _ptr(scratch), scratch.numel(),
                                        _stream_ptr(stream)))
    return dw


def lss_linear_gelu_fwd(a, w, u=None, g=None, stream=None):
    """u = a w and g = GeLU(u) in one kernel; returns (u, g), both [..., N] bf16."""
    K, N = w.shape
    if a.shape[-1] != K:
        raise ValueError("a's last dimension must equal w's rows")
    _dev(a, torch.bfloat16, "a"); _dev(w, torch.bfloat16, "w")
    u = _out(u, (*a.shape[:-1], N), torch.bfloat16, a)
    g = _out(g, (*a.shape[:-1], N), torch.bfloat16, a)
    _check(load().lss_linear_gelu_fwd(_ptr(a), _ptr(w), a.numel() // K, K, N, _ptr(u), _ptr(g), _stream_ptr(stream)))
    return u, g


def lss_linear_bwd_input_gelu(dc, w, u, du=None, stream=None):
    """du = (dc w^T) * GeLU'(u) in one kernel.  dc [..., N], w [K, N], u [..., K] -> du [..., K], bf16."""
    K, N = w.shape
    if dc.shape[-1] != N or u.shape[-1] != K or u.numel() // K != dc.numel() // N:
        raise ValueError("shapes disagree")
    for t, nm in ((dc, "dc"), (w, "w"), (u, "u")):
        _dev(t, torch.bfloat16, nm)
    du = _out(du, u.shape, torch.bfloat16, u)
    _check(load().lss_linear_bwd_input_gelu(_ptr(dc), _ptr(w), _ptr(u), dc.numel() // N, K, N, _ptr(du), _stream_ptr(stream)))
    return du


def lss_gelu_fwd(u, g=None, stream=None):
    """g = GeLU(u) = u Phi(u), elementwise, bf16."""
    _dev(u, torch.bfloat16, "u")
    g = _out(g, u.shape, torch.bfloat16, u)
    _check(load().lss_gelu_fwd(_ptr(u), u.numel(), _ptr(g), _stream_ptr(stream)))
    return g


def lss_gelu_bwd(u, dg, du=None, stream=None):
    """du = dg * GeLU'(u), elementwise, bf16."""
    _dev(u, torch.bfloat16, "u"); _dev(dg, torch.bfloat16, "dg")
    if dg.shape != u.shape:
        raise ValueError("u and dg must have the same shape")
    du = _out(du, u.shape, torch.bfloat16, u)
    _check(load().lss_gelu_bwd(_ptr(u), _ptr(dg), u.numel(), _ptr(du), _stream_ptr(stream)))
    return du
