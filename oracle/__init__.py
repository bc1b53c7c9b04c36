"""fp64 CPU oracle for segment attention (LSS Transformer, Section 3, Eq. 2).

TEST INFRASTRUCTURE ONLY.  This package is the checker for the HIP library:
it may be imported by the tests, by the smoke entry and by the benchmark's
``cpu_baseline`` leg, and by nothing else.  It imports nothing from the HIP
package and shares no code with it.

The arithmetic lives in ``lss_oracle.c`` (plain loops in double precision);
this module only compiles that file with gcc, loads it with ctypes and
marshals numpy arrays.  Activations are ``[B, L, H, d]`` float64, C-contiguous;
``lse`` is ``[B, H, l_s]``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "lss_oracle.c"
_LIB = _HERE / "liblss_oracle.so"
_lib = None


def build(force: bool = False) -> Path:
    """Compile the oracle with gcc (-O2, OpenMP).  Returns the library path."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = _LIB.with_suffix(f".so.tmp{os.getpid()}")
        subprocess.run(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra",
             "-o", str(tmp), str(_SRC), "-lm"],
            check=True,
        )
        os.replace(tmp, _LIB)
    return _LIB


def build_sanitized() -> Path:
    """Compile lss_oracle.c together with san_check.c under AddressSanitizer and UndefinedBehaviorSanitizer
    (host code only; the sanitizer runtimes are linked statically, so the program needs no preloading)
    into a stand-alone checker.  Returns the program's path; run it, exit status 0 means clean."""
    exe = _SRC.with_name("san_check")
    tmp = exe.with_suffix(f".tmp{os.getpid()}")
    subprocess.run(
        ["gcc", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
         "-static-libasan", "-static-libubsan", "-fopenmp", "-Wall", "-Wextra",
         "-o", str(tmp), str(_SRC.with_name("san_check.c")), str(_SRC), "-lm"],
        check=True,
    )
    os.replace(tmp, exe)
    return exe


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(str(build()))
        i64, dp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
        lib.lss_oracle_segment_fwd.argtypes = [dp, dp, dp, i64, i64, i64, i64, i64, i64, ci, dp, dp]
        lib.lss_oracle_segment_bwd.argtypes = [dp, dp, dp, i64, i64, i64, i64, i64, i64, ci, dp, dp, dp, dp]
        lib.lss_oracle_segment_weights.argtypes = [dp, dp, i64, i64, i64, i64, i64, i64, ci, dp]
        lib.lss_oracle_reduce_partials.argtypes = [dp, ci, i64, dp]
        f64, u64 = ctypes.c_double, ctypes.c_uint64
        lib.lss_oracle_segment_fwd_dropout.argtypes = [dp, dp, dp, i64, i64, i64, i64, i64, i64, ci, f64, u64, dp, dp]
        lib.lss_oracle_segment_bwd_dropout.argtypes = [dp, dp, dp, i64, i64, i64, i64, i64, i64, ci, f64, u64, dp, dp, dp, dp]
        lib.lss_oracle_dropout_mask.argtypes = [f64, u64, i64, i64, i64, i64, i64, dp]
        lib.lss_oracle_activation_keep.argtypes = [f64, u64, i64, i64, i64, i64, dp]
        for f in (lib.lss_oracle_segment_fwd_dropout, lib.lss_oracle_segment_bwd_dropout, lib.lss_oracle_dropout_mask,
                  lib.lss_oracle_activation_keep):
            f.restype = ci
        for f in (lib.lss_oracle_segment_fwd, lib.lss_oracle_segment_bwd,
                  lib.lss_oracle_segment_weights, lib.lss_oracle_reduce_partials,
                  lib.lss_oracle_threads):
            f.restype = ci
        _lib = lib
    return _lib


def threads() -> int:
    """Number of OpenMP threads the oracle will use."""
    return int(_load().lss_oracle_threads())


def _f64(a, shape=None):
    a = np.ascontiguousarray(a, dtype=np.float64)
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {tuple(a.shape)}")
    return a


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _dims(q_seg, k, v):
    if q_seg.ndim != 4 or k.ndim != 4 or k.shape != v.shape:
        raise ValueError("q_seg, k, v must be [B, L, H, d] with k.shape == v.shape")
    B, l_s, H, d = q_seg.shape
    if k.shape[0] != B or k.shape[2] != H or k.shape[3] != d:
        raise ValueError("q_seg and k disagree on B, H or d")
    return B, l_s, k.shape[1], H, d


def segment_fwd(q_seg, k, v, seg_offset: int, causal: bool = True):
    """Eq. 2 for one segment.  Returns (out [B,l_s,H,d], lse [B,H,l_s])."""
    q_seg, k, v = _f64(q_seg), _f64(k), _f64(v)
    B, l_s, l_x, H, d = _dims(q_seg, k, v)
    out = np.empty((B, l_s, H, d), dtype=np.float64)
    lse = np.empty((B, H, l_s), dtype=np.float64)
    rc = _load().lss_oracle_segment_fwd(_p(q_seg), _p(k), _p(v), seg_offset, l_s, l_x, B, H, d,
                                        int(bool(causal)), _p(out), _p(lse))
    if rc != 0:
        raise ValueError(f"lss_oracle_segment_fwd rejected the shape (rc={rc})")
    return out, lse


def segment_bwd(q_seg, k, v, d_out, seg_offset: int, causal: bool = True):
    """Gradient of Eq. 2 for one segment.

    Returns (dq [B,l_s,H,d], dk_partial [B,l_x,H,d], dv_partial [B,l_x,H,d]).
    """
    q_seg, k, v = _f64(q_seg), _f64(k), _f64(v)
    B, l_s, l_x, H, d = _dims(q_seg, k, v)
    d_out = _f64(d_out, q_seg.shape)
    dq = np.empty_like(q_seg)
    dk = np.empty_like(k)
    dv = np.empty_like(k)
    rc = _load().lss_oracle_segment_bwd(_p(q_seg), _p(k), _p(v), seg_offset, l_s, l_x, B, H, d,
                                        int(bool(causal)), _p(d_out), _p(dq), _p(dk), _p(dv))
    if rc != 0:
        raise ValueError(f"lss_oracle_segment_bwd failed (rc={rc})")
    return dq, dk, dv


def segment_weights(q_seg, k, seg_offset: int, causal: bool = True):
    """The segment's softmax rows (partial A_w): [B, H, l_s, l_x], masked entries 0."""
    q_seg, k = _f64(q_seg), _f64(k)
    B, l_s, l_x, H, d = _dims(q_seg, k, k)
    P = np.empty((B, H, l_s, l_x), dtype=np.float64)
    rc = _load().lss_oracle_segment_weights(_p(q_seg), _p(k), seg_offset, l_s, l_x, B, H, d,
                                            int(bool(causal)), _p(P))
    if rc != 0:
        raise ValueError(f"lss_oracle_segment_weights rejected the shape (rc={rc})")
    return P


def segment_fwd_dropout(q_seg, k, v, seg_offset: int, causal: bool, p: float, seed: int):
    """Eq. 2 with dropout on the weights (Section 2.2): returns (out, lse); lse is that of the scores."""
    q_seg, k, v = _f64(q_seg), _f64(k), _f64(v)
    B, l_s, l_x, H, d = _dims(q_seg, k, v)
    out = np.empty((B, l_s, H, d), dtype=np.float64)
    lse = np.empty((B, H, l_s), dtype=np.float64)
    rc = _load().lss_oracle_segment_fwd_dropout(_p(q_seg), _p(k), _p(v), seg_offset, l_s, l_x, B, H, d,
                                                int(bool(causal)), float(p), int(seed), _p(out), _p(lse))
    if rc != 0:
        raise ValueError(f"lss_oracle_segment_fwd_dropout rejected the arguments (rc={rc})")
    return out, lse


def segment_bwd_dropout(q_seg, k, v, d_out, seg_offset: int, causal: bool, p: float, seed: int):
    """Gradient of the forward with dropout, same mask.  Returns (dq, dk_partial, dv_partial)."""
    q_seg, k, v = _f64(q_seg), _f64(k), _f64(v)
    B, l_s, l_x, H, d = _dims(q_seg, k, v)
    d_out = _f64(d_out, q_seg.shape)
    dq, dk, dv = np.empty_like(q_seg), np.empty_like(k), np.empty_like(k)
    rc = _load().lss_oracle_segment_bwd_dropout(_p(q_seg), _p(k), _p(v), seg_offset, l_s, l_x, B, H, d,
                                                int(bool(causal)), float(p), int(seed), _p(d_out), _p(dq), _p(dk), _p(dv))
    if rc != 0:
        raise ValueError(f"lss_oracle_segment_bwd_dropout failed (rc={rc})")
    return dq, dk, dv


def dropout_mask(p: float, seed: int, seg_offset: int, l_s: int, l_x: int, B: int, H: int):
    """Keep mask of a segment's weights: uint8 [B, H, l_s, l_x], 1 = kept (all key positions, masked or not)."""
    mask = np.empty((B, H, l_s, l_x), dtype=np.uint8)
    rc = _load().lss_oracle_dropout_mask(float(p), int(seed), seg_offset, l_s, l_x, B, H, _p(mask))
    if rc != 0:
        raise ValueError(f"lss_oracle_dropout_mask rejected the arguments (rc={rc})")
    return mask


def reduce_partials(parts):
    """Segment sum of per-segment partials, in list order (Fig. 2(v) reduce-scatter arithmetic)."""
    parts = [_f64(p) for p in parts]
    if not parts:
        raise ValueError("need at least one partial")
    out = np.empty_like(parts[0])
    arr = (ctypes.c_void_p * len(parts))(*[p.ctypes.data for p in parts])
    rc = _load().lss_oracle_reduce_partials(arr, len(parts), out.size, _p(out))
    if rc != 0:
        raise ValueError("lss_oracle_reduce_partials failed")
    return out


# ---- the linear maps either side of the segment attention (fused-communication form) ----------
# Section 2.2 gives Q, K and V only as linear maps of x with the shape of x; the
# reading taken here is Q = x W_q, K = x W_k, V = x W_v with square E_m x E_m weights and no bias.
# Section 3, Principle 3 and Fig. 2(ii): a segment projects its query from its own rows x_i, and
# the key and value from the gathered sequence x.  W_kv holds [W_k | W_v] side by side (E_m x 2E_m).
# Head h of a projected row is its columns [h d, (h+1) d), as in the attention functions above.
# Plain numpy float64 matrix products; nothing is blocked or fused.

def project_qkv(x, w_q, w_kv, seg_offset: int, l_s: int, H: int):
    """Q_i = x_i W_q, K = x W_k, V = x W_v.  x [B,l_x,E]; returns q_seg [B,l_s,H,d], k, v [B,l_x,H,d]."""
    x, w_q, w_kv = _f64(x), _f64(w_q), _f64(w_kv)
    B, l_x, E = x.shape
    if w_q.shape != (E, E) or w_kv.shape != (E, 2 * E) or E % H:
        raise ValueError("weights must be [E,E] and [E,2E], E a multiple of H")
    if not (0 <= seg_offset and seg_offset + l_s <= l_x):
        raise ValueError("segment outside the sequence")
    d = E // H
    x_i = x[:, seg_offset:seg_offset + l_s, :]
    q = np.matmul(x_i, w_q).reshape(B, l_s, H, d)
    k = np.matmul(x, w_kv[:, :E]).reshape(B, l_x, H, d)
    v = np.matmul(x, w_kv[:, E:]).reshape(B, l_x, H, d)
    return q, k, v


def project_bwd(dq, dk_partial, dv_partial, w_q, w_kv):
    """Gradients with respect to the projections' inputs, for one segment.

    dx_q [B,l_s,E] = dQ_i W_q^T is the gradient reaching the segment's own rows x_i through the
    query; dx_partial [B,l_x,E] = dK_part W_k^T + dV_part W_v^T is this segment's contribution to
    the gradient of the gathered x, the quantity the reduce-scatter of Fig. 2(v) sums over segments.
    """
    dq, dk, dv = _f64(dq), _f64(dk_partial), _f64(dv_partial)
    w_q, w_kv = _f64(w_q), _f64(w_kv)
    B, l_s, H, d = dq.shape
    E = H * d
    l_x = dk.shape[1]
    if dk.shape != (B, l_x, H, d) or dv.shape != dk.shape or w_q.shape != (E, E) or w_kv.shape != (E, 2 * E):
        raise ValueError("shapes disagree")
    dx_q = np.matmul(dq.reshape(B, l_s, E), w_q.T)
    dx_part = np.matmul(dk.reshape(B, l_x, E), w_kv[:, :E].T) + np.matmul(dv.reshape(B, l_x, E), w_kv[:, E:].T)
    return dx_q, dx_part


def project_bwd_weight(x, dq, dk_partial, dv_partial, seg_offset: int):
    """One segment's contribution to the gradients of the projection weights:
    dW_q [E,E] = sum_b x_i^T dQ_i and dW_kv [E,2E] = sum_b x^T [dK_part | dV_part] (the segment
    projects K and V of the whole gathered x itself, Fig. 2(ii), so its share of dW_k, dW_v runs over
    all l_x rows).  The gradient averaging over the sequence-parallel group (Section 4) adds the
    segments' contributions."""
    x, dq, dk, dv = _f64(x), _f64(dq), _f64(dk_partial), _f64(dv_partial)
    B, l_s, H, d = dq.shape
    E = H * d
    l_x = x.shape[1]
    if x.shape != (B, l_x, E) or dk.shape != (B, l_x, H, d) or dv.shape != dk.shape:
        raise ValueError("shapes disagree")
    if not (0 <= seg_offset and seg_offset + l_s <= l_x):
        raise ValueError("segment outside the sequence")
    x_i = x[:, seg_offset:seg_offset + l_s, :].reshape(B * l_s, E)
    dw_q = np.matmul(x_i.T, dq.reshape(B * l_s, E))
    xf = x.reshape(B * l_x, E)
    dw_kv = np.concatenate([np.matmul(xf.T, dk.reshape(B * l_x, E)), np.matmul(xf.T, dv.reshape(B * l_x, E))], axis=1)
    return dw_q, dw_kv


# ---- the segment-local remainder of a layer (Section 3, Principles 1 and 2) ----------------------
# Everything except the self-attention is computed independently per sequence segment: positional
# embedding (a segment looks up only its own contiguous rows of the table), layer normalisation,
# residual connections, and the feed-forward unit linear -> GeLU -> linear, whose matrix products
# are row-distributed (Principle 1).  The paper names these operations without formulas; the
# readings taken are the standard ones of the GPT models it trains (Section 5.1):
#   layer normalisation over the E_m columns of a row with learned scale and shift,
#       y = (x - mean) / sqrt(var + eps) * gamma + beta,  var the biased variance;
#   GeLU(u) = u Phi(u) with the exact normal distribution function;
#   feed-forward y = GeLU(h W_1) W_2, no bias (none is mentioned), D_inner columns in between.
#   residual connection with dropout on the branch (Principle 1 lists dropout among the operations
#       that act on segments independently): out = x + dropout(delta), inverted dropout as for the
#       attention weights, the keep decision of element (batch b, global row g, column c) drawn by
#       the same generator with (batch*head, row, key) := (b, g, c) -- a function of the position in
#       the whole sequence, so the segments' results concatenate to the sequential one.
# Plain numpy float64; nothing blocked or fused.

def embed_pe(tok, pe_table, seg_offset: int):
    """x_i = tok_i + PE[seg_offset : seg_offset + l_s]  (Principle 2).  tok [B,l_s,E], pe_table [l_x,E]."""
    tok, pe_table = _f64(tok), _f64(pe_table)
    l_s = tok.shape[1]
    if not (0 <= seg_offset and seg_offset + l_s <= pe_table.shape[0]) or tok.shape[2] != pe_table.shape[1]:
        raise ValueError("segment outside the table, or widths disagree")
    return tok + pe_table[None, seg_offset:seg_offset + l_s, :]


def embed_pe_bwd(dx):
    """Gradient of the segment's rows of the table: the sum of dx over the batch, [l_s, E].
    (The gradient of tok is dx itself.)"""
    return _f64(dx).sum(axis=0)


def residual_dropout_add(x, delta, seg_offset: int, p: float = 0.0, seed: int = 0):
    """out = x + dropout(delta) on a segment's rows [B, l_s, E] (x may be None: the dropout alone).
    Being linear and diagonal in delta, the same call maps d out to d delta."""
    delta = _f64(delta)
    B, l_s, E = delta.shape
    keep = np.empty((B, l_s, E), dtype=np.uint8)
    rc = _load().lss_oracle_activation_keep(float(p), int(seed), int(seg_offset), l_s, E, B, _p(keep))
    if rc != 0:
        raise ValueError(f"lss_oracle_activation_keep rejected the arguments (rc={rc})")
    y = delta * keep / (1.0 - p)
    return y if x is None else _f64(x, delta.shape) + y


def layernorm_fwd(x, gamma, beta, eps: float = 1e-5):
    """Row-wise layer normalisation.  x [..., E].  Returns (y, mean [...], rstd [...])."""
    x, gamma, beta = _f64(x), _f64(gamma), _f64(beta)
    mean = x.mean(axis=-1)
    var = ((x - mean[..., None]) ** 2).mean(axis=-1)
    rstd = 1.0 / np.sqrt(var + eps)
    y = (x - mean[..., None]) * rstd[..., None] * gamma + beta
    return y, mean, rstd


def layernorm_bwd(x, gamma, dy, eps: float = 1e-5):
    """Gradients of layernorm_fwd: (dx like x, dgamma [E], dbeta [E])."""
    x, gamma, dy = _f64(x), _f64(gamma), _f64(dy)
    E = x.shape[-1]
    mean = x.mean(axis=-1, keepdims=True)
    var = ((x - mean) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xh = (x - mean) * rstd
    g = dy * gamma
    dx = rstd * (g - g.mean(axis=-1, keepdims=True) - xh * (g * xh).mean(axis=-1, keepdims=True))
    dgamma = (dy * xh).reshape(-1, E).sum(axis=0)
    dbeta = dy.reshape(-1, E).sum(axis=0)
    return dx, dgamma, dbeta


def gelu(u):
    """GeLU(u) = u Phi(u), Phi the standard normal distribution function."""
    from math import erf
    u = _f64(u)
    return u * 0.5 * (1.0 + np.vectorize(erf)(u / np.sqrt(2.0)))


def gelu_grad(u):
    """d GeLU / du = Phi(u) + u phi(u)."""
    from math import erf
    u = _f64(u)
    return 0.5 * (1.0 + np.vectorize(erf)(u / np.sqrt(2.0))) + u * np.exp(-0.5 * u * u) / np.sqrt(2.0 * np.pi)


def ffn_fwd(h, w1, w2):
    """Feed-forward unit on a segment's rows (Principle 1): u = h W_1, y = GeLU(u) W_2.
    h [B,l_s,E], w1 [E,Di], w2 [Di,E].  Returns (y, u)."""
    h, w1, w2 = _f64(h), _f64(w1), _f64(w2)
    u = np.matmul(h, w1)
    return np.matmul(gelu(u), w2), u


def ffn_bwd(dy, u, w1, w2):
    """Gradient of ffn_fwd with respect to h: dh = ((dy W_2^T) * GeLU'(u)) W_1^T."""
    dy, u, w1, w2 = _f64(dy), _f64(u), _f64(w1), _f64(w2)
    return np.matmul(np.matmul(dy, w2.T) * gelu_grad(u), w1.T)


def linear_bwd_weight(a, dc):
    """Gradient of c = a w with respect to w, summed over every row of the segment (and batch):
    dw[k, n] = sum_rows a[row, k] dc[row, n].  a [..., K], dc [..., N] -> dw [K, N].  This is one
    segment's contribution; the paper's gradient averaging over the sequence-parallel group (Section 4)
    adds the segments' contributions."""
    a, dc = _f64(a), _f64(dc)
    if a.shape[:-1] != dc.shape[:-1]:
        raise ValueError("a and dc must have the same rows")
    return np.matmul(a.reshape(-1, a.shape[-1]).T, dc.reshape(-1, dc.shape[-1]))
