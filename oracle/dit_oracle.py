"""ctypes binding of oracle/dit_oracle.c (test infrastructure, fp64, CPU only).

Arrays go in as numpy: uint16 (bf16 bit patterns), float32 or float64, dense
[B, L, H, D].  Results come back as float64.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dit_oracle.c")
_LIB = os.path.join(_HERE, "libdit_oracle.so")
_lib = None

_I32x3 = ctypes.c_int32 * 3


def build(force=False):
    """Compile the oracle with gcc (-O2, OpenMP, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.oracle_num_threads.restype = ctypes.c_int
        for name in ("oracle_self_attn", "oracle_cross_attn", "oracle_rope3d",
                     "oracle_token_positions"):
            getattr(_lib, name).restype = ctypes.c_int
    return _lib


def num_threads():
    return int(_load().oracle_num_threads())


def _dtype_code(a):
    if a.dtype == np.uint16:
        return 0
    if a.dtype == np.float32:
        return 1
    if a.dtype == np.float64:
        return 2
    raise TypeError("oracle inputs must be uint16 (bf16 bits), float32 or float64, got %s" % a.dtype)


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p) if a is not None else None


def token_positions(grid, origin=(0, 0, 0), n_tokens=None):
    n = int(np.prod(grid)) if n_tokens is None else int(n_tokens)
    out = np.empty((n, 3), dtype=np.int64)
    rc = _load().oracle_token_positions(_I32x3(*grid), _I32x3(*origin), ctypes.c_int64(n), _ptr(out))
    assert rc == 0
    return out


def rope3d(x, pos, split, base=10000.0):
    """Rotate x[L, D] (float64) at integer positions pos[L, 3]."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    pos = np.ascontiguousarray(pos, dtype=np.int64)
    L, D = x.shape
    assert pos.shape == (L, 3)
    y = np.empty_like(x)
    rc = _load().oracle_rope3d(_ptr(x), _ptr(y), ctypes.c_int64(L), ctypes.c_int32(D), _ptr(pos),
                               _I32x3(*split), ctypes.c_double(base))
    if rc != 0:
        raise ValueError("oracle_rope3d rejected its arguments (rc=%d)" % rc)
    return y


def self_attn(q, k, v, grid, split, origin=(0, 0, 0), base=10000.0, scale=0.0, rows=None,
              want_lse=False, probs_of=None):
    """Self-attention with 3-axis RoPE.  q, k, v: [B, L, H, D].

    rows: token indices to compute (default: all).  Returns out [B, n_rows, H, D] float64,
    plus lse [B, H, n_rows] if want_lse, plus probs [n_rows, L] of (b, h) = probs_of.
    """
    q, k, v = (np.ascontiguousarray(a) for a in (q, k, v))
    dt = _dtype_code(q)
    assert k.dtype == q.dtype and v.dtype == q.dtype and q.shape == k.shape == v.shape
    B, L, H, D = q.shape
    assert L == int(np.prod(grid)), "L must equal T*Hg*Wg"
    rows = np.arange(L, dtype=np.int64) if rows is None else np.ascontiguousarray(rows, dtype=np.int64)
    n_rows = rows.shape[0]
    out = np.empty((B, n_rows, H, D), dtype=np.float64)
    lse = np.empty((B, H, n_rows), dtype=np.float64) if want_lse else None
    probs = np.empty((n_rows, L), dtype=np.float64) if probs_of is not None else None
    pb, ph = probs_of if probs_of is not None else (0, 0)
    rc = _load().oracle_self_attn(
        _ptr(q), _ptr(k), _ptr(v), ctypes.c_int32(dt), ctypes.c_int32(B), ctypes.c_int32(H),
        ctypes.c_int32(D), _I32x3(*grid), _I32x3(*origin), _I32x3(*split), ctypes.c_double(base),
        ctypes.c_double(scale), _ptr(rows), ctypes.c_int64(n_rows), _ptr(out), _ptr(lse),
        _ptr(probs), ctypes.c_int32(pb), ctypes.c_int32(ph))
    if rc != 0:
        raise ValueError("oracle_self_attn rejected its arguments (rc=%d)" % rc)
    res = (out,)
    if want_lse:
        res += (lse,)
    if probs_of is not None:
        res += (probs,)
    return res[0] if len(res) == 1 else res


def as_f64(a):
    """uint16 bf16 bit patterns, float32 or float64 -> float64 values."""
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def qk_rmsnorm(x, gamma=None, eps=1e-6, mode="head"):
    """Root-mean-square normalisation of query or key rows before the rotation.

    x: [..., H, D].  mode "head": the mean square runs over the D channels of each head;
    mode "token": over all H*D channels of the token.  y = x * gamma / sqrt(mean(x^2) + eps),
    gamma: [H, D] (or None = 1).  Returns float64.
    """
    x = as_f64(x)
    if mode == "head":
        ms = np.mean(x * x, axis=-1, keepdims=True)
    elif mode == "token":
        ms = np.mean(x * x, axis=(-2, -1), keepdims=True)
    else:
        raise ValueError(mode)
    y = x / np.sqrt(ms + eps)
    if gamma is not None:
        y = y * np.asarray(gamma, dtype=np.float64).reshape(x.shape[-2:])
    return y


def self_attn_normed(q, k, v, grid, split, q_gamma=None, k_gamma=None, eps=1e-6, mode="head", **kw):
    """Self-attention whose q and k rows are RMS-normalised (qk_rmsnorm) before the rotation:
    the definition written out as normalise, then self_attn on the float64 results."""
    return self_attn(qk_rmsnorm(q, q_gamma, eps, mode), qk_rmsnorm(k, k_gamma, eps, mode), as_f64(v), grid, split,
                     **kw)


def self_attn_packed(q, k, v, grids, split, origin=(0, 0, 0), base=10000.0, scale=0.0, want_lse=False):
    """Self-attention of several requests packed along the token axis: q, k, v [sum L_i, H, D],
    request i on its own grid grids[i] = (T, Hg, Wg) with L_i = T*Hg*Wg tokens.  Requests do not
    see each other, so this is the definition written out: one self_attn call per request on its
    rows.  Returns out [sum L_i, H, D] float64 (and lse [H, sum L_i])."""
    q, k, v = (np.ascontiguousarray(a) for a in (q, k, v))
    N, H, D = q.shape
    assert sum(int(np.prod(g)) for g in grids) == N, "grids must add up to the packed token count"
    out = np.empty((N, H, D), dtype=np.float64)
    lse = np.empty((H, N), dtype=np.float64) if want_lse else None
    n0 = 0
    for g in grids:
        L = int(np.prod(g))
        sl = slice(n0, n0 + L)
        res = self_attn(q[None, sl], k[None, sl], v[None, sl], g, split, origin=origin, base=base, scale=scale,
                        want_lse=want_lse)
        if want_lse:
            out[sl], lse[:, sl] = res[0][0], res[1][0]
        else:
            out[sl] = res[0]
        n0 += L
    return (out, lse) if want_lse else out


def cross_attn(q, k, v, kv_valid=None, scale=0.0, rows=None, want_lse=False, probs_of=None):
    """Cross-attention, joint softmax over Lk keys with a key-padding mask.

    q: [B, Lq, H, D]; k, v: [B, Lk, H, D]; kv_valid: [B, Lk] uint8 (1 = attend) or None.
    """
    q, k, v = (np.ascontiguousarray(a) for a in (q, k, v))
    dt = _dtype_code(q)
    assert k.dtype == q.dtype and v.dtype == q.dtype and k.shape == v.shape
    B, Lq, H, D = q.shape
    Lk = k.shape[1]
    assert k.shape == (B, Lk, H, D)
    if kv_valid is not None:
        kv_valid = np.ascontiguousarray(kv_valid, dtype=np.uint8)
        assert kv_valid.shape == (B, Lk)
    rows = np.arange(Lq, dtype=np.int64) if rows is None else np.ascontiguousarray(rows, dtype=np.int64)
    n_rows = rows.shape[0]
    out = np.empty((B, n_rows, H, D), dtype=np.float64)
    lse = np.empty((B, H, n_rows), dtype=np.float64) if want_lse else None
    probs = np.empty((n_rows, Lk), dtype=np.float64) if probs_of is not None else None
    pb, ph = probs_of if probs_of is not None else (0, 0)
    rc = _load().oracle_cross_attn(
        _ptr(q), _ptr(k), _ptr(v), _ptr(kv_valid), ctypes.c_int32(dt), ctypes.c_int32(B),
        ctypes.c_int32(H), ctypes.c_int32(D), ctypes.c_int64(Lq), ctypes.c_int64(Lk),
        ctypes.c_double(scale), _ptr(rows), ctypes.c_int64(n_rows), _ptr(out), _ptr(lse),
        _ptr(probs), ctypes.c_int32(pb), ctypes.c_int32(ph))
    if rc != 0:
        raise ValueError("oracle_cross_attn rejected its arguments (rc=%d)" % rc)
    res = (out,)
    if want_lse:
        res += (lse,)
    if probs_of is not None:
        res += (probs,)
    return res[0] if len(res) == 1 else res


def cross_attn_decoupled(q, k, v, split, kv_valid=None, scale=0.0, rows=None):
    """Decoupled cross-attention: keys [0, split) and [split, Lk) are two separate conditioning
    sequences (text, image), each with its OWN softmax; the two attention outputs are added:

        out = softmax(scale q k_A^T) v_A + softmax(scale q k_B^T) v_B.

    A group with no valid key (or no key at all) contributes zero.  This is the definition written
    out: two independent calls of the joint-softmax routine on the two key ranges, summed.
    """
    k = np.ascontiguousarray(k)
    v = np.ascontiguousarray(v)
    Lk = k.shape[1]
    if not 0 <= split <= Lk:
        raise ValueError("split must lie in [0, Lk]")
    total = None
    for lo, hi in ((0, split), (split, Lk)):
        if hi == lo:
            continue
        val = None if kv_valid is None else np.ascontiguousarray(kv_valid[:, lo:hi])
        part = cross_attn(q, k[:, lo:hi], v[:, lo:hi], val, scale=scale, rows=rows)
        total = part if total is None else total + part
    return total


# ---- the optional 8-bit score operands (library flag DIT_FLAG_QK_FP8): a MODEL of the quantiser ----
# e4m3_round is the published format and is pinned against its code table.  self_attn_fp8_scores, by contrast, is
# NOT part of the oracle's definition of attention: it was written after the 8-bit kernel and models that kernel's
# choices (what is rounded, the power-of-two row factor, where scale*log2(e) is folded in).  The parity evidence
# for the 8-bit path is the comparison with the plain self_attn above, judged with the error statistics derived
# from the format in tests/fp8_error_model.py; this model only serves as a diagnostic and to validate those
# statistics on the CPU.

E4M3_MAX = 448.0


def e4m3_round(x):
    """Nearest value of the OCP 8-bit floating-point format E4M3 (1 sign, 4 exponent bits with bias
    7, 3 mantissa bits; normal numbers 2^-6 .. 448, subnormals in steps of 2^-9), ties to the even
    mantissa, magnitudes beyond 448 saturate to 448.  Input and result float64."""
    x = np.asarray(x, dtype=np.float64)
    a = np.abs(x)
    _, ex = np.frexp(np.maximum(a, 2.0 ** -6))  # a in [2^(ex-1), 2^ex); below 2^-6 the subnormal step applies
    step = np.ldexp(1.0, ex - 1 - 3)
    r = np.minimum(np.round(a / step) * step, E4M3_MAX)  # numpy rounds halves to even
    return np.copysign(r, x)


def e4m3_quantise_rows(x):
    """Each row (last axis) is multiplied by the power of two that brings its largest magnitude
    into [128, 256), rounded to E4M3, and divided back; an all-zero row stays zero.  Returns the
    float64 values the 8-bit operands stand for."""
    x = np.asarray(x, dtype=np.float64)
    amax = np.max(np.abs(x), axis=-1, keepdims=True)
    _, ex = np.frexp(amax)  # amax in [2^(ex-1), 2^ex)
    e = np.where(amax > 0, 8 - ex, 0)
    return np.ldexp(e4m3_round(np.ldexp(x, e)), -e)


def self_attn_fp8_scores(q, k, v, grid, split, origin=(0, 0, 0), base=10000.0, scale=0.0):
    """MODEL (see above), not a definition.  Self-attention whose SCORE operands are rounded to E4M3: q' = rope(q) * scale * log2(e) and
    k' = rope(k), each row quantised by e4m3_quantise_rows; scores = q' k'^T (in base-2 units),
    softmax and the value product in float64.  q, k, v: [B, L, H, D]; returns [B, L, H, D] float64.
    Sizes the plain numpy products below can hold (L up to a few thousand)."""
    q, k, v = as_f64(q), as_f64(k), as_f64(v)
    B, L, H, D = q.shape
    pos = token_positions(grid, origin)
    if scale <= 0:
        scale = 1.0 / np.sqrt(D)
    out = np.empty_like(q)
    for b in range(B):
        for h in range(H):
            qr = e4m3_quantise_rows(rope3d(q[b, :, h], pos, split, base) * (scale * np.log2(np.e)))
            kr = e4m3_quantise_rows(rope3d(k[b, :, h], pos, split, base))
            s = qr @ kr.T
            p = np.exp2(s - s.max(axis=1, keepdims=True))
            out[b, :, h] = (p @ v[b, :, h]) / p.sum(axis=1, keepdims=True)
    return out


def linear(x, w, bias=None):
    """Dense projection of token rows, y = x w^T + bias: the query/key/value and output projections
    either side of attention in a block of the Diffusion stage (Section 2.4, the AIGC workflow;
    the model is the cited video transformer, whose layers store a weight as [out, in]).

    x: [M, K], w: [N, K], bias: [N] or None; uint16 bf16 bit patterns, float32 or float64.
    Returns float64 [M, N]: every input converted exactly, one fp64 matrix product.
    """
    y = as_f64(x) @ as_f64(w).T
    if bias is not None:
        y = y + as_f64(bias)[None, :]
    return y
