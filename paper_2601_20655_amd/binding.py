"""ctypes binding of include/dit_attn.h: argument marshalling only.

Every function here has the name of the C entry point it calls.  torch is used for device
memory (tensors, workspace) and for the current HIP stream; all arithmetic happens in the
library's kernels.  If libdit_attn.so has not been built, loading fails with an error --
there is no fallback path.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdit_attn.so")

DIT_OK = 0
DIT_ERR_INVALID_ARG = -1
DIT_ERR_UNSUPPORTED = -2
DIT_ERR_ALIGNMENT = -3
DIT_ERR_WORKSPACE = -4
DIT_ERR_HIP = -5

DIT_BF16 = 0
DIT_F32 = 1

DIT_FLAG_QK_BF16 = 1 << 0
DIT_FLAG_QK_F16 = 1 << 1
DIT_FLAG_PV_BF16 = 1 << 2
DIT_FLAG_PV_F16 = 1 << 3
DIT_FLAG_KV_PREPACK = 1 << 4
DIT_FLAG_KV_FUSED = 1 << 5
DIT_FLAG_WIDE_QTILE = 1 << 6
DIT_FLAG_SIMPLE_SCHEDULE = 1 << 7
DIT_FLAG_BIG_WORKGROUP = 1 << 8
DIT_FLAG_SMALL_WORKGROUP = 1 << 9
DIT_FLAG_PIPELINED_SCHEDULE = 1 << 10
DIT_FLAG_KV_RESIDENT = 1 << 11
DIT_FLAG_QK_FP8 = 1 << 12
DIT_FLAG_MFMA_32X32 = 1 << 13

EXPORTS = (
    "dit_attn_workspace_bytes",
    "dit_attn_forward",
    "dit_cross_attn_workspace_bytes",
    "dit_cross_attn_forward",
    "dit_cross_attn_forward_static",
    "dit_cross_attn_forward_lengths",
    "dit_attn_varlen_workspace_bytes",
    "dit_attn_varlen_forward",
    "dit_linear_forward",
    "dit_qkv_proj_forward",
    "dit_mfma_probe",
    "dit_attn_set_timing_events",
    "dit_strerror",
    "dit_last_hip_error",
    "dit_attn_version",
)


class dit_strides(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int64), ("token", ctypes.c_int64), ("head", ctypes.c_int64)]


DIT_NORM_NONE = 0
DIT_NORM_HEAD = 1
DIT_NORM_TOKEN = 2


class dit_qk_norm(ctypes.Structure):
    _fields_ = [("mode", ctypes.c_int32), ("eps", ctypes.c_float),
                ("q_gamma", ctypes.c_void_p), ("k_gamma", ctypes.c_void_p)]


class dit_self_attn_params(ctypes.Structure):
    _fields_ = [
        ("B", ctypes.c_int32), ("H", ctypes.c_int32), ("D", ctypes.c_int32),
        ("T", ctypes.c_int32), ("Hg", ctypes.c_int32), ("Wg", ctypes.c_int32),
        ("t0", ctypes.c_int32), ("h0", ctypes.c_int32), ("w0", ctypes.c_int32),
        ("d_t", ctypes.c_int32), ("d_h", ctypes.c_int32), ("d_w", ctypes.c_int32),
        ("rope_base", ctypes.c_float), ("scale", ctypes.c_float),
        ("in_dtype", ctypes.c_int32), ("out_dtype", ctypes.c_int32),
        ("flags", ctypes.c_uint32),
        ("sq", dit_strides), ("sk", dit_strides), ("sv", dit_strides), ("so", dit_strides),
        ("norm", dit_qk_norm),
    ]


class dit_cross_attn_params(ctypes.Structure):
    _fields_ = [
        ("B", ctypes.c_int32), ("H", ctypes.c_int32), ("D", ctypes.c_int32),
        ("Lq", ctypes.c_int32), ("Lk", ctypes.c_int32),
        ("scale", ctypes.c_float),
        ("in_dtype", ctypes.c_int32), ("out_dtype", ctypes.c_int32),
        ("flags", ctypes.c_uint32), ("Lk_split", ctypes.c_int32),
        ("sq", dit_strides), ("sk", dit_strides), ("sv", dit_strides), ("so", dit_strides),
        ("norm", dit_qk_norm),
    ]


DIT_MAX_REQUESTS = 64


class dit_grid(ctypes.Structure):
    _fields_ = [("T", ctypes.c_int32), ("Hg", ctypes.c_int32), ("Wg", ctypes.c_int32)]


class dit_varlen_attn_params(ctypes.Structure):
    _fields_ = [
        ("n_requests", ctypes.c_int32), ("H", ctypes.c_int32), ("D", ctypes.c_int32),
        ("grids", ctypes.POINTER(dit_grid)),
        ("t0", ctypes.c_int32), ("h0", ctypes.c_int32), ("w0", ctypes.c_int32),
        ("d_t", ctypes.c_int32), ("d_h", ctypes.c_int32), ("d_w", ctypes.c_int32),
        ("rope_base", ctypes.c_float), ("scale", ctypes.c_float),
        ("in_dtype", ctypes.c_int32), ("out_dtype", ctypes.c_int32),
        ("flags", ctypes.c_uint32),
        ("sq", dit_strides), ("sk", dit_strides), ("sv", dit_strides), ("so", dit_strides),
        ("norm", dit_qk_norm),
    ]


class dit_linear_params(ctypes.Structure):
    _fields_ = [
        ("M", ctypes.c_int32), ("N", ctypes.c_int32), ("K", ctypes.c_int32),
        ("ldx", ctypes.c_int64), ("ldw", ctypes.c_int64), ("ldy", ctypes.c_int64),
        ("out_dtype", ctypes.c_int32), ("flags", ctypes.c_uint32),
    ]


class DitError(RuntimeError):
    def __init__(self, status, what):
        self.status = int(status)
        super().__init__("%s failed: %s (status %d)%s" % (
            what, dit_strerror(status), status,
            (" -- " + dit_last_hip_error()) if status == DIT_ERR_HIP else ""))


_lib = None


def lib():
    """The loaded shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                "libdit_attn.so is not built (run `python -m paper_2601_20655_amd.build`); "
                "there is no CPU fallback")
        L = ctypes.CDLL(LIB_PATH)
        vp = ctypes.c_void_p
        L.dit_attn_workspace_bytes.restype = ctypes.c_size_t
        L.dit_attn_workspace_bytes.argtypes = [ctypes.POINTER(dit_self_attn_params)]
        L.dit_cross_attn_workspace_bytes.restype = ctypes.c_size_t
        L.dit_cross_attn_workspace_bytes.argtypes = [ctypes.POINTER(dit_cross_attn_params)]
        L.dit_attn_forward.restype = ctypes.c_int
        L.dit_attn_forward.argtypes = [vp, vp, vp, vp, vp, ctypes.POINTER(dit_self_attn_params), vp,
                                       ctypes.c_size_t, vp]
        L.dit_cross_attn_forward.restype = ctypes.c_int
        L.dit_cross_attn_forward.argtypes = [vp, vp, vp, vp, vp, vp, ctypes.POINTER(dit_cross_attn_params),
                                             vp, ctypes.c_size_t, vp]
        L.dit_cross_attn_forward_lengths.restype = ctypes.c_int
        L.dit_cross_attn_forward_lengths.argtypes = [vp, vp, vp, vp, ctypes.c_int32, vp, vp,
                                                     ctypes.POINTER(dit_cross_attn_params), vp, ctypes.c_size_t, vp]
        L.dit_cross_attn_forward_static.restype = ctypes.c_int
        L.dit_cross_attn_forward_static.argtypes = [vp, vp, vp, vp, vp, vp, ctypes.POINTER(dit_cross_attn_params), vp]
        L.dit_attn_varlen_workspace_bytes.restype = ctypes.c_size_t
        L.dit_attn_varlen_workspace_bytes.argtypes = [ctypes.POINTER(dit_varlen_attn_params)]
        L.dit_attn_varlen_forward.restype = ctypes.c_int
        L.dit_attn_varlen_forward.argtypes = [vp, vp, vp, vp, vp, ctypes.POINTER(dit_varlen_attn_params), vp,
                                              ctypes.c_size_t, vp]
        L.dit_linear_forward.restype = ctypes.c_int
        L.dit_linear_forward.argtypes = [vp, vp, vp, vp, ctypes.POINTER(dit_linear_params), vp]
        L.dit_qkv_proj_forward.restype = ctypes.c_int
        L.dit_qkv_proj_forward.argtypes = [vp, vp, vp, vp, ctypes.POINTER(dit_linear_params),
                                           ctypes.POINTER(dit_self_attn_params), vp, ctypes.c_size_t, vp]
        L.dit_mfma_probe.restype = ctypes.c_int
        L.dit_mfma_probe.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int64, vp, ctypes.c_size_t,
                                     ctypes.POINTER(ctypes.c_double), vp]
        L.dit_attn_set_timing_events.restype = None
        L.dit_attn_set_timing_events.argtypes = [vp, vp]
        L.dit_strerror.restype = ctypes.c_char_p
        L.dit_strerror.argtypes = [ctypes.c_int]
        L.dit_last_hip_error.restype = ctypes.c_char_p
        L.dit_attn_version.restype = ctypes.c_int
        _lib = L
    return _lib


def dit_strerror(status):
    return lib().dit_strerror(int(status)).decode()


def dit_last_hip_error():
    return lib().dit_last_hip_error().decode()


def dit_attn_set_timing_events(before, after):
    """before/after: raw hipEvent_t handles (ints) or None to switch the hook off."""
    lib().dit_attn_set_timing_events(before, after)


def dit_attn_version():
    return int(lib().dit_attn_version())


def _dtype_code(t):
    import torch

    if t.dtype == torch.bfloat16:
        return DIT_BF16
    if t.dtype == torch.float32:
        return DIT_F32
    raise TypeError("tensors must be bfloat16 or float32, got %s" % t.dtype)


def _strides(t):
    """[B, L, H, D] tensor (any permutation underneath) -> dit_strides; channel stride must be 1."""
    if t.dim() != 4 or t.stride(3) != 1:
        raise ValueError("expected a [B, L, H, D] tensor with contiguous channels")
    return dit_strides(t.stride(0), t.stride(1), t.stride(2))


def _stream_ptr(stream):
    import torch

    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def qk_norm(norm, H, D):
    """norm: None, or (mode, eps, q_gamma, k_gamma) with mode "head" / "token" and the weights
    device float32 tensors of H*D elements (or None)."""
    if norm is None:
        return dit_qk_norm()
    import torch

    mode, eps, gq, gk = norm
    ptrs = []
    for g in (gq, gk):
        if g is not None and (not g.is_cuda or g.dtype != torch.float32 or g.numel() != H * D or not g.is_contiguous()):
            raise ValueError("normalisation weights must be dense float32 device tensors of H*D elements")
        ptrs.append(g.data_ptr() if g is not None else None)
    return dit_qk_norm({"head": DIT_NORM_HEAD, "token": DIT_NORM_TOKEN}[mode], eps, ptrs[0], ptrs[1])


def self_attn_params(q, k, v, out, grid, split, origin=(0, 0, 0), rope_base=10000.0, scale=0.0, flags=0,
                     norm=None):
    B, L, H, D = q.shape
    return dit_self_attn_params(
        B, H, D, grid[0], grid[1], grid[2], origin[0], origin[1], origin[2], split[0], split[1], split[2],
        rope_base, scale, _dtype_code(q), _dtype_code(out), flags,
        _strides(q), _strides(k), _strides(v), _strides(out), qk_norm(norm, H, D))


def cross_attn_params(q, k, v, out, scale=0.0, flags=0, split=0, norm=None):
    B, Lq, H, D = q.shape
    return dit_cross_attn_params(B, H, D, Lq, k.shape[1], scale, _dtype_code(q), _dtype_code(out), flags, split,
                                 _strides(q), _strides(k), _strides(v), _strides(out), qk_norm(norm, H, D))


def _strides3(t):
    """[N, H, D] tensor (packed requests) -> dit_strides with batch stride 0."""
    if t.dim() != 3 or t.stride(2) != 1:
        raise ValueError("expected a [tokens, H, D] tensor with contiguous channels")
    return dit_strides(0, t.stride(0), t.stride(1))


def varlen_attn_params(q, k, v, out, grids, split, origin=(0, 0, 0), rope_base=10000.0, scale=0.0, flags=0,
                       norm=None):
    """grids: sequence of (T, Hg, Wg).  The returned struct keeps the host grid array alive."""
    N, H, D = q.shape
    arr = (dit_grid * max(len(grids), 1))(*[dit_grid(*g) for g in grids])
    p = dit_varlen_attn_params(
        len(grids), H, D, ctypes.cast(arr, ctypes.POINTER(dit_grid)), origin[0], origin[1], origin[2],
        split[0], split[1], split[2], rope_base, scale, _dtype_code(q), _dtype_code(out), flags,
        _strides3(q), _strides3(k), _strides3(v), _strides3(out), qk_norm(norm, H, D))
    p._grids_keepalive = arr
    return p


def dit_attn_varlen_workspace_bytes(params):
    return int(lib().dit_attn_varlen_workspace_bytes(ctypes.byref(params)))


def dit_attn_workspace_bytes(params):
    return int(lib().dit_attn_workspace_bytes(ctypes.byref(params)))


def dit_cross_attn_workspace_bytes(params):
    return int(lib().dit_cross_attn_workspace_bytes(ctypes.byref(params)))


def _check_tensors(what, q, k, v, out, lse, kv_shape, lse_shape, resident=False):
    """The C side addresses memory from the shapes in the params struct alone, so every tensor handed over
    must really have the extent those shapes imply: raise instead of letting a kernel run past an allocation.
    Shapes and dtypes are checked first, devices last."""
    import torch

    qshape = tuple(q.shape)
    kv = () if resident else (("k", k), ("v", v))
    for name, t in kv:
        if t is None or tuple(t.shape) != tuple(kv_shape):
            raise ValueError("%s: %s has shape %s, expected %s" % (
                what, name, None if t is None else tuple(t.shape), tuple(kv_shape)))
        if t.dtype != q.dtype:
            raise ValueError("%s: q, k and v must share one dtype (q %s, %s %s)" % (what, q.dtype, name, t.dtype))
    if out is not None and tuple(out.shape) != qshape:
        raise ValueError("%s: out has shape %s, expected q's shape %s" % (what, tuple(out.shape), qshape))
    if lse is not None and (lse.dtype != torch.float32 or not lse.is_contiguous()
                            or tuple(lse.shape) != tuple(lse_shape)):
        raise ValueError("%s: lse must be a dense float32 tensor of shape %s" % (what, tuple(lse_shape)))
    for name, t in (("q", q),) + kv + (("out", out), ("lse", lse)):
        if t is not None and (not t.is_cuda or t.device != q.device):
            raise ValueError("%s needs device tensors on one device (%s is on %s)" % (what, name, t.device))


def _check_workspace(what, workspace, need, device):
    if not workspace.is_cuda or workspace.device != device or not workspace.is_contiguous():
        raise ValueError("%s: workspace must be a dense tensor on q's device" % what)
    if workspace.numel() * workspace.element_size() < need:
        raise ValueError("%s: workspace holds %d bytes, %d needed" % (
            what, workspace.numel() * workspace.element_size(), need))


def _workspace(nbytes, device):
    import torch

    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def dit_attn_forward(q, k, v, grid, split, out=None, lse=None, origin=(0, 0, 0), rope_base=10000.0,
                     scale=0.0, flags=0, out_dtype=None, workspace=None, stream=None, want_lse=False, norm=None):
    """Self-attention with 3-axis RoPE on device tensors q, k, v of shape [B, L, H, D].
    norm: None or (mode, eps, q_gamma, k_gamma), see qk_norm.

    Allocates `out` (and `lse`, `workspace`) with torch when not given; returns out, or
    (out, lse) when an lse buffer is requested.  Asynchronous on the stream.
    """
    import torch

    if q.dim() != 4:
        raise ValueError("dit_attn_forward: q must be [B, L, H, D]")
    B, L, H, D = q.shape
    if len(grid) != 3 or int(grid[0]) * int(grid[1]) * int(grid[2]) != L:
        raise ValueError("dit_attn_forward: grid %s does not have q's %d tokens" % (tuple(grid), L))
    resident = bool(flags & DIT_FLAG_KV_RESIDENT)
    _check_tensors("dit_attn_forward", q, k, v, out, lse, (B, L, H, D), (B, H, L), resident)
    if out is None:
        out = torch.empty((B, L, H, D), dtype=out_dtype or q.dtype, device=q.device)
    if lse is None and want_lse:
        lse = torch.empty((B, H, L), dtype=torch.float32, device=q.device)
    if resident and (k is None or v is None):
        k = v = q  # strides only; the key-side passes are skipped and the pointers are not read
    p = self_attn_params(q, k, v, out, grid, split, origin, rope_base, scale, flags, norm)
    need = dit_attn_workspace_bytes(p)
    if workspace is None:
        workspace = _workspace(need, q.device)
    _check_workspace("dit_attn_forward", workspace, need, q.device)
    st = lib().dit_attn_forward(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(),
                                lse.data_ptr() if lse is not None else None, ctypes.byref(p),
                                workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                _stream_ptr(stream))
    if st != DIT_OK:
        raise DitError(st, "dit_attn_forward")
    return (out, lse) if lse is not None else out


def _check_kv_valid(kv_valid, q, B, Lk, device_too=False):
    """Shape and dtype of the key mask; with device_too (after the other tensors' shapes are known good) its device."""
    import torch

    if kv_valid is None:
        return
    if kv_valid.dtype != torch.uint8 or not kv_valid.is_contiguous() or tuple(kv_valid.shape) != (B, Lk):
        raise ValueError("kv_valid must be a dense uint8 [B, Lk] tensor")
    if device_too and (not kv_valid.is_cuda or kv_valid.device != q.device):
        raise ValueError("kv_valid must be on q's device")


def dit_cross_attn_forward(q, k, v, kv_valid=None, out=None, lse=None, scale=0.0, flags=0, out_dtype=None,
                           workspace=None, stream=None, want_lse=False, split=0, norm=None):
    """Cross-attention: q [B, Lq, H, D]; k, v [B, Lk, H, D]; kv_valid uint8 [B, Lk] or None.
    split > 0 selects the decoupled form (separate softmax over keys [0, split) and [split, Lk))."""
    import torch

    if q.dim() != 4 or k.dim() != 4:
        raise ValueError("dit_cross_attn_forward: q must be [B, Lq, H, D] and k, v [B, Lk, H, D]")
    B, Lq, H, D = q.shape
    Lk = k.shape[1]
    _check_kv_valid(kv_valid, q, B, Lk)
    _check_tensors("dit_cross_attn_forward", q, k, v, out, lse, (B, Lk, H, D), (B, H, Lq))
    if out is None:
        out = torch.empty((B, Lq, H, D), dtype=out_dtype or q.dtype, device=q.device)
    if lse is None and want_lse:
        lse = torch.empty((B, H, Lq), dtype=torch.float32, device=q.device)
    _check_kv_valid(kv_valid, q, B, Lk, device_too=True)
    p = cross_attn_params(q, k, v, out, scale, flags, split, norm)
    need = dit_cross_attn_workspace_bytes(p)
    if workspace is None:
        workspace = _workspace(need, q.device)
    _check_workspace("dit_cross_attn_forward", workspace, need, q.device)
    st = lib().dit_cross_attn_forward(q.data_ptr(), k.data_ptr(), v.data_ptr(),
                                      kv_valid.data_ptr() if kv_valid is not None else None,
                                      out.data_ptr(), lse.data_ptr() if lse is not None else None,
                                      ctypes.byref(p), workspace.data_ptr(),
                                      workspace.numel() * workspace.element_size(), _stream_ptr(stream))
    if st != DIT_OK:
        raise DitError(st, "dit_cross_attn_forward")
    return (out, lse) if lse is not None else out


def dit_cross_attn_forward_lengths(q, k, v, kv_len, second_start, out=None, lse=None, scale=0.0, flags=0,
                                   out_dtype=None, workspace=None, stream=None, want_lse=False, split=0, norm=None):
    """Cross-attention with per-request key counts: kv_len int32 [B, 2] on the device; the keys that attend are
    the first kv_len[b, 0] of [0, second_start) and the first kv_len[b, 1] of [second_start, Lk)."""
    import torch

    if q.dim() != 4 or k.dim() != 4:
        raise ValueError("dit_cross_attn_forward_lengths: q must be [B, Lq, H, D] and k, v [B, Lk, H, D]")
    B, Lq, H, D = q.shape
    Lk = k.shape[1]
    resident = bool(flags & DIT_FLAG_KV_RESIDENT)
    if kv_len is None:
        if not resident:
            raise ValueError("kv_len is required (it may only be None with DIT_FLAG_KV_RESIDENT)")
    else:
        if kv_len.dtype != torch.int32 or tuple(kv_len.shape) != (B, 2) or not kv_len.is_contiguous():
            raise ValueError("kv_len must be a contiguous int32 tensor of shape [B, 2]")
    _check_tensors("dit_cross_attn_forward_lengths", q, k, v, out, lse, (B, Lk, H, D), (B, H, Lq), resident)
    if kv_len is not None and kv_len.device != q.device:
        raise ValueError("kv_len must be on the device of q")
    if out is None:
        out = torch.empty((B, Lq, H, D), dtype=out_dtype or q.dtype, device=q.device)
    if lse is None and want_lse:
        lse = torch.empty((B, H, Lq), dtype=torch.float32, device=q.device)
    p = cross_attn_params(q, k, v, out, scale, flags, split, norm)
    need = dit_cross_attn_workspace_bytes(p)
    if workspace is None:
        workspace = _workspace(need, q.device)
    _check_workspace("dit_cross_attn_forward_lengths", workspace, need, q.device)
    st = lib().dit_cross_attn_forward_lengths(q.data_ptr(), k.data_ptr() if k is not None else None,
                                              v.data_ptr() if v is not None else None,
                                              kv_len.data_ptr() if kv_len is not None else None, int(second_start),
                                              out.data_ptr(), lse.data_ptr() if lse is not None else None,
                                              ctypes.byref(p), workspace.data_ptr(),
                                              workspace.numel() * workspace.element_size(), _stream_ptr(stream))
    if st != DIT_OK:
        raise DitError(st, "dit_cross_attn_forward_lengths")
    return (out, lse) if lse is not None else out


DIT_STATIC_WORKSPACE_BYTES = 96 << 20


def dit_cross_attn_forward_static(q, k, v, kv_valid=None, out=None, lse=None, scale=0.0, flags=0, split=0,
                                  stream=None, norm=None):
    """dit_cross_attn_forward on the library's own static device workspace.  `out` (and `lse`) must be
    given: this wrapper allocates nothing either."""
    import torch

    if out is None:
        raise ValueError("dit_cross_attn_forward_static needs a caller-provided out")
    if q.dim() != 4 or k.dim() != 4:
        raise ValueError("dit_cross_attn_forward_static: q must be [B, Lq, H, D] and k, v [B, Lk, H, D]")
    B, Lq, H, D = q.shape
    Lk = k.shape[1]
    _check_kv_valid(kv_valid, q, B, Lk)
    _check_tensors("dit_cross_attn_forward_static", q, k, v, out, lse, (B, Lk, H, D), (B, H, Lq))
    _check_kv_valid(kv_valid, q, B, Lk, device_too=True)
    p = cross_attn_params(q, k, v, out, scale, flags, split, norm)
    st = lib().dit_cross_attn_forward_static(q.data_ptr(), k.data_ptr(), v.data_ptr(),
                                             kv_valid.data_ptr() if kv_valid is not None else None,
                                             out.data_ptr(), lse.data_ptr() if lse is not None else None,
                                             ctypes.byref(p), _stream_ptr(stream))
    if st != DIT_OK:
        raise DitError(st, "dit_cross_attn_forward_static")
    return (out, lse) if lse is not None else out


def dit_attn_varlen_forward(q, k, v, grids, split, out=None, lse=None, origin=(0, 0, 0), rope_base=10000.0,
                            scale=0.0, flags=0, out_dtype=None, workspace=None, stream=None, want_lse=False,
                            norm=None):
    """Self-attention of several requests packed along the token axis: q, k, v [sum L_i, H, D],
    grids = [(T, Hg, Wg), ...] with L_i = T*Hg*Wg.  Returns out (and lse [H, sum L_i] if asked)."""
    import torch

    if q.dim() != 3:
        raise ValueError("dit_attn_varlen_forward: q must be [tokens, H, D]")
    N, H, D = q.shape
    if sum(g[0] * g[1] * g[2] for g in grids) != N:
        raise ValueError("the grids do not add up to the token count of q")
    _check_tensors("dit_attn_varlen_forward", q, k, v, out, lse, (N, H, D), (H, N),
                   bool(flags & DIT_FLAG_KV_RESIDENT))
    if out is None:
        out = torch.empty((N, H, D), dtype=out_dtype or q.dtype, device=q.device)
    if lse is None and want_lse:
        lse = torch.empty((H, N), dtype=torch.float32, device=q.device)
    p = varlen_attn_params(q, k, v, out, grids, split, origin, rope_base, scale, flags, norm)
    need = dit_attn_varlen_workspace_bytes(p)
    if workspace is None:
        workspace = _workspace(need, q.device)
    _check_workspace("dit_attn_varlen_forward", workspace, need, q.device)
    st = lib().dit_attn_varlen_forward(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(),
                                       lse.data_ptr() if lse is not None else None, ctypes.byref(p),
                                       workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                       _stream_ptr(stream))
    if st != DIT_OK:
        raise DitError(st, "dit_attn_varlen_forward")
    return (out, lse) if lse is not None else out


def linear_params(x, w, y, flags=0):
    if x.dim() != 2 or w.dim() != 2 or y.dim() != 2 or x.stride(1) != 1 or w.stride(1) != 1 or y.stride(1) != 1:
        raise ValueError("expected 2-D tensors with contiguous rows")
    if x.shape[1] != w.shape[1] or tuple(y.shape) != (x.shape[0], w.shape[0]):
        raise ValueError("shapes do not fit y[M, N] = x[M, K] w[N, K]^T")
    return dit_linear_params(x.shape[0], w.shape[0], x.shape[1], x.stride(0), w.stride(0), y.stride(0),
                             _dtype_code(y), flags)


def dit_linear_forward(x, w, bias=None, out=None, out_dtype=None, stream=None):
    """y = x w^T + bias: x [M, K] bf16, w [N, K] bf16, bias [N] bf16 or None; y [M, N] bf16 or fp32."""
    import torch

    if not x.is_cuda:
        raise ValueError("dit_linear_forward needs device tensors")
    if x.dtype != torch.bfloat16 or w.dtype != torch.bfloat16 or (bias is not None and bias.dtype != torch.bfloat16):
        raise TypeError("x, w and bias must be bfloat16")
    if bias is not None and (bias.dim() != 1 or bias.shape[0] != w.shape[0] or bias.stride(0) != 1):
        raise ValueError("bias must be a dense [N] tensor")
    if out is None:
        out = torch.empty((x.shape[0], w.shape[0]), dtype=out_dtype or x.dtype, device=x.device)
    p = linear_params(x, w, out)
    st = lib().dit_linear_forward(x.data_ptr(), w.data_ptr(), bias.data_ptr() if bias is not None else None,
                                  out.data_ptr(), ctypes.byref(p), _stream_ptr(stream))
    if st != DIT_OK:
        raise DitError(st, "dit_linear_forward")
    return out


def dit_qkv_proj_forward(x, w, bias, grid, split, H, q_out=None, origin=(0, 0, 0), rope_base=10000.0, scale=0.0,
                         flags=0, workspace=None, stream=None, norm=None):
    """Fused q/k/v projection in front of dit_attn_forward: x [L, K] bf16, w [3*H*128, K] bf16 (rows [q; k; v]),
    bias [3*H*128] bf16 or None, L = T*Hg*Wg.  Returns (q_out [1, L, H, 128] bf16, workspace): the workspace then
    holds the rotation table and the K'/V^T tile images (k and v rounded to bf16 first, as dit_linear_forward's rows), and
        dit_attn_forward(q_out, k=None, v=None, grid, split, flags=flags | DIT_FLAG_KV_RESIDENT, workspace=workspace)
    completes the attention (k and v are not read).  norm: None or (mode, eps, q_gamma, k_gamma): the k rows are
    normalised here; pass the same norm to dit_attn_forward, which normalises the q rows as it reads them."""
    import torch

    D = 128
    if x.dim() != 2 or w.dim() != 2 or x.stride(1) != 1 or w.stride(1) != 1:
        raise ValueError("x and w must be 2-D with contiguous rows")
    if not x.is_cuda or w.device != x.device:
        raise ValueError("dit_qkv_proj_forward needs device tensors on one device")
    if x.dtype != torch.bfloat16 or w.dtype != torch.bfloat16 or (bias is not None and bias.dtype != torch.bfloat16):
        raise TypeError("x, w and bias must be bfloat16")
    L = grid[0] * grid[1] * grid[2]
    if x.shape[0] != L or w.shape[0] != 3 * H * D or w.shape[1] != x.shape[1]:
        raise ValueError("shapes do not fit: x [T*Hg*Wg, K], w [3*H*128, K]")
    if bias is not None and (bias.dim() != 1 or bias.shape[0] != 3 * H * D or bias.stride(0) != 1 or
                             bias.device != x.device):
        raise ValueError("bias must be a dense [3*H*128] tensor on the device of x")
    if q_out is None:
        q_out = torch.empty((1, L, H, D), dtype=torch.bfloat16, device=x.device)
    if tuple(q_out.shape) != (1, L, H, D) or q_out.dtype != torch.bfloat16 or q_out.device != x.device:
        raise ValueError("q_out must be a bfloat16 [1, L, H, 128] tensor on the device of x")
    ap = self_attn_params(q_out, q_out, q_out, q_out, grid, split, origin, rope_base, scale, flags, norm)
    lp = dit_linear_params(L, 3 * H * D, x.shape[1], x.stride(0), w.stride(0), 3 * H * D, DIT_BF16, 0)
    need = dit_attn_workspace_bytes(ap)
    if workspace is None:
        workspace = _workspace(need, x.device)
    _check_workspace("dit_qkv_proj_forward", workspace, need, x.device)
    st = lib().dit_qkv_proj_forward(x.data_ptr(), w.data_ptr(), bias.data_ptr() if bias is not None else None,
                                    q_out.data_ptr(), ctypes.byref(lp), ctypes.byref(ap), workspace.data_ptr(),
                                    workspace.numel() * workspace.element_size(), _stream_ptr(stream))
    if st != DIT_OK:
        raise DitError(st, "dit_qkv_proj_forward")
    return q_out, workspace


DIT_PROBE_BF16 = 0
DIT_PROBE_F16 = 1


def dit_mfma_probe(operand_dtype, bits_a, bits_b, mfma_per_wavefront, sink, stream=None):
    """Enqueue the MFMA-only probe kernel; bits_a / bits_b: 0 = constant operands, n = random operands of n
    significant bits; sink: device float32 tensor (2 * CUs * 256 elements or more).
    Returns the flops the kernel performs; the caller times it."""
    flops = ctypes.c_double(0.0)
    st = lib().dit_mfma_probe(operand_dtype, int(bits_a), int(bits_b), int(mfma_per_wavefront), sink.data_ptr(),
                              sink.numel() * sink.element_size(), ctypes.byref(flops), _stream_ptr(stream))
    if st != DIT_OK:
        raise DitError(st, "dit_mfma_probe")
    return flops.value
