"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
public header declares, sizes its workspace as documented and rejects bad arguments before any
launch (so these calls never touch the HIP runtime)."""
import ctypes
import os
import re

import pytest

from paper_2601_20655_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "dit_attn.h")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dit_[a-z_]+)\s*\(", text)))


def test_header_symbols_are_exported():
    names = declared_functions()
    assert set(names) == set(B.EXPORTS)
    lib = B.lib()
    for n in names:
        assert hasattr(lib, n), n


def test_version_and_strerror():
    ver = B.dit_attn_version()  # major*10000 + minor*100 + patch, as the header documents
    major, minor, patch = ver // 10000, ver // 100 % 100, ver % 100
    assert major >= 1 and 0 <= minor < 100 and 0 <= patch < 100 and ver >= 10500
    assert B.dit_strerror(B.DIT_OK) == "ok"
    for code in (-1, -2, -3, -4, -5):
        assert B.dit_strerror(code) not in ("", "ok", "unknown status")
    assert B.dit_strerror(-99) == "unknown status"
    assert B.dit_last_hip_error() == ""


def self_params(B_=1, H=2, D=128, grid=(2, 3, 4), split=(44, 42, 42), flags=0, in_dtype=B.DIT_BF16,
                out_dtype=B.DIT_BF16, base=10000.0):
    L = grid[0] * grid[1] * grid[2]
    s = B.dit_strides(L * H * D, H * D, D)
    return B.dit_self_attn_params(B_, H, D, grid[0], grid[1], grid[2], 0, 0, 0, split[0], split[1], split[2],
                                  base, 0.0, in_dtype, out_dtype, flags, s, s, s, s)


def cross_params(B_=2, H=2, D=128, Lq=100, Lk=769, flags=0, split=0):
    sq = B.dit_strides(Lq * H * D, H * D, D)
    sk = B.dit_strides(Lk * H * D, H * D, D)
    return B.dit_cross_attn_params(B_, H, D, Lq, Lk, 0.0, B.DIT_BF16, B.DIT_BF16, flags, split, sq, sk, sk, sq)


def up(x, a=256):
    return (x + a - 1) // a * a


def test_workspace_size_formula():
    # tile image: 64 K' rows of (2D+16) bytes and D V^T rows of 144 bytes, each part padded to 18 / 10 KiB
    for D, split in ((128, (44, 42, 42)), (64, (22, 20, 22))):
        tile = 2 * (18 if D == 128 else 10) * 1024
        assert 64 * (2 * D + 16) <= tile // 2 and D * 144 <= tile // 2
        for grid in ((2, 3, 4), (21, 30, 52), (1, 1, 65)):
            L = grid[0] * grid[1] * grid[2]
            p = self_params(B_=2, H=3, D=D, grid=grid, split=split)
            tab = grid[0] * split[0] // 2 + grid[1] * split[1] // 2 + grid[2] * split[2] // 2
            want = up(tab * 8) + up(2 * 3 * ((L + 63) // 64) * tile)
            assert B.dit_attn_workspace_bytes(p) == want
    p = self_params(flags=B.DIT_FLAG_KV_FUSED | B.DIT_FLAG_PV_BF16)
    assert B.dit_attn_workspace_bytes(p) == up((2 * 22 + 3 * 21 + 4 * 21) * 8)
    c = cross_params()
    assert B.dit_cross_attn_workspace_bytes(c) == (up(2 * 13 * 8) + up(2 * 13 * 4) + 2 * up(2 * 4) + up(2 * 13 * 64 * 4)
                                                   + up(2 * 2 * 13 * 36 * 1024))


FAKE = 0x1000  # a 16-byte aligned non-NULL address that is never dereferenced: validation fails first


def call_self(p, q=FAKE, k=FAKE, v=FAKE, out=FAKE, ws=0x10000, ws_bytes=1 << 40):
    return B.lib().dit_attn_forward(q, k, v, out, None, ctypes.byref(p), ws, ws_bytes, None)


def call_self_no_launch(p):
    """For parameter sets that must be rejected: were they accepted, the call would stop at the workspace
    check (no workspace is passed) instead of launching anything on fake pointers."""
    return B.lib().dit_attn_forward(FAKE, FAKE, FAKE, FAKE, None, ctypes.byref(p), None, 0, None)


def call_cross(p, q=FAKE, k=FAKE, v=FAKE, out=FAKE, ws=0x10000, ws_bytes=1 << 40):
    return B.lib().dit_cross_attn_forward(q, k, v, None, out, None, ctypes.byref(p), ws, ws_bytes, None)


def test_self_attn_rejects_bad_arguments():
    assert B.lib().dit_attn_forward(FAKE, FAKE, FAKE, FAKE, None, None, 0x10000, 1 << 30, None) == B.DIT_ERR_INVALID_ARG
    assert call_self(self_params(split=(44, 42, 40))) == B.DIT_ERR_INVALID_ARG      # sum != D
    assert call_self(self_params(split=(43, 43, 42))) == B.DIT_ERR_INVALID_ARG      # odd sections
    assert call_self(self_params(split=(-2, 88, 42))) == B.DIT_ERR_INVALID_ARG
    assert call_self(self_params(grid=(0, 3, 4))) == B.DIT_ERR_INVALID_ARG
    assert call_self(self_params(base=0.0)) == B.DIT_ERR_INVALID_ARG
    assert call_self(self_params(in_dtype=7)) == B.DIT_ERR_INVALID_ARG
    assert call_self(self_params(D=96, split=(32, 32, 32))) == B.DIT_ERR_UNSUPPORTED
    assert call_self(self_params(flags=B.DIT_FLAG_QK_BF16 | B.DIT_FLAG_QK_F16)) == B.DIT_ERR_INVALID_ARG
    assert call_self(self_params(flags=B.DIT_FLAG_KV_PREPACK | B.DIT_FLAG_KV_FUSED)) == B.DIT_ERR_INVALID_ARG
    assert call_self(self_params(flags=1 << 20)) == B.DIT_ERR_INVALID_ARG
    assert call_self(self_params(flags=B.DIT_FLAG_KV_RESIDENT | B.DIT_FLAG_KV_FUSED | B.DIT_FLAG_PV_BF16)) == B.DIT_ERR_INVALID_ARG
    # 8-bit score operands: not together with a 16-bit choice, and only in the pipelined 32-row kernel
    assert call_self(self_params(flags=B.DIT_FLAG_QK_FP8 | B.DIT_FLAG_QK_F16)) == B.DIT_ERR_INVALID_ARG
    assert call_self(self_params(flags=B.DIT_FLAG_QK_FP8 | B.DIT_FLAG_QK_BF16)) == B.DIT_ERR_INVALID_ARG
    for other in (B.DIT_FLAG_SIMPLE_SCHEDULE, B.DIT_FLAG_WIDE_QTILE, B.DIT_FLAG_KV_FUSED | B.DIT_FLAG_PV_BF16):
        assert call_self(self_params(flags=B.DIT_FLAG_QK_FP8 | other)) == B.DIT_ERR_UNSUPPORTED
    assert call_self(self_params(flags=B.DIT_FLAG_WIDE_QTILE | B.DIT_FLAG_BIG_WORKGROUP)) == B.DIT_ERR_UNSUPPORTED
    assert call_self(self_params(flags=B.DIT_FLAG_SMALL_WORKGROUP | B.DIT_FLAG_BIG_WORKGROUP)) == B.DIT_ERR_INVALID_ARG
    # fused staging needs bf16 inputs, bf16 PV operands, head_dim 128
    assert call_self(self_params(flags=B.DIT_FLAG_KV_FUSED)) == B.DIT_ERR_UNSUPPORTED
    assert call_self(self_params(flags=B.DIT_FLAG_KV_FUSED | B.DIT_FLAG_PV_BF16, in_dtype=B.DIT_F32)) == B.DIT_ERR_UNSUPPORTED
    assert call_self(self_params(), q=0) == B.DIT_ERR_INVALID_ARG
    assert call_self(self_params(), out=0) == B.DIT_ERR_INVALID_ARG
    assert call_self(self_params(), k=FAKE + 2) == B.DIT_ERR_ALIGNMENT
    p = self_params()
    p.sv.token = 2 * 128 + 4                                                           # rows not 16-byte aligned
    assert call_self(p) == B.DIT_ERR_ALIGNMENT
    p = self_params()
    p.sq.token = 0
    assert call_self(p) == B.DIT_ERR_INVALID_ARG
    assert call_self(self_params(), ws=0) == B.DIT_ERR_WORKSPACE
    assert call_self(self_params(), ws=0x10010) == B.DIT_ERR_WORKSPACE                 # not 256-byte aligned
    need = B.dit_attn_workspace_bytes(self_params())
    assert call_self(self_params(), ws_bytes=need - 1) == B.DIT_ERR_WORKSPACE
    assert B.dit_attn_workspace_bytes(self_params(split=(44, 42, 40))) == 0


def test_cross_attn_rejects_bad_arguments():
    # the pipelined form keeps its tile list in the 64 lanes of a wavefront
    assert call_cross(cross_params(Lk=4097, flags=B.DIT_FLAG_PIPELINED_SCHEDULE)) == B.DIT_ERR_UNSUPPORTED
    assert B.dit_cross_attn_workspace_bytes(cross_params(Lk=4096, flags=B.DIT_FLAG_PIPELINED_SCHEDULE)) > 0
    assert B.dit_cross_attn_workspace_bytes(cross_params(Lk=4097)) > 0
    assert call_cross(cross_params(Lk=0)) == B.DIT_ERR_INVALID_ARG
    assert call_cross(cross_params(D=32)) == B.DIT_ERR_UNSUPPORTED
    assert call_cross(cross_params(flags=B.DIT_FLAG_KV_FUSED | B.DIT_FLAG_PV_BF16)) == B.DIT_ERR_UNSUPPORTED
    assert call_cross(cross_params(flags=B.DIT_FLAG_QK_FP8)) == B.DIT_ERR_UNSUPPORTED
    assert call_cross(cross_params(), v=0) == B.DIT_ERR_INVALID_ARG
    assert call_cross(cross_params(split=770)) == B.DIT_ERR_INVALID_ARG
    assert call_cross(cross_params(split=-1)) == B.DIT_ERR_INVALID_ARG
    assert call_cross(cross_params(split=512, flags=B.DIT_FLAG_PIPELINED_SCHEDULE)) == B.DIT_ERR_UNSUPPORTED
    assert call_cross(cross_params(split=512, flags=B.DIT_FLAG_WIDE_QTILE)) == B.DIT_ERR_UNSUPPORTED
    # a split that is not a tile multiple needs one more tile: 500 -> 8 + 5 tiles of 64 keys
    assert B.dit_cross_attn_workspace_bytes(cross_params(split=500)) == \
        up(2 * 13 * 8) + up(2 * 13 * 4) + 2 * up(2 * 4) + up(2 * 13 * 64 * 4) + up(2 * 2 * 13 * 36 * 1024)
    assert B.dit_cross_attn_workspace_bytes(cross_params(split=10)) == \
        up(2 * 13 * 8) + up(2 * 13 * 4) + 2 * up(2 * 4) + up(2 * 13 * 64 * 4) + up(2 * 2 * 13 * 36 * 1024)
    assert B.dit_cross_attn_workspace_bytes(cross_params(split=65)) == \
        up(2 * 13 * 8) + up(2 * 13 * 4) + 2 * up(2 * 4) + up(2 * 13 * 64 * 4) + up(2 * 2 * 13 * 36 * 1024)
    assert call_cross(cross_params(), q=FAKE + 8) == B.DIT_ERR_ALIGNMENT
    need = B.dit_cross_attn_workspace_bytes(cross_params())
    assert call_cross(cross_params(), ws_bytes=need - 1) == B.DIT_ERR_WORKSPACE
    assert B.dit_last_hip_error() == ""


def test_cross_attn_key_counts_rejections():
    """dit_cross_attn_forward_lengths: everything is checked before any launch (no workspace is passed, so a
    parameter set that got through the checks stops at DIT_ERR_WORKSPACE instead of touching the fake pointers)."""
    f = B.lib().dit_cross_attn_forward_lengths

    def call(p, kv_len=FAKE, second_start=512, q=FAKE):
        return f(q, FAKE, FAKE, kv_len, second_start, FAKE, None, ctypes.byref(p), None, 0, None)

    assert call(cross_params()) == B.DIT_ERR_WORKSPACE                      # accepted
    assert call(cross_params(), second_start=0) == B.DIT_ERR_WORKSPACE
    assert call(cross_params(), second_start=769) == B.DIT_ERR_WORKSPACE
    assert call(cross_params(), second_start=-1) == B.DIT_ERR_INVALID_ARG
    assert call(cross_params(), second_start=770) == B.DIT_ERR_INVALID_ARG
    assert call(cross_params(), kv_len=None) == B.DIT_ERR_INVALID_ARG
    assert call(cross_params(flags=B.DIT_FLAG_KV_RESIDENT), kv_len=None) == B.DIT_ERR_WORKSPACE
    assert call(cross_params(), kv_len=FAKE + 2) == B.DIT_ERR_ALIGNMENT
    # one softmax per sequence: the second range starts where the split is
    assert call(cross_params(split=512), second_start=512) == B.DIT_ERR_WORKSPACE
    assert call(cross_params(split=512), second_start=500) == B.DIT_ERR_INVALID_ARG
    assert call(cross_params(D=32)) == B.DIT_ERR_UNSUPPORTED
    assert call(cross_params(), q=0) == B.DIT_ERR_INVALID_ARG


def test_fused_qkv_projection_rejections():
    """dit_qkv_proj_forward checks everything before any launch; an accepted parameter set stops at
    DIT_ERR_WORKSPACE here because no workspace is passed."""
    f = B.lib().dit_qkv_proj_forward

    def call(ap, M=24, N=768, K=64, ldx=None, ldw=None, x=FAKE, w=FAKE, bias=FAKE, q=FAKE, out_dtype=B.DIT_BF16,
             lflags=0):
        lp = B.dit_linear_params(M, N, K, K if ldx is None else ldx, K if ldw is None else ldw, N, out_dtype, lflags)
        return f(x, w, bias, q, ctypes.byref(lp), ctypes.byref(ap), None, 0, None)

    assert call(self_params()) == B.DIT_ERR_WORKSPACE                                  # accepted
    assert call(self_params(), bias=None) == B.DIT_ERR_WORKSPACE
    assert call(self_params(flags=B.DIT_FLAG_QK_BF16 | B.DIT_FLAG_PV_BF16)) == B.DIT_ERR_WORKSPACE
    assert call(self_params(), x=None) == B.DIT_ERR_INVALID_ARG
    assert call(self_params(), q=None) == B.DIT_ERR_INVALID_ARG
    assert call(self_params(), M=25) == B.DIT_ERR_INVALID_ARG                          # rows are not the grid's tokens
    assert call(self_params(), N=512) == B.DIT_ERR_INVALID_ARG                         # not 3 H D features
    assert call(self_params(), ldx=32) == B.DIT_ERR_INVALID_ARG
    assert call(self_params(), out_dtype=B.DIT_F32) == B.DIT_ERR_INVALID_ARG
    assert call(self_params(), lflags=1) == B.DIT_ERR_INVALID_ARG
    assert call(self_params(), K=72, ldx=72, ldw=72) == B.DIT_ERR_UNSUPPORTED          # K is not a multiple of 64
    assert call(self_params(), x=FAKE + 2) == B.DIT_ERR_ALIGNMENT
    assert call(self_params(), ldw=68) == B.DIT_ERR_ALIGNMENT
    assert call(self_params(), bias=FAKE + 2) == B.DIT_ERR_ALIGNMENT
    # what the fused form does not cover: several sequences, an odd number of heads, head_dim 64, fp32 rows,
    # the other attention kernels, tiles that are already resident
    assert call(self_params(B_=2)) == B.DIT_ERR_UNSUPPORTED
    assert call(self_params(H=3), N=1152) == B.DIT_ERR_UNSUPPORTED
    assert call(self_params(D=64, split=(22, 20, 22)), N=384) == B.DIT_ERR_UNSUPPORTED
    assert call(self_params(in_dtype=B.DIT_F32)) == B.DIT_ERR_UNSUPPORTED
    for fl in (B.DIT_FLAG_KV_RESIDENT, B.DIT_FLAG_MFMA_32X32, B.DIT_FLAG_SIMPLE_SCHEDULE, B.DIT_FLAG_KV_FUSED,
               B.DIT_FLAG_QK_FP8, B.DIT_FLAG_WIDE_QTILE):
        assert call(self_params(flags=fl)) == B.DIT_ERR_UNSUPPORTED, fl
    p = self_params()
    p.norm = B.dit_qk_norm(B.DIT_NORM_HEAD, 1e-6, None, None)
    assert call(p) == B.DIT_ERR_WORKSPACE                                              # accepted: tile-local
    p.norm = B.dit_qk_norm(B.DIT_NORM_HEAD, 1e-6, None, 0x20004)
    assert call(p) == B.DIT_ERR_ALIGNMENT
    p.norm = B.dit_qk_norm(B.DIT_NORM_TOKEN, 1e-6, None, None)
    assert call(p) == B.DIT_ERR_WORKSPACE                                              # accepted: a second pass


def test_qk_norm_arguments():
    L, H = 24, 2
    base = B.dit_attn_workspace_bytes(self_params())
    p = self_params()
    p.norm = B.dit_qk_norm(B.DIT_NORM_HEAD, 1e-6, None, None)
    assert B.dit_attn_workspace_bytes(p) == base                    # per-head statistics need no table
    p.norm.mode = B.DIT_NORM_TOKEN
    assert B.dit_attn_workspace_bytes(p) == base + 2 * up(4 * L)    # one fp32 factor per q row and per k row
    p.norm.mode = 3
    assert call_self(p) == B.DIT_ERR_INVALID_ARG
    p.norm = B.dit_qk_norm(B.DIT_NORM_HEAD, -1.0, None, None)
    assert call_self(p) == B.DIT_ERR_INVALID_ARG
    p.norm = B.dit_qk_norm(B.DIT_NORM_HEAD, float("nan"), None, None)
    assert call_self(p) == B.DIT_ERR_INVALID_ARG
    p.norm = B.dit_qk_norm(B.DIT_NORM_HEAD, 1e-6, 0x20004, None)
    assert call_self(p) == B.DIT_ERR_ALIGNMENT
    p = self_params(flags=B.DIT_FLAG_KV_FUSED | B.DIT_FLAG_PV_BF16)
    p.norm = B.dit_qk_norm(B.DIT_NORM_HEAD, 1e-6, None, None)
    assert call_self(p) == B.DIT_ERR_UNSUPPORTED
    c = cross_params()
    cbase = B.dit_cross_attn_workspace_bytes(c)
    c.norm = B.dit_qk_norm(B.DIT_NORM_TOKEN, 1e-6, None, None)
    assert B.dit_cross_attn_workspace_bytes(c) == cbase + up(4 * 2 * 100) + up(4 * 2 * 769)
    c.norm.mode = -1
    assert call_cross(c) == B.DIT_ERR_INVALID_ARG
    v = varlen_params()
    vbase = B.dit_attn_varlen_workspace_bytes(v)
    v.norm = B.dit_qk_norm(B.DIT_NORM_TOKEN, 0.0, None, None)
    assert B.dit_attn_varlen_workspace_bytes(v) == vbase + 2 * up(4 * 49)


def varlen_params(grids=((2, 3, 4), (1, 5, 5)), H=2, D=128, split=(44, 42, 42), flags=0):
    arr = (B.dit_grid * max(len(grids), 1))(*[B.dit_grid(*g) for g in grids])
    s = B.dit_strides(0, H * D, D)
    p = B.dit_varlen_attn_params(len(grids), H, D, ctypes.cast(arr, ctypes.POINTER(B.dit_grid)), 0, 0, 0,
                                 split[0], split[1], split[2], 10000.0, 0.0, B.DIT_BF16, B.DIT_BF16, flags,
                                 s, s, s, s)
    p._keep = arr
    return p


def call_varlen(p, q=FAKE, ws=0x10000, ws_bytes=1 << 40):
    return B.lib().dit_attn_varlen_forward(q, FAKE, FAKE, FAKE, None, ctypes.byref(p), ws, ws_bytes, None)


def test_varlen_workspace_and_rejections():
    tile = 36 * 1024
    grids = ((2, 3, 4), (1, 5, 5), (3, 9, 9))  # 24, 25, 243 tokens -> 1 + 1 + 4 key tiles
    p = varlen_params(grids, H=3)
    table = 3 * 22 + 9 * 21 + 9 * 21  # longest extent per axis x pairs per axis
    assert B.dit_attn_varlen_workspace_bytes(p) == up(table * 8) + up(6 * 3 * tile)
    assert call_varlen(p, ws_bytes=B.dit_attn_varlen_workspace_bytes(p) - 1) == B.DIT_ERR_WORKSPACE
    assert call_varlen(p, q=0) == B.DIT_ERR_INVALID_ARG
    assert call_varlen(varlen_params(((2, 0, 4),))) == B.DIT_ERR_INVALID_ARG
    assert call_varlen(varlen_params(())) == B.DIT_ERR_INVALID_ARG
    assert call_varlen(varlen_params(((1, 1, 1),) * (B.DIT_MAX_REQUESTS + 1))) == B.DIT_ERR_UNSUPPORTED
    assert B.dit_attn_varlen_workspace_bytes(varlen_params(((1, 1, 1),) * B.DIT_MAX_REQUESTS)) > 0
    assert call_varlen(varlen_params(((256, 256, 256), (1, 1, 1)))) == B.DIT_ERR_UNSUPPORTED  # > 2^24 tokens
    assert call_varlen(varlen_params(split=(44, 42, 40))) == B.DIT_ERR_INVALID_ARG
    for f in (B.DIT_FLAG_KV_FUSED | B.DIT_FLAG_PV_BF16, B.DIT_FLAG_WIDE_QTILE, B.DIT_FLAG_SIMPLE_SCHEDULE):
        assert call_varlen(varlen_params(flags=f)) == B.DIT_ERR_UNSUPPORTED
    p = varlen_params()
    p.grids = None
    assert call_varlen(p) == B.DIT_ERR_INVALID_ARG
    p = varlen_params()
    p.sk.token = 2 * 128 + 4
    assert call_varlen(p) == B.DIT_ERR_ALIGNMENT


def linear_call(M=64, N=64, K=64, ldx=None, ldw=None, ldy=None, out_dtype=None, flags=0, x=FAKE, w=FAKE, y=FAKE,
                bias=None):
    p = B.dit_linear_params(M, N, K, K if ldx is None else ldx, K if ldw is None else ldw, N if ldy is None else ldy,
                            B.DIT_BF16 if out_dtype is None else out_dtype, flags)
    return B.lib().dit_linear_forward(x, w, bias, y, ctypes.byref(p), None)


def test_linear_rejects_bad_arguments():
    for kw in (dict(x=0), dict(w=0), dict(y=0), dict(M=0), dict(N=0), dict(K=0), dict(flags=1), dict(out_dtype=2),
               dict(ldx=56), dict(ldw=56), dict(ldy=56)):
        assert linear_call(**kw) == B.DIT_ERR_INVALID_ARG, kw
    assert B.lib().dit_linear_forward(FAKE, FAKE, None, FAKE, None, None) == B.DIT_ERR_INVALID_ARG
    for kw in (dict(K=96), dict(N=60), dict(K=8), dict(ldx=(1 << 22) + 8), dict(ldw=(1 << 22) + 8)):
        assert linear_call(**kw) == B.DIT_ERR_UNSUPPORTED, kw
    for kw in (dict(x=FAKE + 8), dict(w=FAKE + 2), dict(y=FAKE + 4), dict(ldx=68), dict(ldw=70), dict(ldy=68),
               dict(bias=FAKE + 4), dict(out_dtype=B.DIT_F32, ldy=66)):
        assert linear_call(**kw) == B.DIT_ERR_ALIGNMENT, kw


def test_overlapping_rows_are_rejected():
    """Rows of D channels may not overlap: an output layout whose rows share memory would let workgroups race."""
    L, H, D = 24, 2, 128
    ok_layouts = [
        B.dit_strides(L * H * D, H * D, D),          # [B, L, H, D]
        B.dit_strides(L * H * D, D, L * D),          # [B, H, L, D]
        B.dit_strides(H * D, 2 * H * D, D),          # [L, B, H, D]: batches interleaved
        B.dit_strides(3 * L * H * D, 3 * H * D, D),  # a q/k/v-fused buffer: token stride 3*H*D
    ]
    for st in ok_layouts:
        p = self_params(B_=2)
        p.so = st
        assert call_self_no_launch(p) == B.DIT_ERR_WORKSPACE, (st.batch, st.token, st.head)  # accepted
    bad_layouts = [
        B.dit_strides(L * H * D, 64, D),             # token stride shorter than a row
        B.dit_strides(L * H * D, H * D, 64),         # head stride shorter than a row
        B.dit_strides(L * H * D, D, D),              # heads on top of tokens
        B.dit_strides(L * H * D, H * D - 8, D),      # token stride does not clear the H heads of a token
        B.dit_strides(L * H * D, D, (L - 1) * D),    # head stride does not clear the L tokens of a head
        B.dit_strides(64, H * D, D),                 # batch stride shorter than a row
    ]
    for st in bad_layouts:
        for field in ("sq", "sk", "sv", "so"):
            p = self_params(B_=2)
            setattr(p, field, st)
            assert call_self_no_launch(p) == B.DIT_ERR_INVALID_ARG, (field, st.batch, st.token, st.head)
    # one head: the token stride alone decides
    p = self_params(H=1, split=(44, 42, 42))
    p.so = B.dit_strides(L * 128, 64, 128)
    assert call_self_no_launch(p) == B.DIT_ERR_INVALID_ARG
    c = cross_params()
    c.so = B.dit_strides(100 * 2 * 128, 128, 128)
    assert call_cross(c) == B.DIT_ERR_INVALID_ARG
    v = varlen_params()
    v.so = B.dit_strides(0, 64, 128)
    assert call_varlen(v) == B.DIT_ERR_INVALID_ARG


def test_python_wrappers_check_extents_before_any_call():
    """The wrappers refuse tensors whose shapes, dtypes or grid do not match what the C side will address
    (checked on host tensors: the shape checks come before the device check)."""
    import torch

    def t(*shape, dtype=torch.bfloat16):
        return torch.zeros(shape, dtype=dtype)

    q = t(1, 24, 2, 128)
    grid, split = (2, 3, 4), (44, 42, 42)
    with pytest.raises(ValueError, match="grid"):
        B.dit_attn_forward(q, q, q, (2, 3, 5), split)
    with pytest.raises(ValueError, match="k has shape"):
        B.dit_attn_forward(q, t(1, 23, 2, 128), q, grid, split)
    with pytest.raises(ValueError, match="v has shape"):
        B.dit_attn_forward(q, q, t(1, 24, 1, 128), grid, split)
    with pytest.raises(ValueError, match="share one dtype"):
        B.dit_attn_forward(q, t(1, 24, 2, 128, dtype=torch.float32), q, grid, split)
    with pytest.raises(ValueError, match="out has shape"):
        B.dit_attn_forward(q, q, q, grid, split, out=t(1, 24, 2, 64))
    with pytest.raises(ValueError, match="lse"):
        B.dit_attn_forward(q, q, q, grid, split, lse=torch.zeros((1, 24, 2)))
    kc = t(1, 77, 2, 128)
    with pytest.raises(ValueError, match="v has shape"):
        B.dit_cross_attn_forward(q, kc, t(1, 76, 2, 128))
    with pytest.raises(ValueError, match="k has shape"):
        B.dit_cross_attn_forward(q, t(2, 77, 2, 128), t(2, 77, 2, 128))
    with pytest.raises(ValueError, match="share one dtype"):
        B.dit_cross_attn_forward(q, kc, t(1, 77, 2, 128, dtype=torch.float32))
    with pytest.raises(ValueError, match="kv_valid"):
        B.dit_cross_attn_forward(q, kc, kc, torch.zeros((1, 76), dtype=torch.uint8))
    with pytest.raises(ValueError, match="kv_valid"):
        B.dit_cross_attn_forward_static(q, kc, kc, torch.zeros((1, 77), dtype=torch.int32), out=q)
    qv = t(24, 2, 128)
    with pytest.raises(ValueError, match="grids"):
        B.dit_attn_varlen_forward(qv, qv, qv, [(2, 3, 4), (1, 1, 1)], split)
    with pytest.raises(ValueError, match="k has shape"):
        B.dit_attn_varlen_forward(qv, t(25, 2, 128), qv, [(2, 3, 4)], split)
    # everything fits, but the tensors are on the host
    with pytest.raises(ValueError, match="device"):
        B.dit_attn_forward(q, q, q, grid, split)


def test_python_wrappers_refuse_host_tensors():
    import torch

    q = torch.zeros((1, 24, 2, 128), dtype=torch.bfloat16)
    with pytest.raises(ValueError):
        B.dit_attn_forward(q, q, q, (2, 3, 4), (44, 42, 42))
    with pytest.raises(ValueError):
        B.dit_cross_attn_forward(q, q, q)


@pytest.mark.parametrize("compiler,std", [("gcc", "-std=c99"), ("gcc", "-std=c11"), ("g++", "-std=c++11")])
def test_public_header_is_plain_c(compiler, std, tmp_path):
    """The boundary is a C ABI: the header must compile on its own as C99, C11 and C++ with no
    HIP or torch header in sight, and the structs must have the layout the Python binding mirrors."""
    import shutil
    import subprocess

    if shutil.which(compiler) is None:
        pytest.skip(compiler + " not found")
    src = tmp_path / ("t.c" if compiler == "gcc" else "t.cpp")
    src.write_text(
        '#include "dit_attn.h"\n#include <stdio.h>\n'
        "int main(void) {\n"
        '  printf("%zu %zu %zu %zu %zu %zu %zu\\n", sizeof(dit_strides), sizeof(dit_qk_norm), sizeof(dit_self_attn_params),\n'
        "         sizeof(dit_cross_attn_params), sizeof(dit_varlen_attn_params), sizeof(dit_grid),\n"
        "         sizeof(dit_linear_params));\n"
        "  return 0;\n}\n")
    exe = str(tmp_path / "t")
    subprocess.check_call([compiler, std, "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", os.path.join(ROOT, "include"),
                           str(src), "-o", exe])
    sizes = [int(x) for x in subprocess.check_output([exe]).split()]
    assert sizes == [ctypes.sizeof(B.dit_strides), ctypes.sizeof(B.dit_qk_norm), ctypes.sizeof(B.dit_self_attn_params),
                     ctypes.sizeof(B.dit_cross_attn_params), ctypes.sizeof(B.dit_varlen_attn_params),
                     ctypes.sizeof(B.dit_grid), ctypes.sizeof(B.dit_linear_params)]


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU; asking for more exits with a message instead of a number."""
    import subprocess
    import sys

    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], stdout=subprocess.PIPE,
                       stderr=subprocess.PIPE, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_static_workspace_rejects_what_does_not_fit():
    # 8 x 64 heads x 13 tiles x 36 KiB = 234 MiB of tiles: beyond the array; refused before any launch
    Bz, Lq, Lk, H, D = 8, 64, 769, 64, 128
    sq = B.dit_strides(Lq * H * D, H * D, D)
    sk = B.dit_strides(Lk * H * D, H * D, D)
    p = B.dit_cross_attn_params(Bz, H, D, Lq, Lk, 0.0, B.DIT_BF16, B.DIT_BF16, 0, 0, sq, sk, sk, sq)
    assert B.dit_cross_attn_workspace_bytes(p) > B.DIT_STATIC_WORKSPACE_BYTES
    fake = 0x1000
    st = B.lib().dit_cross_attn_forward_static(fake, fake, fake, None, fake, None, ctypes.byref(p), None)
    assert st == B.DIT_ERR_WORKSPACE
    # invalid parameters come back with the ordinary entry point's status
    p.D = 96
    st = B.lib().dit_cross_attn_forward_static(fake, fake, fake, None, fake, None, ctypes.byref(p), None)
    assert st == B.DIT_ERR_UNSUPPORTED


def test_counter_summary_is_of_this_library_version():
    """bench.py reports the measured HBM traffic of the headline kernel only when the counter summary under
    profiles/ names the version of the library that runs: a summary left behind by an older version would turn the
    figure into null without anybody noticing."""
    import importlib.util
    import os

    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    spec = importlib.util.spec_from_file_location("bench_for_test", os.path.join(root, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    traffic = bench.traffic_bytes_for(B.dit_attn_version())
    assert traffic is not None and 1e9 < traffic < 1e10
    assert bench.traffic_bytes_for(B.dit_attn_version() + 1) is None
