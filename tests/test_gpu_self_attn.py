"""GPU parity of dit_attn_forward (through the C ABI) against the CPU fp64 oracle."""
import numpy as np
import pytest

import oracle
from paper_2601_20655_amd import binding as B
from paper_2601_20655_amd import workloads as wl
from gpu_util import TOL, compare, to_dev, to_f64

pytestmark = pytest.mark.gpu

VARIANTS = {
    "default_f16_f16": 0,
    "qk_f16_pv_bf16": B.DIT_FLAG_QK_F16 | B.DIT_FLAG_PV_BF16,
}


def run_self(cfg, q, k, v, flags=0, out_dtype=None, origin=(0, 0, 0), want_lse=False, scale=0.0, base=10000.0):
    import torch

    qd, kd, vd = to_dev(q), to_dev(k), to_dev(v)
    res = B.dit_attn_forward(qd, kd, vd, cfg["grid"], cfg["split"], origin=origin, flags=flags,
                             out_dtype=out_dtype, want_lse=want_lse, scale=scale, rope_base=base)
    torch.cuda.synchronize()
    return res


def test_tiny_config_fp32_inputs_all_rows():
    import torch

    cfg = wl.CONFIGS["tiny"]
    q, k, v = wl.self_attn_inputs(cfg)
    ref, ref_lse = oracle.self_attn(q, k, v, cfg["grid"], cfg["split"], want_lse=True)
    out, lse = run_self(cfg, q, k, v, out_dtype=torch.float32, want_lse=True)
    compare(to_f64(out), ref, what="tiny f32->f32")
    assert np.max(np.abs(to_f64(lse) - ref_lse)) < 5e-3
    out = run_self(cfg, q, k, v, flags=B.DIT_FLAG_WIDE_QTILE, out_dtype=torch.float32)
    compare(to_f64(out), ref, what="tiny f32->f32 wide")
    # same config with inputs pre-rounded to bf16 (comparable with the bf16 configs)
    qb, kb, vb = wl.self_attn_inputs(cfg, dtype="bf16")
    refb = oracle.self_attn(qb, kb, vb, cfg["grid"], cfg["split"])
    outb = run_self(cfg, qb, kb, vb, out_dtype=torch.float32)
    compare(to_f64(outb), refb, what="tiny bf16->f32")
    outb = run_self(cfg, qb, kb, vb)
    compare(to_f64(outb), refb, bf16_out=True, what="tiny bf16->bf16")


SHAPES = {
    "auto": 0,
    "qb1_4w": B.DIT_FLAG_SMALL_WORKGROUP,
    "qb2_4w": B.DIT_FLAG_WIDE_QTILE,
    "qb1_8w": B.DIT_FLAG_BIG_WORKGROUP,
    # the same pipeline on 32x32x16 matrix instructions (the default runs on 16x16x32)
    "m32_4w": B.DIT_FLAG_MFMA_32X32 | B.DIT_FLAG_SMALL_WORKGROUP,
    "m32_8w": B.DIT_FLAG_MFMA_32X32 | B.DIT_FLAG_BIG_WORKGROUP,
    "simple_qb1": B.DIT_FLAG_SIMPLE_SCHEDULE,
    "simple_qb2": B.DIT_FLAG_SIMPLE_SCHEDULE | B.DIT_FLAG_WIDE_QTILE,
}


@pytest.mark.parametrize("name", sorted(VARIANTS))
@pytest.mark.parametrize("wide", sorted(SHAPES))
def test_mid_config_all_rows(name, wide):
    """6,240 tokens x 4 heads: 98 key tiles (ragged tail of 32), all rows compared, for every
    operand-type variant and every kernel shape (query rows per wavefront, wavefronts per
    workgroup, pipelined or plain schedule)."""
    import torch

    cfg = wl.CONFIGS["mid"]
    q, k, v = wl.self_attn_inputs(cfg)
    ref = oracle.self_attn(q, k, v, cfg["grid"], cfg["split"])
    flags = VARIANTS[name] | SHAPES[wide]
    out = run_self(cfg, q, k, v, flags=flags, out_dtype=torch.float32)
    compare(to_f64(out), ref, what="mid %s wide=%s f32 out" % (name, wide))
    out = run_self(cfg, q, k, v, flags=flags)
    compare(to_f64(out), ref, bf16_out=True, what="mid %s wide=%s bf16 out" % (name, wide))


@pytest.mark.parametrize("pv", [B.DIT_FLAG_PV_BF16, B.DIT_FLAG_PV_F16])
def test_mid_config_bf16_score_operands_reported(pv):
    """q', k' re-rounded to bf16 (8 significant bits) after the rotation put max|err| at about
    2.5e-2 x RMS over 3.2M outputs -- past the 2e-2 bar, which is why fp16 score operands are the
    default.  The variant is selectable; its error is printed and held to a looser 4e-2."""
    import torch

    cfg = wl.CONFIGS["mid"]
    q, k, v = wl.self_attn_inputs(cfg)
    ref = oracle.self_attn(q, k, v, cfg["grid"], cfg["split"])
    out = run_self(cfg, q, k, v, flags=B.DIT_FLAG_QK_BF16 | pv, out_dtype=torch.float32)
    compare(to_f64(out), ref, tol=4e-2, what="mid bf16 score operands, pv flag %d, f32 out" % pv)


@pytest.mark.parametrize("wide", [False, True])
def test_fused_rope_on_load(wide):
    import torch

    cfg = wl.CONFIGS["mid"]
    q, k, v = wl.self_attn_inputs(cfg)
    ref, ref_lse = oracle.self_attn(q, k, v, cfg["grid"], cfg["split"], want_lse=True)
    flags = B.DIT_FLAG_KV_FUSED | B.DIT_FLAG_PV_BF16 | (B.DIT_FLAG_WIDE_QTILE if wide else 0)
    out, lse = run_self(cfg, q, k, v, flags=flags, out_dtype=torch.float32, want_lse=True)
    compare(to_f64(out), ref, what="mid fused wide=%s" % wide)
    assert np.max(np.abs(to_f64(lse) - ref_lse)) < 5e-3


@pytest.mark.parametrize("grid", [(1, 1, 1), (1, 1, 2), (1, 3, 21), (1, 1, 64), (1, 5, 13), (2, 8, 8), (1, 3, 43),
                                  (3, 7, 19)])
@pytest.mark.parametrize("D", [64, 128])
def test_ragged_sizes(grid, D):
    """Token counts 1, 2, 63, 64, 65, 128, 129, 399: below, at and just past tile boundaries."""
    import torch

    split = (22, 20, 22) if D == 64 else (44, 42, 42)
    cfg = dict(B=2, grid=grid, H=3, D=D, split=split, dtype="bf16", seed=99 + D + grid[2])
    q, k, v = wl.self_attn_inputs(cfg)
    ref, ref_lse = oracle.self_attn(q, k, v, grid, split, want_lse=True)
    for flags in tuple(SHAPES.values()) + ((B.DIT_FLAG_KV_FUSED | B.DIT_FLAG_PV_BF16,) if D == 128 else ()):
        out, lse = run_self(cfg, q, k, v, flags=flags, out_dtype=torch.float32, want_lse=True)
        compare(to_f64(out), ref, what="ragged %s D=%d flags=%d" % (grid, D, flags))
        assert np.max(np.abs(to_f64(lse) - ref_lse)) < 5e-3


@pytest.mark.parametrize("name", ["qb1_8w", "qb1_4w", "m32_8w", "m32_4w", "qb2_4w", "simple_qb1"])
def test_head_dim_64_steady_state_all_rows(name):
    """head_dim 64 over 68 key tiles and 17 (8-wavefront) or 34 query tiles per head: the key loop of each form
    in steady state (the ragged cases above end after seven tiles), every row against the oracle, fp32 inputs
    as in the tiny reference shape and bf16 inputs."""
    import torch

    for dtype, seed in (("bf16", 6401), ("f32", 6402)):
        cfg = dict(B=1, grid=(4, 32, 34), H=2, D=64, split=(22, 20, 22), dtype=dtype, seed=seed)
        q, k, v = wl.self_attn_inputs(cfg)
        ref, ref_lse = oracle.self_attn(q, k, v, cfg["grid"], cfg["split"], want_lse=True)
        out, lse = run_self(cfg, q, k, v, flags=SHAPES[name], out_dtype=torch.float32, want_lse=True)
        compare(to_f64(out), ref, what="d64, 4,352 tokens, %s, %s in" % (name, dtype))
        assert np.max(np.abs(to_f64(lse) - ref_lse)) < 5e-3


def test_peaky_softmax_origin_scale_base():
    """q, k scaled x2 with scale 0.11: scores ~ N(0, 5^2), the softmax concentrates on a few keys
    and the running maximum keeps moving; non-zero origin, explicit scale and base.  (Larger
    scores push the rounding of the 16-bit score operands themselves past the bar: the absolute
    score error grows with |score| while the bar is fixed.)"""
    import torch

    cfg = dict(B=1, grid=(3, 9, 17), H=2, D=128, split=(44, 42, 42), dtype="bf16", seed=4242)
    q, k, v = wl.self_attn_inputs(cfg, gain=2.0)
    ref = oracle.self_attn(q, k, v, cfg["grid"], cfg["split"], origin=(5, -3, 11), scale=0.11, base=500.0)
    for flags in tuple(SHAPES.values()) + (B.DIT_FLAG_KV_FUSED | B.DIT_FLAG_PV_BF16,):
        out = run_self(cfg, q, k, v, flags=flags, out_dtype=torch.float32, origin=(5, -3, 11), scale=0.11, base=500.0)
        compare(to_f64(out), ref, what="peaky flags=%d" % flags)


def test_head_major_layout_and_determinism():
    """[B, H, L, D] storage through strides; two runs are bitwise identical."""
    import torch

    cfg = dict(B=2, grid=(2, 6, 11), H=3, D=128, split=(44, 42, 42), dtype="bf16", seed=777)
    q, k, v = wl.self_attn_inputs(cfg)
    ref = oracle.self_attn(q, k, v, cfg["grid"], cfg["split"])
    qd, kd, vd = (to_dev(a).permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3) for a in (q, k, v))
    assert qd.stride(2) > qd.stride(1)
    out = torch.empty((2, 3, 132, 128), dtype=torch.float32, device="cuda").permute(0, 2, 1, 3)
    B.dit_attn_forward(qd, kd, vd, cfg["grid"], cfg["split"], out=out)
    torch.cuda.synchronize()
    compare(to_f64(out), ref, what="head-major layout")
    out2 = torch.empty_like(out)
    B.dit_attn_forward(qd, kd, vd, cfg["grid"], cfg["split"], out=out2)
    torch.cuda.synchronize()
    assert torch.equal(out, out2)


FULL = {
    "dit_1p3b": dict(edge=64, n_random=128),
    "dit_14b": dict(edge=64, n_random=128),
    "dit_14b_hires": dict(edge=64, n_random=32),
}


@pytest.mark.parametrize("name", sorted(FULL))
def test_full_size_sampled_rows(name):
    """The reference shapes at full size, default flags (the configuration the benchmark times);
    rows {0..63}, {L-64..L-1} and seeded random rows of every head are checked."""
    import torch

    cfg = wl.CONFIGS[name]
    q, k, v = wl.self_attn_inputs(cfg)
    L = q.shape[1]
    rows = wl.sample_rows(L, cfg["seed"], **FULL[name])
    ref = oracle.self_attn(q, k, v, cfg["grid"], cfg["split"], rows=rows)
    out = run_self(cfg, q, k, v, out_dtype=torch.float32)
    compare(to_f64(out[:, torch.from_numpy(rows).cuda()]), ref, what="%s f32 out" % name)
    del out
    out = run_self(cfg, q, k, v)
    compare(to_f64(out[:, torch.from_numpy(rows).cuda()]), ref, bf16_out=True, what="%s bf16 out" % name)
