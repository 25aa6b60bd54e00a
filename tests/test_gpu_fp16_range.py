"""What happens at the edge of the fp16 range.  The default MFMA operands are fp16, whose largest finite
value is 65504, while bf16 inputs can hold far larger magnitudes.  The documented behaviour: fp16 operands
saturate at +-65504 (the result is the definition applied to the clamped operands, finite and deterministic),
and DIT_FLAG_QK_BF16 | DIT_FLAG_PV_BF16 is the opt-out that keeps the whole bf16 range.

The expected values come from the oracle alone: for the saturating case it is given the same inputs with the
out-of-range entries clamped (as float32, since 65504 has no bf16 bit pattern)."""
import numpy as np
import pytest

import oracle
from paper_2601_20655_amd import binding as B
from paper_2601_20655_amd import workloads as wl
from gpu_util import compare, to_dev, to_f64

pytestmark = pytest.mark.gpu

BIG = 7.0e4  # finite in bf16 (rounds to 70144), beyond fp16
F16_MAX = 65504.0
BF16_ALL = B.DIT_FLAG_QK_BF16 | B.DIT_FLAG_PV_BF16


def plant(bits, rng, n, value):
    """Overwrite n random entries of a bf16 tensor with +-value; returns the positions."""
    x = wl.bf16_bits_to_f32(bits).copy()
    flat = x.reshape(-1)
    idx = rng.choice(flat.size, size=n, replace=False)
    flat[idx] = value * rng.choice([-1.0, 1.0], size=n)
    return wl.f32_to_bf16_bits(x), idx


def test_self_attention_values_beyond_fp16():
    """|v| = 7e4 in a few hundred entries: default flags give the clamped-v result, bf16 operands the exact one."""
    import torch

    cfg = dict(B=1, grid=(2, 9, 17), H=2, D=128, split=(44, 42, 42), dtype="bf16", seed=77)
    q, k, v = wl.self_attn_inputs(cfg)
    v_big, _ = plant(v, np.random.default_rng(5), 300, BIG)
    widen = wl.bf16_bits_to_f32
    v_clamped = np.clip(widen(v_big), -F16_MAX, F16_MAX)
    assert np.abs(widen(v_big)).max() > 7e4 and np.abs(v_clamped).max() == F16_MAX
    ref_clamped = oracle.self_attn(widen(q), widen(k), v_clamped, cfg["grid"], cfg["split"])
    ref_exact = oracle.self_attn(q, k, v_big, cfg["grid"], cfg["split"])
    assert np.abs(ref_clamped - ref_exact).max() > 0.05 * np.sqrt(np.mean(ref_exact ** 2))  # the clamp is visible

    qd, kd, vd = to_dev(q), to_dev(k), to_dev(v_big)
    for name, flags in (("default", 0), ("plain schedule", B.DIT_FLAG_SIMPLE_SCHEDULE)):
        out = B.dit_attn_forward(qd, kd, vd, cfg["grid"], cfg["split"], out_dtype=torch.float32, flags=flags)
        torch.cuda.synchronize()
        compare(to_f64(out), ref_clamped, what="v beyond fp16, %s: saturated operands" % name)
    # bf16 operands: no saturation, the exact definition.  The outputs that a huge value feeds are thousands of
    # times the others, so the bar is taken per element: the documented 4e-2 x RMS of bf16 score operands on the
    # scale of the ORDINARY outputs (those of the unplanted v) plus 2 % of the element's magnitude (bf16 P: 2^-9 per
    # probability, bf16 scores: a per cent or two of a probability) -- a third of the 6.6 % by which a clamp at
    # 65504 would lower the planted contributions, so the two behaviours stay distinguishable.
    out = B.dit_attn_forward(qd, kd, vd, cfg["grid"], cfg["split"], out_dtype=torch.float32, flags=BF16_ALL)
    torch.cuda.synchronize()
    rms_plain = np.sqrt(np.mean(oracle.self_attn(q, k, v, cfg["grid"], cfg["split"]) ** 2))
    # "the element itself" without cancellation between planted values of opposite sign: sum_j p_j |v_j|
    magnitude = oracle.self_attn(q, k, v_big & np.uint16(0x7FFF), cfg["grid"], cfg["split"])
    allow = 4e-2 * rms_plain + 2e-2 * magnitude
    got = to_f64(out)
    assert np.all(np.isfinite(got))
    assert np.all(np.abs(got - ref_exact) <= allow), "bf16 operands: max err/allowed %.3f" % np.max(
        np.abs(got - ref_exact) / allow)
    assert np.any(np.abs(ref_clamped - ref_exact) > 2.0 * allow)  # a saturating path would fail the line above


def test_cross_attention_keys_beyond_fp16():
    """|k| = 7e4 in one channel of four keys per (request, head); q is zero except for +-2^-10 in that channel,
    so the four keys score +-6.0 exactly (+-5.6 once clamped to 65504) against ~0 for all others: large enough
    to tell the clamped result from the exact one, small enough that operand rounding cannot flip anything.
    An unclamped fp16 conversion would make these keys infinite and the output NaN."""
    import torch

    cfg = dict(B=2, Lq=150, n_text=100, n_image=57, H=2, D=128, dtype="bf16", min_text=20, seed=78)
    q, k, v, valid, _ = wl.cross_attn_inputs(cfg)
    rng = np.random.default_rng(6)
    c0 = 37
    widen = wl.bf16_bits_to_f32
    qf = np.zeros(q.shape, dtype=np.float32)
    qf[..., c0] = 2.0 ** -10 * rng.choice([-1.0, 1.0], size=q.shape[:-1])
    kf = widen(k).copy()
    for b in range(cfg["B"]):
        keys_ok = np.flatnonzero(valid[b])
        for h in range(cfg["H"]):
            pick = rng.choice(keys_ok, size=4, replace=False)
            kf[b, pick[:2], h, c0] = BIG
            kf[b, pick[2:], h, c0] = -BIG
    q_bits, k_bits = wl.f32_to_bf16_bits(qf), wl.f32_to_bf16_bits(kf)
    assert np.array_equal(widen(q_bits), qf)
    ref_clamped = oracle.cross_attn(qf, np.clip(widen(k_bits), -F16_MAX, F16_MAX), widen(v), valid)
    ref_exact = oracle.cross_attn(q_bits, k_bits, v, valid)
    rms = np.sqrt(np.mean(ref_exact ** 2))
    assert np.abs(ref_clamped - ref_exact).max() > 3e-2 * rms  # the two behaviours can be told apart

    qd, kd, vd, md = to_dev(q_bits), to_dev(k_bits), to_dev(v), torch.from_numpy(valid).cuda()
    for name, flags in (("default", 0), ("pipelined", B.DIT_FLAG_PIPELINED_SCHEDULE)):
        out = B.dit_cross_attn_forward(qd, kd, vd, md, out_dtype=torch.float32, flags=flags)
        torch.cuda.synchronize()
        compare(to_f64(out), ref_clamped, what="k beyond fp16, %s: saturated operands" % name)
    out = B.dit_cross_attn_forward(qd, kd, vd, md, out_dtype=torch.float32, flags=BF16_ALL)
    torch.cuda.synchronize()
    compare(to_f64(out), ref_exact, what="k beyond fp16, bf16 operands: full range")
