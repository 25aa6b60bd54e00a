"""GPU checks of the 8-bit score path (DIT_FLAG_QK_FP8) against the CPU fp64 oracle.

This path does NOT meet the 16-bit parity bar and is never the default.  Its contract follows from the operand
format (E4M3, 3 stored mantissa bits, round to nearest even, one power-of-two factor per q' and k' row; the
reading is written out in tests/fp8_error_model.py and in the design notes) and nothing else:

THE CREDITED CHECK is against the plain definition, oracle.self_attn (and its normalised / packed forms), which
knows nothing of 8-bit operands.  tests/fp8_error_model.py derives, by first-order propagation of independent
rounding errors of the format's own step size, the standard deviation s_nc each output element's error should
have.  Every element must then satisfy
      |gpu - oracle|  <=  1.15 * z(N) * s_nc  +  the ordinary 16-bit bar (2e-2 x output RMS),
z(N) = the two-sided Gaussian quantile at which N elements hold 0.01 expected exceedances (5.3 at 65 thousand
elements, 6.0 at 3 million), 1.15 = room for the first-order and independence approximations; and, where there
are enough elements for a statistic, the RMS of (gpu - oracle) / s_nc must lie in [0.85, 1.15]: an error as
small as the 16-bit path's would mean the flag was ignored, a larger one that something besides the format's
rounding adds error.  No constant here is fitted to an observed run; the model itself is checked on the CPU
(tests/test_fp8_error_model.py) against the quantiser written out in numpy.

A SECONDARY, labelled check compares with oracle.self_attn_fp8_scores, a numpy MODEL of the quantiser written
after the kernel; it is a diagnostic for the row-factor and rounding rules, not the parity evidence.
"""
import numpy as np
import pytest

import oracle
import fp8_error_model as em
from paper_2601_20655_amd import binding as B
from paper_2601_20655_amd import workloads as wl
from gpu_util import TOL, bf16_half_ulp, to_dev, to_f64

pytestmark = pytest.mark.gpu

FP8 = B.DIT_FLAG_QK_FP8
SHAPES = {"auto": 0, "4w": B.DIT_FLAG_SMALL_WORKGROUP, "8w": B.DIT_FLAG_BIG_WORKGROUP}
MARGIN = 1.15          # first-order / independence approximations of the error model
RMS_WINDOW = (0.85, 1.15)
MIN_FOR_STATISTIC = 20000


def check(gpu, ref, pred, what="", bf16_out=False):
    """Element-wise bound from the predicted error std `pred` plus the 16-bit bar; RMS window where n allows."""
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert gpu.shape == ref.shape == pred.shape and np.all(np.isfinite(gpu)), what
    rms = float(np.sqrt(np.mean(ref * ref)))
    err = np.abs(gpu - ref)
    z_tail = em.gaussian_tail_z(ref.size)
    allow = MARGIN * z_tail * pred + TOL * rms + (bf16_half_ulp(ref) if bf16_out else 0.0)
    worst = float(np.max(err / allow))
    zr = float(np.sqrt(np.mean((err / np.maximum(pred, 1e-300))[pred > 0] ** 2))) if np.any(pred > 0) else 0.0
    print("%s: %d elements, RMS err %.3e, max err %.3e (x output RMS); RMS of err/predicted %.3f; "
          "largest err/allowed %.3f (z = %.2f)" % (what, ref.size, float(np.sqrt(np.mean(err * err))) / rms,
                                                   float(err.max()) / rms, zr, worst, z_tail))
    assert worst <= 1.0, what
    if ref.size >= MIN_FOR_STATISTIC:
        assert RMS_WINDOW[0] <= zr <= RMS_WINDOW[1], what
    return zr


def run_self(cfg, q, k, v, **kw):
    import torch

    res = B.dit_attn_forward(to_dev(q), to_dev(k), to_dev(v), cfg["grid"], cfg["split"], **kw)
    torch.cuda.synchronize()
    return res


_CASES = {}


def case(name):
    """(q, k, v, oracle output, oracle lse, predicted error std of out, of lse) of a named config, computed once."""
    if name not in _CASES:
        cfg = wl.CONFIGS[name]
        q, k, v = wl.self_attn_inputs(cfg)
        ref, ref_lse = oracle.self_attn(q, k, v, cfg["grid"], cfg["split"], want_lse=True)
        pred, pred_lse = em.predicted_std_self(q, k, v, cfg["grid"], cfg["split"], want_lse=True)
        _CASES[name] = (q, k, v, ref, ref_lse, pred, pred_lse)
    return _CASES[name]


@pytest.mark.parametrize("shape", sorted(SHAPES))
@pytest.mark.parametrize("pv", [0, B.DIT_FLAG_PV_BF16])
def test_mid_config_all_rows(shape, pv):
    """6,240 tokens x 4 heads x d128 (97.5 key tiles: ragged tail), every row, plus the log-sum-exp."""
    import torch

    cfg = wl.CONFIGS["mid"]
    q, k, v, ref, ref_lse, pred, pred_lse = case("mid")
    out, lse = run_self(cfg, q, k, v, flags=FP8 | SHAPES[shape] | pv, out_dtype=torch.float32, want_lse=True)
    check(to_f64(out), ref, pred, what="mid %s pv=%d" % (shape, pv))
    # the log-sum-exp: its own predicted spread, plus the 5e-3 the 16-bit tests allow it
    dl = np.abs(to_f64(lse) - ref_lse)
    assert np.all(dl <= MARGIN * em.gaussian_tail_z(dl.size) * pred_lse + 5e-3)
    out = run_self(cfg, q, k, v, flags=FP8 | SHAPES[shape] | pv)
    check(to_f64(out), ref, pred, what="mid %s pv=%d, bf16 out" % (shape, pv), bf16_out=True)


def test_tiny_config_d64_fp32_inputs():
    import torch

    cfg = wl.CONFIGS["tiny"]
    q, k, v, ref, _, pred, _ = case("tiny")
    for shape in sorted(SHAPES):
        out = run_self(cfg, q, k, v, flags=FP8 | SHAPES[shape], out_dtype=torch.float32)
        check(to_f64(out), ref, pred, what="tiny %s" % shape)


@pytest.mark.parametrize("grid", [(1, 1, 1), (1, 1, 2), (1, 3, 21), (1, 1, 64), (1, 5, 13), (2, 8, 8), (1, 3, 43),
                                  (3, 7, 19)])
@pytest.mark.parametrize("D", [64, 128])
def test_ragged_sizes(grid, D):
    """Token counts 1 .. 399 around the tile boundaries (too few elements for the RMS statistic below 20,000:
    the element-wise bound alone); a single token must come back exactly (P = 1)."""
    import torch

    split = (22, 20, 22) if D == 64 else (44, 42, 42)
    cfg = dict(B=2, grid=grid, H=3, D=D, split=split, dtype="bf16", seed=99 + D + grid[2])
    q, k, v = wl.self_attn_inputs(cfg)
    ref = oracle.self_attn(q, k, v, grid, split)
    pred = em.predicted_std_self(q, k, v, grid, split)
    for shape in sorted(SHAPES):
        out = to_f64(run_self(cfg, q, k, v, flags=FP8 | SHAPES[shape], out_dtype=torch.float32))
        if int(np.prod(grid)) == 1:
            assert np.array_equal(out, ref)
        else:
            check(out, ref, pred, what="ragged %s D=%d %s" % (grid, D, shape))


def test_wider_scores_scale_the_error():
    """q, k scaled x2 with scale 0.11: scores ~ N(0, 5^2), non-zero origin, other base.  The error follows the
    score spread (9e-2 x output RMS here), and the model follows it element by element."""
    import torch

    cfg = dict(B=1, grid=(3, 9, 17), H=2, D=128, split=(44, 42, 42), dtype="bf16", seed=4242)
    q, k, v = wl.self_attn_inputs(cfg, gain=2.0)
    kw = dict(origin=(5, -3, 11), scale=0.11)
    ref = oracle.self_attn(q, k, v, cfg["grid"], cfg["split"], base=500.0, **kw)
    pred = em.predicted_std_self(q, k, v, cfg["grid"], cfg["split"], base=500.0, **kw)
    out = run_self(cfg, q, k, v, flags=FP8, out_dtype=torch.float32, rope_base=500.0, **kw)
    check(to_f64(out), ref, pred, what="peaky")


def test_normalised_q_k_and_packed_requests():
    """Token-mode q/k normalisation ahead of the 8-bit rounding; packed requests of mixed sizes."""
    import torch

    cfg = wl.CONFIGS["mid"]
    q, k, v = wl.self_attn_inputs(cfg, gain=3.0)
    gq, gk = wl.norm_weights(cfg)
    ref = oracle.self_attn_normed(q, k, v, cfg["grid"], cfg["split"], gq, gk, 1e-6, "token")
    pred = em.predicted_std_self(q, k, v, cfg["grid"], cfg["split"],
                                 q_rot_in=oracle.qk_rmsnorm(q, gq, 1e-6, "token"),
                                 k_rot_in=oracle.qk_rmsnorm(k, gk, 1e-6, "token"))
    out = run_self(cfg, q, k, v, flags=FP8, out_dtype=torch.float32, norm=("token", 1e-6, to_dev(gq), to_dev(gk)))
    check(to_f64(out), ref, pred, what="mid normed")

    cfg = wl.CONFIGS["varlen_small"]
    q, k, v = wl.varlen_attn_inputs(cfg)
    ref = oracle.self_attn_packed(q, k, v, cfg["grids"], cfg["split"])
    pred = np.empty_like(ref)
    t0 = 0
    for g in cfg["grids"]:  # a token attends within its own request (requests of 1 to 1,024 tokens)
        n = g[0] * g[1] * g[2]
        pred[t0:t0 + n] = em.predicted_std_self(q[None, t0:t0 + n], k[None, t0:t0 + n], v[None, t0:t0 + n], g,
                                                cfg["split"])[0]
        t0 += n
    for shape in sorted(SHAPES):
        out = B.dit_attn_varlen_forward(to_dev(q), to_dev(k), to_dev(v), cfg["grids"], cfg["split"],
                                        flags=FP8 | SHAPES[shape], out_dtype=torch.float32)
        torch.cuda.synchronize()
        check(to_f64(out), ref, pred, what="packed requests %s" % shape)


def test_full_size_sampled_rows_and_resident_tiles():
    """32,760 tokens x 40 heads x d128, the shape the benchmark times (8-wavefront workgroups): sampled
    rows of every head; then a second call on the resident 8-bit tiles returns the same bits."""
    import torch

    cfg = wl.CONFIGS["dit_14b"]
    q, k, v = wl.self_attn_inputs(cfg)
    rows = wl.sample_rows(q.shape[1], cfg["seed"], edge=64, n_random=128)
    ref = oracle.self_attn(q, k, v, cfg["grid"], cfg["split"], rows=rows)
    pred = em.predicted_std_self(q, k, v, cfg["grid"], cfg["split"], rows=rows)
    qd, kd, vd = to_dev(q), to_dev(k), to_dev(v)
    p = B.self_attn_params(qd, kd, vd, qd, cfg["grid"], cfg["split"], flags=FP8)
    ws = torch.empty(B.dit_attn_workspace_bytes(p), dtype=torch.uint8, device="cuda")
    out = B.dit_attn_forward(qd, kd, vd, cfg["grid"], cfg["split"], flags=FP8, workspace=ws)
    torch.cuda.synchronize()
    check(to_f64(out[:, torch.from_numpy(rows).cuda()]), ref, pred, what="dit_14b sampled rows, bf16 out",
          bf16_out=True)
    out2 = B.dit_attn_forward(qd, kd, vd, cfg["grid"], cfg["split"], flags=FP8 | B.DIT_FLAG_KV_RESIDENT,
                              workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(out, out2)


# ---- secondary: against the numpy MODEL of the quantiser (not the parity evidence) ----

# An operand whose fp32 value on the GPU and fp64 value in the model fall on different sides of an E4M3 rounding
# boundary moves by a whole 8-bit step.  With a relative fp32-vs-fp64 difference of at most 2^-23 (rotation:
# two products, one sum, table entries rounded to fp32; then the scale fold) and boundaries one step = 2^-3 / m
# apart relative to an operand of significand m in [1, 2) (mean of m over a log-uniform significand: 1.44), an
# operand straddles a boundary with probability at most 8 * 1.44 * 2^-23 = 1.4e-6.  A flipped q' operand moves
# all D outputs of its row: at most D * 1.4e-6 of the rows, hence of the elements, may leave the 16-bit bar;
# the test allows twice that.  How far: the row's scores move by step(q'_c) * k'_c <= 2^-3 * max|q'| * k'_c in
# base-2 units, which is the error model's own per-key term with step(q') in place of step(q') / sqrt(12) in one
# channel: no more than sqrt(12) / sqrt(D) * max|q'| / rms(q') times the row's predicted std summed over all
# channels -- bounded here by the element's allowance of the credited check.
P_FLIP = 8.0 * 1.44 * 2.0 ** -23


def close_to_model(gpu, ref8, pred, D, what):
    rms = float(np.sqrt(np.mean(ref8 * ref8)))
    err = np.abs(np.asarray(gpu, dtype=np.float64) - ref8)
    beyond = int((err > TOL * rms).sum())
    allowed = 2.0 * D * P_FLIP * err.size
    print("%s: max|err|/RMS = %.3e, %d of %d elements beyond 2e-2 (allowed %.1f)" % (
        what, err.max() / rms, beyond, err.size, allowed))
    assert np.all(np.isfinite(gpu)) and beyond <= max(allowed, 1.0), what
    assert np.all(err <= MARGIN * em.gaussian_tail_z(err.size) * pred + TOL * rms), what


@pytest.mark.parametrize("name", ["tiny", "mid"])
def test_matches_the_model_of_the_quantiser(name):
    """Against oracle.self_attn_fp8_scores (numpy: same power-of-two row factors, ties to even) what remains is
    fp32 vs fp64 arithmetic and the 16-bit rounding of P and V: the ordinary 16-bit bar, except where an operand
    sits on a rounding boundary (derivation above)."""
    import torch

    cfg = wl.CONFIGS[name]
    q, k, v = wl.self_attn_inputs(cfg)
    kw = dict(origin=(2, -3, 1), scale=0.1)
    ref8 = oracle.self_attn_fp8_scores(q, k, v, cfg["grid"], cfg["split"], **kw)
    pred = em.predicted_std_self(q, k, v, cfg["grid"], cfg["split"], **kw)
    for shape in sorted(SHAPES):
        out = run_self(cfg, q, k, v, flags=FP8 | SHAPES[shape], out_dtype=torch.float32, **kw)
        close_to_model(to_f64(out), ref8, pred, cfg["D"], "%s %s vs quantiser model" % (name, shape))
    # and the packed-request entry point on one request
    out = B.dit_attn_varlen_forward(to_dev(q)[0], to_dev(k)[0], to_dev(v)[0], [cfg["grid"]], cfg["split"], flags=FP8,
                                    out_dtype=torch.float32, **kw)
    torch.cuda.synchronize()
    close_to_model(to_f64(out), ref8[0], pred[0], cfg["D"], "%s packed entry point vs quantiser model" % name)
