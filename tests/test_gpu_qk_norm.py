"""GPU parity of the fused q/k RMS normalisation (per head or per token, ahead of the rotation)
in all three entry points, against the CPU fp64 oracle."""
import numpy as np
import pytest

import oracle
from paper_2601_20655_amd import binding as B
from paper_2601_20655_amd import workloads as wl
from gpu_util import compare, to_dev, to_f64

pytestmark = pytest.mark.gpu

EPS = 1e-6
SHAPES = {"auto": 0, "8w": B.DIT_FLAG_BIG_WORKGROUP, "plain": B.DIT_FLAG_SIMPLE_SCHEDULE,
          "plain_wide": B.DIT_FLAG_SIMPLE_SCHEDULE | B.DIT_FLAG_WIDE_QTILE,
          "m32_8w": B.DIT_FLAG_MFMA_32X32 | B.DIT_FLAG_BIG_WORKGROUP}


def dev_norm(mode, gq, gk, eps=EPS):
    return (mode, eps, to_dev(gq) if gq is not None else None, to_dev(gk) if gk is not None else None)


@pytest.mark.parametrize("mode", ["head", "token"])
@pytest.mark.parametrize("shape", sorted(SHAPES))
def test_mid_config_normed_all_rows(mode, shape):
    """6,240 tokens x 4 heads, q and k drawn with gain 3 (the normalisation removes it), random
    channel weights: all rows, pipelined and plain kernels."""
    import torch

    cfg = wl.CONFIGS["mid"]
    q, k, v = wl.self_attn_inputs(cfg, gain=3.0)
    gq, gk = wl.norm_weights(cfg)
    ref = oracle.self_attn_normed(q, k, v, cfg["grid"], cfg["split"], gq, gk, EPS, mode)
    out = B.dit_attn_forward(to_dev(q), to_dev(k), to_dev(v), cfg["grid"], cfg["split"], flags=SHAPES[shape],
                             out_dtype=torch.float32, norm=dev_norm(mode, gq, gk))
    torch.cuda.synchronize()
    compare(to_f64(out), ref, what="mid normed %s %s" % (mode, shape))


def test_tiny_fp32_inputs_no_weights_large_eps():
    """d64, fp32 inputs, no channel weights, an eps comparable with the mean square."""
    import torch

    cfg = wl.CONFIGS["tiny"]
    q, k, v = wl.self_attn_inputs(cfg)
    for mode in ("head", "token"):
        ref = oracle.self_attn_normed(q, k, v, cfg["grid"], cfg["split"], None, None, 0.5, mode)
        out = B.dit_attn_forward(to_dev(q), to_dev(k), to_dev(v), cfg["grid"], cfg["split"],
                                 out_dtype=torch.float32, norm=dev_norm(mode, None, None, 0.5))
        torch.cuda.synchronize()
        compare(to_f64(out), ref, what="tiny normed %s" % mode)


@pytest.mark.parametrize("mode", ["head", "token"])
@pytest.mark.parametrize("split", [0, 96])
def test_cross_attention_normed(mode, split):
    """Cross-attention (joint and decoupled) with normalised q and k, key-padding mask, batch 2."""
    import torch

    cfg = dict(wl.CONFIGS["cross_14b"], B=2, Lq=300, H=3, n_text=96, n_image=70, min_text=5)
    q, k, v, valid, _ = wl.cross_attn_inputs(cfg)
    gq, gk = wl.norm_weights(cfg)
    qn, kn = oracle.qk_rmsnorm(q, gq, EPS, mode), oracle.qk_rmsnorm(k, gk, EPS, mode)
    if split:
        ref = oracle.cross_attn_decoupled(qn, kn, oracle.as_f64(v), split, valid)
    else:
        ref = oracle.cross_attn(qn, kn, oracle.as_f64(v), valid)
    out = B.dit_cross_attn_forward(to_dev(q), to_dev(k), to_dev(v), to_dev(valid), out_dtype=torch.float32,
                                   split=split, norm=dev_norm(mode, gq, gk))
    torch.cuda.synchronize()
    compare(to_f64(out), ref, what="cross normed %s split=%d" % (mode, split))


@pytest.mark.parametrize("mode", ["head", "token"])
@pytest.mark.parametrize("big", [False, True])
def test_cross_attention_normed_chained_query_tiles(mode, big):
    """Normalised q and k on the chained kernel with enough query tiles that a workgroup takes two or three in a row
    (the operands of the NEXT query tile are normalised at the boundary, with the next tile's row factors) and a ragged
    last query tile; four- and eight-wavefront forms; sampled rows of every request against the oracle."""
    import torch

    Lq = 256 * 150 + 37 if big else 128 * 201 + 37
    cfg = dict(wl.CONFIGS["cross_14b"], B=4, Lq=Lq, H=6, n_text=150, n_image=42, min_text=5, seed=91)
    q, k, v, valid, _ = wl.cross_attn_inputs(cfg)
    gq, gk = wl.norm_weights(cfg)
    rows = np.unique(np.concatenate([np.arange(0, 300), np.arange(Lq - 300, Lq),
                                     np.random.default_rng(5).integers(0, Lq, 400)]))
    qn = oracle.qk_rmsnorm(np.ascontiguousarray(q[:, rows]), gq, EPS, mode)
    kn = oracle.qk_rmsnorm(k, gk, EPS, mode)
    ref = oracle.cross_attn(qn, kn, oracle.as_f64(v), valid)
    flags = B.DIT_FLAG_BIG_WORKGROUP if big else B.DIT_FLAG_SMALL_WORKGROUP
    out = B.dit_cross_attn_forward(to_dev(q), to_dev(k), to_dev(v), to_dev(valid), out_dtype=torch.float32,
                                   flags=flags, norm=dev_norm(mode, gq, gk))
    torch.cuda.synchronize()
    got = to_f64(out[:, torch.from_numpy(rows).cuda()])
    compare(got, ref, what="chained cross normed %s, %d wavefronts" % (mode, 8 if big else 4))


@pytest.mark.parametrize("mode", ["head", "token"])
def test_packed_requests_normed(mode):
    import torch

    cfg = wl.CONFIGS["varlen_small"]
    q, k, v = wl.varlen_attn_inputs(cfg)
    gq, gk = wl.norm_weights(cfg)
    ref = oracle.self_attn_packed(oracle.qk_rmsnorm(q, gq, EPS, mode), oracle.qk_rmsnorm(k, gk, EPS, mode),
                                  oracle.as_f64(v), cfg["grids"], cfg["split"])
    out = B.dit_attn_varlen_forward(to_dev(q), to_dev(k), to_dev(v), cfg["grids"], cfg["split"],
                                    out_dtype=torch.float32, norm=dev_norm(mode, gq, gk))
    torch.cuda.synchronize()
    got = to_f64(out)
    n0 = 0
    for i, g in enumerate(cfg["grids"]):
        L = int(np.prod(g))
        compare(got[n0:n0 + L], ref[n0:n0 + L], what="packed normed %s request %d" % (mode, i))
        n0 += L


@pytest.mark.parametrize("mode", ["head", "token"])
def test_full_size_normed_sampled_rows(mode):
    """32,760 tokens x 40 heads x d128 with the normalisation switched on: sampled rows."""
    import torch

    cfg = wl.CONFIGS["dit_14b"]
    q, k, v = wl.self_attn_inputs(cfg, gain=2.0)
    gq, gk = wl.norm_weights(cfg)
    rows = wl.sample_rows(int(np.prod(cfg["grid"])), seed=cfg["seed"], edge=16, n_random=32)
    qn, kn = oracle.qk_rmsnorm(q, gq, EPS, mode), oracle.qk_rmsnorm(k, gk, EPS, mode)
    ref = oracle.self_attn(qn, kn, oracle.as_f64(v), cfg["grid"], cfg["split"], rows=rows)
    out = B.dit_attn_forward(to_dev(q), to_dev(k), to_dev(v), cfg["grid"], cfg["split"],
                             out_dtype=torch.float32, norm=dev_norm(mode, gq, gk))
    torch.cuda.synchronize()
    got = to_f64(out[:, torch.from_numpy(np.asarray(rows, dtype=np.int64)).cuda()])
    compare(got, ref, what="dit_14b normed %s, %d sampled rows" % (mode, len(rows)))
