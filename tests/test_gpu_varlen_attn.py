"""GPU parity of dit_attn_varlen_forward (several requests with their own latent grids packed
along the token axis) against the CPU fp64 oracle, request by request."""
import numpy as np
import pytest

import oracle
from paper_2601_20655_amd import binding as B
from paper_2601_20655_amd import workloads as wl
from gpu_util import compare, to_dev, to_f64

pytestmark = pytest.mark.gpu

SHAPES = {"auto": 0, "4w": B.DIT_FLAG_SMALL_WORKGROUP, "8w": B.DIT_FLAG_BIG_WORKGROUP,
          "m32_4w": B.DIT_FLAG_MFMA_32X32 | B.DIT_FLAG_SMALL_WORKGROUP,
          "m32_8w": B.DIT_FLAG_MFMA_32X32 | B.DIT_FLAG_BIG_WORKGROUP}


def compare_per_request(got, ref, grids, what, **kw):
    """The parity bar is relative to the output RMS of ONE attention problem; short requests have
    much larger outputs than long ones, so every request is held to the bar on its own rows."""
    n0, worst = 0, 0.0
    for i, g in enumerate(grids):
        L = int(np.prod(g))
        worst = max(worst, compare(got[n0:n0 + L], ref[n0:n0 + L], what="%s request %d" % (what, i), **kw))
        n0 += L
    return worst


def run_varlen(cfg, q, k, v, grids=None, **kw):
    import torch

    res = B.dit_attn_varlen_forward(to_dev(q), to_dev(k), to_dev(v), grids or cfg["grids"], cfg["split"], **kw)
    torch.cuda.synchronize()
    return res


@pytest.mark.parametrize("shape", sorted(SHAPES))
@pytest.mark.parametrize("ops", [0, B.DIT_FLAG_PV_BF16])
def test_small_mixed_grids_all_rows(shape, ops):
    """Six requests from 1 to 1,024 tokens (ragged tails, one single-token request, one that fills
    its tiles exactly), 4 heads, d128: every row against the oracle, bf16 and fp32 outputs, plus
    the per-row log-sum-exp."""
    import torch

    cfg = wl.CONFIGS["varlen_small"]
    q, k, v = wl.varlen_attn_inputs(cfg)
    ref, ref_lse = oracle.self_attn_packed(q, k, v, cfg["grids"], cfg["split"], want_lse=True)
    out, lse = run_varlen(cfg, q, k, v, flags=SHAPES[shape] | ops, out_dtype=torch.float32, want_lse=True)
    compare_per_request(to_f64(out), ref, cfg["grids"], "varlen_small %s f32 out" % shape)
    assert np.max(np.abs(to_f64(lse) - ref_lse)) < 5e-3
    out = run_varlen(cfg, q, k, v, flags=SHAPES[shape] | ops)
    compare_per_request(to_f64(out), ref, cfg["grids"], "varlen_small %s bf16 out" % shape, bf16_out=True)


def test_d64_fp32_inputs_with_origin_and_scale():
    import torch

    cfg = wl.CONFIGS["varlen_small_d64"]
    q, k, v = wl.varlen_attn_inputs(cfg)
    ref = oracle.self_attn_packed(q, k, v, cfg["grids"], cfg["split"], origin=(3, 1, 2), base=500.0, scale=0.2)
    out = run_varlen(cfg, q, k, v, origin=(3, 1, 2), rope_base=500.0, scale=0.2, out_dtype=torch.float32)
    compare_per_request(to_f64(out), ref, cfg["grids"], "varlen d64 f32")


def test_one_request_equals_plain_entry_point_bitwise():
    """A batch of one request runs the same kernel body on the same tiles as dit_attn_forward."""
    cfg = wl.CONFIGS["mid"]
    q, k, v = wl.self_attn_inputs(cfg)
    qd, kd, vd = to_dev(q), to_dev(k), to_dev(v)
    import torch

    plain = B.dit_attn_forward(qd, kd, vd, cfg["grid"], cfg["split"])
    packed = B.dit_attn_varlen_forward(qd[0], kd[0], vd[0], [cfg["grid"]], cfg["split"])
    torch.cuda.synchronize()
    assert torch.equal(plain[0].view(torch.int16), packed.view(torch.int16))


def test_request_order_and_neighbours_do_not_matter():
    """Each request's output depends on its own tokens only: permuting the requests, or replacing
    the neighbours by huge values, leaves its rows bit-identical."""
    import torch

    cfg = wl.CONFIGS["varlen_small"]
    grids = list(cfg["grids"])
    q, k, v = wl.varlen_attn_inputs(cfg)
    base = run_varlen(cfg, q, k, v).view(torch.int16).cpu().numpy()
    Ls = [int(np.prod(g)) for g in grids]
    starts = np.concatenate([[0], np.cumsum(Ls)])
    perm = [3, 0, 5, 1, 4, 2]
    idx = np.concatenate([np.arange(starts[i], starts[i + 1]) for i in perm])
    outp = run_varlen(cfg, q[idx], k[idx], v[idx], grids=[grids[i] for i in perm]).view(torch.int16).cpu().numpy()
    np.testing.assert_array_equal(outp, base[idx])
    # request 1 with loud neighbours
    q2, k2, v2 = q.copy(), k.copy(), v.copy()
    loud = wl.f32_to_bf16_bits(np.full((1,), 3.0e4, dtype=np.float32))[0]
    keep = np.zeros(len(q), dtype=bool)
    keep[starts[1]:starts[2]] = True
    for a in (q2, k2, v2):
        a[~keep] = loud
    out2 = run_varlen(cfg, q2, k2, v2).view(torch.int16).cpu().numpy()
    np.testing.assert_array_equal(out2[keep], base[keep])


def test_full_size_mixed_batch_sampled_rows():
    """Seven requests (720p and 480p clips of 81, 49 and 33 frames, one still image; 238,920 tokens)
    at 40 heads, d128, in the launch shape the timing runs use: sampled rows of every request
    against the oracle."""
    import torch

    cfg = wl.CONFIGS["varlen_14b"]
    q, k, v = wl.varlen_attn_inputs(cfg)
    out = run_varlen(cfg, q, k, v, out_dtype=torch.float32)
    n0 = 0
    worst = 0.0
    for i, g in enumerate(cfg["grids"]):
        L = int(np.prod(g))
        rows = wl.sample_rows(L, seed=cfg["seed"] + i, edge=4, n_random=8)
        sl = slice(n0, n0 + L)
        ref = oracle.self_attn(q[None, sl], k[None, sl], v[None, sl], g, cfg["split"], rows=rows)[0]
        got = to_f64(out[torch.from_numpy(n0 + np.asarray(rows, dtype=np.int64)).cuda()])
        worst = max(worst, compare(got, ref, what="varlen_14b request %d %s" % (i, (g,))))
        n0 += L
    print("varlen_14b worst max|err|/RMS = %.3e" % worst)


def test_sixty_four_small_requests_odd_head_count():
    """The request table at its limit (64 entries) with 5 heads, so that the per-XCD queues get
    unequal numbers of (request, head) pairs and some workgroups find their queue empty; grids
    from 1 to 150 tokens, d64, fp32 inputs."""
    import torch

    grids = [(1 + k % 3, 1 + k % 5, 1 + (7 * k) % 10) for k in range(64)]
    cfg = dict(kind="varlen", grids=grids, H=5, D=64, split=(22, 20, 22), dtype="f32", seed=777)
    q, k, v = wl.varlen_attn_inputs(cfg)
    ref = oracle.self_attn_packed(q, k, v, grids, cfg["split"])
    for flags in sorted(SHAPES.values()):
        out = run_varlen(cfg, q, k, v, flags=flags, out_dtype=torch.float32)
        compare_per_request(to_f64(out), ref, grids, "64 requests flags=%d" % flags)
