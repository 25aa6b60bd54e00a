"""GPU parity of the fused q/k/v projection (dit_qkv_proj_forward) followed by self-attention on the tile images
it leaves in the workspace (dit_attn_forward with DIT_FLAG_KV_RESIDENT, k = v = None).

What is compared, all against the CPU fp64 oracle: y = oracle.linear(x, w, bias) in float64, rounded to bf16 as the
projection delivers its rows; its q columns against q_out; and oracle.self_attn on those rounded q, k, v columns
against the attention output, to the ordinary 16-bit bar.  A second check compares with the library's own separate
route (dit_linear_forward with bf16 output, then dit_attn_forward on the q, k, v columns of that output): the fused
form passes k and v through bf16 exactly as those rows would, so the two results must be equal bit for bit."""
import numpy as np
import pytest

import oracle
from paper_2601_20655_amd import binding as B
from paper_2601_20655_amd import workloads as wl
from gpu_util import TOL, compare, to_dev, to_f64

pytestmark = pytest.mark.gpu

D = 128
SPLIT = (44, 42, 42)


def inputs(L, H, K, seed):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((L, K)).astype(np.float32)
    w = (rng.standard_normal((3 * H * D, K)) / np.sqrt(K)).astype(np.float32)
    b = (0.1 * rng.standard_normal(3 * H * D)).astype(np.float32)
    return tuple(wl.f32_to_bf16_bits(a) for a in (x, w, b))


@pytest.mark.parametrize("grid,H,K", [((3, 10, 26), 2, 256), ((2, 9, 25), 4, 192), ((1, 8, 8), 2, 64),
                                      ((5, 12, 23), 6, 128)])
@pytest.mark.parametrize("flags", [0, B.DIT_FLAG_QK_BF16 | B.DIT_FLAG_PV_BF16])
@pytest.mark.parametrize("with_bias", [True, False])
def test_fused_projection_then_attention(grid, H, K, flags, with_bias):
    import torch

    L = grid[0] * grid[1] * grid[2]
    xb, wb, bb = inputs(L, H, K, seed=L + H + K)
    y = oracle.linear(xb, wb, bb if with_bias else None)                         # [L, 3 H D] float64
    HD = H * D
    yb = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(y.astype(np.float32)))  # the rows as a bf16 projection delivers them
    q_ref, k_ref, v_ref = yb[:, :HD], yb[:, HD:2 * HD], yb[:, 2 * HD:]
    shape = (1, L, H, D)
    ref = oracle.self_attn(q_ref.reshape(shape), k_ref.reshape(shape), v_ref.reshape(shape), grid, SPLIT)

    x, w = to_dev(xb), to_dev(wb)
    bias = to_dev(bb) if with_bias else None
    q_out, ws = B.dit_qkv_proj_forward(x, w, bias, grid, SPLIT, H, flags=flags)
    torch.cuda.synchronize()
    # q rows: the projection's own bar (fp32 accumulation of K terms, half a bf16 unit for the store)
    compare(to_f64(q_out).reshape(L, HD), y[:, :HD], bf16_out=True, tol=2.0 ** -22 * K ** 0.5, what="q rows")
    out = B.dit_attn_forward(q_out, None, None, grid, SPLIT, flags=flags | B.DIT_FLAG_KV_RESIDENT, workspace=ws,
                             out_dtype=torch.float32)
    torch.cuda.synchronize()
    bf16_ops = bool(flags & B.DIT_FLAG_QK_BF16)
    compare(to_f64(out), ref, tol=2 * TOL if bf16_ops else TOL, what="fused projection + attention, flags %d" % flags)

    # the separate route: the same rows through memory, the same kernels behind them
    yd = B.dit_linear_forward(x, w, bias)
    yq, yk, yv = (yd[:, i * HD:(i + 1) * HD].view(1, L, H, D) for i in range(3))
    assert torch.equal(yq, q_out)
    out2 = B.dit_attn_forward(yq, yk, yv, grid, SPLIT, flags=flags, out_dtype=torch.float32)
    torch.cuda.synchronize()
    assert torch.equal(out, out2), "fused and separate routes differ: max %.3e" % float((out - out2).abs().max())


@pytest.mark.parametrize("grid,H,K", [((3, 10, 26), 2, 256), ((2, 9, 25), 4, 128)])
@pytest.mark.parametrize("with_gamma", [True, False])
@pytest.mark.parametrize("mode", ["head", "token"])
def test_fused_projection_with_norm(grid, H, K, with_gamma, mode):
    """RMS normalisation of q and k.  Per head: k in the projection's epilogue.  Per token: the epilogue applies the
    weights and leaves each head's sum of squares, a second pass over the K' images applies the token's factor.
    q in the attention kernel either way."""
    import torch

    L = grid[0] * grid[1] * grid[2]
    xb, wb, bb = inputs(L, H, K, seed=7 * L + H)
    rng = np.random.default_rng(L)
    gq = (1.0 + 0.3 * rng.standard_normal(H * D)).astype(np.float32) if with_gamma else None
    gk = (1.0 + 0.3 * rng.standard_normal(H * D)).astype(np.float32) if with_gamma else None
    eps = 1e-6
    y = oracle.linear(xb, wb, bb)
    HD = H * D
    shape = (1, L, H, D)
    yb = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(y.astype(np.float32)))
    q_ref, k_ref, v_ref = (yb[:, i * HD:(i + 1) * HD].reshape(shape) for i in range(3))
    ref = oracle.self_attn_normed(q_ref, k_ref, v_ref, grid, SPLIT,
                                  q_gamma=None if gq is None else gq.reshape(H, D),
                                  k_gamma=None if gk is None else gk.reshape(H, D), eps=eps, mode=mode)
    norm = (mode, eps, None if gq is None else torch.from_numpy(gq).cuda(),
            None if gk is None else torch.from_numpy(gk).cuda())
    q_out, ws = B.dit_qkv_proj_forward(to_dev(xb), to_dev(wb), to_dev(bb), grid, SPLIT, H, norm=norm)
    out = B.dit_attn_forward(q_out, None, None, grid, SPLIT, flags=B.DIT_FLAG_KV_RESIDENT, workspace=ws,
                             out_dtype=torch.float32, norm=norm)
    torch.cuda.synchronize()
    compare(to_f64(out), ref, what="fused projection with %s normalisation" % mode)
    # the separate route with the same normalisation: the same to rounding (the sums are taken in another order,
    # and the per-token form rounds K' twice)
    yd = B.dit_linear_forward(to_dev(xb), to_dev(wb), to_dev(bb))
    yq, yk, yv = (yd[:, i * HD:(i + 1) * HD].view(1, L, H, D) for i in range(3))
    out2 = B.dit_attn_forward(yq, yk, yv, grid, SPLIT, out_dtype=torch.float32, norm=norm)
    torch.cuda.synchronize()
    rms = float(np.sqrt(np.mean(ref * ref)))
    diff = float((out - out2).abs().max()) / rms
    print("fused vs separate route, %s normalisation: max diff %.2e x RMS" % (mode, diff))
    assert diff <= (1e-2 if mode == "token" else 3e-3)


def test_fused_projection_rejections():
    import torch

    grid, H, K = (1, 8, 8), 2, 64
    xb, wb, bb = inputs(64, H, K, seed=3)
    x, w, b = to_dev(xb), to_dev(wb), to_dev(bb)
    for bad in (B.DIT_FLAG_KV_RESIDENT, B.DIT_FLAG_MFMA_32X32, B.DIT_FLAG_SIMPLE_SCHEDULE, B.DIT_FLAG_QK_FP8):
        with pytest.raises(B.DitError):
            B.dit_qkv_proj_forward(x, w, b, grid, SPLIT, H, flags=bad)
    with pytest.raises(ValueError):
        B.dit_qkv_proj_forward(x, w[:-8], b, grid, SPLIT, H)
    with pytest.raises(ValueError):
        B.dit_qkv_proj_forward(x, w, b, (1, 8, 9), SPLIT, H)
    xb3, wb3, bb3 = inputs(64, 3, K, seed=4)   # an odd number of heads: a 256-feature tile would straddle q and k
    with pytest.raises(B.DitError):
        B.dit_qkv_proj_forward(to_dev(xb3), to_dev(wb3), to_dev(bb3), grid, SPLIT, 3)
    torch.cuda.synchronize()
