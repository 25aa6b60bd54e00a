"""GPU parity of calls that reuse the K'/V^T tile images a previous call left in the workspace
(DIT_FLAG_KV_RESIDENT): new queries, a new scale, k and v replaced by NaN-filled buffers that must
not be read; every result against the CPU fp64 oracle."""
import numpy as np
import pytest

import oracle
from paper_2601_20655_amd import binding as B
from paper_2601_20655_amd import workloads as wl
from gpu_util import compare, to_dev, to_f64

pytestmark = pytest.mark.gpu

EPS = 1e-6
RES = B.DIT_FLAG_KV_RESIDENT


def poisoned_like(t):
    import torch

    return torch.full_like(t, float("nan"))


def workspace(nbytes=96 << 20):
    import torch

    return torch.empty(nbytes, dtype=torch.uint8, device="cuda")


@pytest.mark.parametrize("shape", [0, B.DIT_FLAG_SIMPLE_SCHEDULE, B.DIT_FLAG_BIG_WORKGROUP, B.DIT_FLAG_MFMA_32X32])
@pytest.mark.parametrize("mode", [None, "token"])
def test_self_attention_second_query_set(shape, mode):
    """6,240 tokens x 4 heads: the first call packs K, V; the second one runs other queries with
    another scale against the resident tiles while k and v point at NaNs."""
    import torch

    cfg = wl.CONFIGS["mid"]
    q1, k, v = wl.self_attn_inputs(cfg)
    q2, _, _ = wl.self_attn_inputs(cfg, seed=cfg["seed"] + 101)
    gq, gk = wl.norm_weights(cfg)
    gq2 = np.ascontiguousarray(gq[::-1])  # the query weights may change, the key weights are baked in
    ws = workspace()
    kd, vd = to_dev(k), to_dev(v)

    def norm(g):
        return None if mode is None else (mode, EPS, to_dev(g), to_dev(gk))

    out1 = B.dit_attn_forward(to_dev(q1), kd, vd, cfg["grid"], cfg["split"], flags=shape, workspace=ws,
                              out_dtype=torch.float32, norm=norm(gq))
    out2 = B.dit_attn_forward(to_dev(q2), poisoned_like(kd), poisoned_like(vd), cfg["grid"], cfg["split"],
                              flags=shape | RES, workspace=ws, out_dtype=torch.float32, scale=0.11,
                              norm=norm(gq2))
    torch.cuda.synchronize()
    if mode is None:
        ref1 = oracle.self_attn(q1, k, v, cfg["grid"], cfg["split"])
        ref2 = oracle.self_attn(q2, k, v, cfg["grid"], cfg["split"], scale=0.11)
    else:
        ref1 = oracle.self_attn_normed(q1, k, v, cfg["grid"], cfg["split"], gq, gk, EPS, mode)
        ref2 = oracle.self_attn_normed(q2, k, v, cfg["grid"], cfg["split"], gq2, gk, EPS, mode, scale=0.11)
    compare(to_f64(out1), ref1, what="packing call")
    compare(to_f64(out2), ref2, what="resident call")


def test_self_attention_null_key_pointers_through_the_c_abi():
    """k = v = NULL are accepted with the flag and refused without it."""
    import ctypes
    import torch

    cfg = wl.CONFIGS["tiny"]
    q, k, v = wl.self_attn_inputs(cfg)
    qd, kd, vd = to_dev(q), to_dev(k), to_dev(v)
    out = torch.empty_like(qd, dtype=torch.float32)
    ws = workspace(8 << 20)
    first = B.dit_attn_forward(qd, kd, vd, cfg["grid"], cfg["split"], workspace=ws, out_dtype=torch.float32)
    p = B.self_attn_params(qd, kd, vd, out, cfg["grid"], cfg["split"], flags=RES)
    stream = B._stream_ptr(None)
    st = B.lib().dit_attn_forward(qd.data_ptr(), None, None, out.data_ptr(), None, ctypes.byref(p), ws.data_ptr(),
                                  ws.numel(), stream)
    assert st == B.DIT_OK
    torch.cuda.synchronize()
    assert torch.equal(out, first)
    p.flags = 0
    st = B.lib().dit_attn_forward(qd.data_ptr(), None, None, out.data_ptr(), None, ctypes.byref(p), ws.data_ptr(),
                                  ws.numel(), stream)
    assert st == B.DIT_ERR_INVALID_ARG


@pytest.mark.parametrize("split", [0, 512])
@pytest.mark.parametrize("shape", [0, B.DIT_FLAG_PIPELINED_SCHEDULE])
def test_cross_attention_over_denoising_steps(split, shape):
    """The conditioning keys and values of cross-attention stay the same from step to step: three
    calls with fresh queries, the last two on the resident tiles with NaN k, v and no mask pointer."""
    import torch

    if split and shape:
        pytest.skip("the decoupled form has no pipelined kernel")
    cfg = dict(B=3, Lq=333, n_text=512, n_image=257, H=2, D=128, dtype="bf16", min_text=16, seed=77)
    q, k, v, valid, _ = wl.cross_attn_inputs(cfg)
    valid[2, :] = 0
    valid[2, 700] = 1
    kd, vd, md = to_dev(k), to_dev(v), to_dev(valid)
    ws = workspace()
    for step in range(3):
        qs = wl.cross_attn_inputs(cfg, seed=cfg["seed"] + step)[0]
        if step == 0:
            out = B.dit_cross_attn_forward(to_dev(qs), kd, vd, md, flags=shape, split=split, workspace=ws,
                                           out_dtype=torch.float32)
        else:
            out = B.dit_cross_attn_forward(to_dev(qs), poisoned_like(kd), poisoned_like(vd), None,
                                           flags=shape | RES, split=split, workspace=ws, out_dtype=torch.float32)
        torch.cuda.synchronize()
        if split:
            ref = oracle.cross_attn_decoupled(qs, k, v, split, valid)
        else:
            ref = oracle.cross_attn(qs, k, v, valid)
        compare(to_f64(out), ref, what="cross step %d split=%d" % (step, split))


def test_packed_requests_second_query_set():
    import torch

    cfg = wl.CONFIGS["varlen_small"]
    q1, k, v = wl.varlen_attn_inputs(cfg)
    q2 = wl.varlen_attn_inputs(cfg, seed=cfg["seed"] + 5)[0]
    kd, vd = to_dev(k), to_dev(v)
    ws = workspace()
    B.dit_attn_varlen_forward(to_dev(q1), kd, vd, cfg["grids"], cfg["split"], workspace=ws)
    out = B.dit_attn_varlen_forward(to_dev(q2), poisoned_like(kd), poisoned_like(vd), cfg["grids"], cfg["split"],
                                    workspace=ws, flags=RES, out_dtype=torch.float32)
    torch.cuda.synchronize()
    ref = oracle.self_attn_packed(q2, k, v, cfg["grids"], cfg["split"])
    n0 = 0
    for g in cfg["grids"]:
        L = int(np.prod(g))
        compare(to_f64(out)[n0:n0 + L], ref[n0:n0 + L], what="request of %d tokens" % L)
        n0 += L
