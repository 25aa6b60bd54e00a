"""dit_cross_attn_forward_static (the entry point that allocates nothing: its workspace is a device array
inside the library) against dit_cross_attn_forward on a caller's workspace, through the C ABI.

Both run the same kernels on the same inputs, so the outputs must agree bit for bit; the static call is
also held to the oracle at the ordinary bar.  Two calls in a row share the one static array, the second
on a smaller problem, so anything a call left behind and a later call wrongly read would show.
Collected last (file name) on purpose.
"""
import numpy as np
import pytest

import oracle
from paper_2601_20655_amd import binding as B
from paper_2601_20655_amd import workloads as wl
from gpu_util import compare, to_dev, to_f64

pytestmark = pytest.mark.gpu


def both_ways(cfg, split=0, flags=0, want_lse=True):
    import torch

    q, k, v, valid, _ = wl.cross_attn_inputs(cfg)
    qd, kd, vd, md = to_dev(q), to_dev(k), to_dev(v), torch.from_numpy(valid).cuda()
    shape = tuple(qd.shape)
    lse_a = lse_b = None
    if want_lse:
        lse_a = torch.full((shape[0], shape[2], shape[1]), 7.0, dtype=torch.float32, device="cuda")
        lse_b = torch.full_like(lse_a, -7.0)
    out_a = torch.full(shape, 3.0, dtype=torch.float32, device="cuda")
    out_b = torch.full(shape, -3.0, dtype=torch.float32, device="cuda")
    B.dit_cross_attn_forward(qd, kd, vd, md, out=out_a, lse=lse_a, flags=flags, split=split)
    B.dit_cross_attn_forward_static(qd, kd, vd, md, out=out_b, lse=lse_b, flags=flags, split=split)
    torch.cuda.synchronize()
    assert torch.equal(out_a, out_b), "static-workspace call differs from the caller-workspace call"
    if want_lse:
        assert torch.equal(lse_a, lse_b)
    ref = oracle.cross_attn_decoupled(q, k, v, split, valid) if split else oracle.cross_attn(q, k, v, valid)
    compare(to_f64(out_b), ref, what="static workspace, B=%d Lq=%d Lk=%d split=%d" % (
        cfg["B"], cfg["Lq"], cfg["n_text"] + cfg["n_image"], split))


def test_static_workspace_two_calls_second_smaller():
    big = dict(B=3, Lq=700, n_text=512, n_image=257, H=4, D=128, dtype="bf16", min_text=16, seed=901)
    small = dict(B=2, Lq=130, n_text=80, n_image=33, H=2, D=128, dtype="bf16", min_text=4, seed=902)
    both_ways(big)
    both_ways(small)
    # the decoupled form and head_dim 64 on the same array, again large then small
    both_ways(dict(big, D=64, seed=903), split=512, want_lse=False)
    both_ways(dict(small, D=64, seed=904), split=80, want_lse=False)
