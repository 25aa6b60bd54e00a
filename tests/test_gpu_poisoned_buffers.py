"""Nothing the library reads may come from memory it has not written in the same call: the
workspace and the output buffers are filled with NaN bit patterns (0xFF bytes) and with zeros
before two otherwise identical calls, and the results must agree bit for bit (every entry point,
the kernel forms that keep state in the workspace: tile images, tile masks and lists, RoPE
tables, per-token normalisation factors)."""
import numpy as np
import pytest

from paper_2601_20655_amd import binding as B
from paper_2601_20655_amd import workloads as wl
from gpu_util import to_dev

pytestmark = pytest.mark.gpu


def twice(call, ws_bytes, out_shape, out_dtype):
    import torch

    results = []
    for fill in (0xFF, 0x00):
        ws = torch.full((ws_bytes + 4096,), fill, dtype=torch.uint8, device="cuda")
        out = torch.full(out_shape, float("nan"), dtype=out_dtype, device="cuda")
        lse = torch.full((int(np.prod(out_shape[:-1])),), float("nan"), dtype=torch.float32, device="cuda")
        call(ws, out, lse)
        torch.cuda.synchronize()
        assert torch.isfinite(out.float()).all()
        # the library stays inside the size it asked for
        assert bool((ws[ws_bytes:] == fill).all())
        results.append((out.clone(), lse.clone()))
    return results


@pytest.mark.parametrize("flags", [0, B.DIT_FLAG_BIG_WORKGROUP, B.DIT_FLAG_SIMPLE_SCHEDULE,
                                   B.DIT_FLAG_MFMA_32X32 | B.DIT_FLAG_BIG_WORKGROUP])
@pytest.mark.parametrize("mode", [None, "token"])
def test_self_attention_ignores_stale_workspace(flags, mode):
    import torch

    cfg = dict(B=2, grid=(3, 7, 19), H=3, D=128, split=(44, 42, 42), dtype="bf16", seed=31)
    q, k, v = (to_dev(a) for a in wl.self_attn_inputs(cfg))
    gq, gk = (to_dev(g) for g in wl.norm_weights(cfg))
    norm = None if mode is None else (mode, 1e-6, gq, gk)
    out0 = torch.empty_like(q)
    need = B.dit_attn_workspace_bytes(B.self_attn_params(q, k, v, out0, cfg["grid"], cfg["split"], flags=flags,
                                                         norm=norm))

    def call(ws, out, lse):
        B.dit_attn_forward(q, k, v, cfg["grid"], cfg["split"], out=out, lse=lse.view(2, 3, -1), flags=flags,
                           workspace=ws[:need], norm=norm)

    (a, la), (b, lb) = twice(call, need, tuple(q.shape), torch.bfloat16)
    assert torch.equal(a.view(torch.int16), b.view(torch.int16)) and torch.equal(la, lb)


@pytest.mark.parametrize("split", [0, 96])
def test_cross_attention_ignores_stale_workspace(split):
    import torch

    cfg = dict(wl.CONFIGS["cross_14b"], B=3, Lq=333, H=2, n_text=96, n_image=70, min_text=5)
    qn, kn, vn, valid, _ = wl.cross_attn_inputs(cfg)
    valid[2] = 0  # one request without any key
    q, k, v, m = to_dev(qn), to_dev(kn), to_dev(vn), to_dev(valid)
    need = B.dit_cross_attn_workspace_bytes(B.cross_attn_params(q, k, v, torch.empty_like(q), split=split))

    def call(ws, out, lse):
        B.dit_cross_attn_forward(q, k, v, m, out=out, lse=None if split else lse.view(3, 2, -1), workspace=ws[:need],
                                 split=split)

    (a, la), (b, lb) = twice(call, need, tuple(q.shape), torch.bfloat16)
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    if not split:
        assert torch.equal(la, lb) and bool(torch.isinf(la.view(3, 2, -1)[2]).all())
    assert bool((a[2] == 0).all())


def test_packed_requests_ignore_stale_workspace():
    import torch

    cfg = wl.CONFIGS["varlen_small"]
    q, k, v = (to_dev(a) for a in wl.varlen_attn_inputs(cfg))
    need = B.dit_attn_varlen_workspace_bytes(B.varlen_attn_params(q, k, v, torch.empty_like(q), cfg["grids"],
                                                                   cfg["split"]))

    def call(ws, out, lse):
        B.dit_attn_varlen_forward(q, k, v, cfg["grids"], cfg["split"], out=out, lse=lse.view(cfg["H"], -1),
                                  workspace=ws[:need])

    (a, la), (b, lb) = twice(call, need, tuple(q.shape), torch.bfloat16)
    assert torch.equal(a.view(torch.int16), b.view(torch.int16)) and torch.equal(la, lb)
