"""The library only enqueues work on the caller's stream: calls on a side stream and calls captured
into a HIP graph (replayed several times, with eager work in between) give the eager result bit for bit."""
import pytest

from paper_2601_20655_amd import binding as B
from paper_2601_20655_amd import workloads as wl
from gpu_util import to_dev

pytestmark = pytest.mark.gpu


def _inputs():
    cfg = dict(B=1, grid=(3, 10, 26), H=4, D=128, split=(44, 42, 42), dtype="bf16", seed=321)
    q, k, v = (to_dev(a) for a in wl.self_attn_inputs(cfg))
    ccfg = dict(B=2, Lq=780, n_text=200, n_image=57, H=4, D=128, dtype="bf16", min_text=10, seed=322)
    cq, ck, cv, valid, _ = wl.cross_attn_inputs(ccfg)
    return cfg, q, k, v, to_dev(cq), to_dev(ck), to_dev(cv), valid


def test_side_stream_matches_default_stream():
    import torch

    cfg, q, k, v, cq, ck, cv, valid = _inputs()
    vd = torch.from_numpy(valid).cuda()
    ref = B.dit_attn_forward(q, k, v, cfg["grid"], cfg["split"])
    cref = B.dit_cross_attn_forward(cq, ck, cv, vd)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    out = torch.empty_like(ref)
    cout = torch.empty_like(cref)
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        B.dit_attn_forward(q, k, v, cfg["grid"], cfg["split"], out=out, stream=side)
        B.dit_cross_attn_forward(cq, ck, cv, vd, out=cout, stream=side)
    side.synchronize()
    assert torch.equal(out, ref) and torch.equal(cout, cref)


def test_graph_replay_matches_eager():
    import torch

    cfg, q, k, v, cq, ck, cv, valid = _inputs()
    vd = torch.from_numpy(valid).cuda()
    out = torch.empty_like(q)
    cout = torch.empty_like(cq)
    ps = B.self_attn_params(q, k, v, out, cfg["grid"], cfg["split"])
    pc = B.cross_attn_params(cq, ck, cv, cout)
    ws = torch.empty(B.dit_attn_workspace_bytes(ps), dtype=torch.uint8, device="cuda")
    cws = torch.empty(B.dit_cross_attn_workspace_bytes(pc), dtype=torch.uint8, device="cuda")
    ref = B.dit_attn_forward(q, k, v, cfg["grid"], cfg["split"], workspace=ws).clone()
    cref = B.dit_cross_attn_forward(cq, ck, cv, vd, workspace=cws).clone()
    torch.cuda.synchronize()

    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            B.dit_attn_forward(q, k, v, cfg["grid"], cfg["split"], out=out, workspace=ws, stream=side)
            B.dit_cross_attn_forward(cq, ck, cv, vd, out=cout, workspace=cws, stream=side)
    torch.cuda.synchronize()
    for rep in range(4):
        out.fill_(7.0)   # fill kernels, not memsets: eager work between replays
        cout.fill_(7.0)
        ws.fill_(rep)    # the workspace is rebuilt by every replay
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, ref), "self-attention replay %d differs from eager" % rep
        assert torch.equal(cout, cref), "cross-attention replay %d differs from eager" % rep


def test_graph_replay_of_the_other_entry_points_and_flags():
    """Packed requests with token-mode q/k normalisation, the 8-bit score path, a cross-attention call
    on resident tiles and a projection, all captured into one graph and replayed with eager work in
    between."""
    import torch

    vcfg = wl.CONFIGS["varlen_small"]
    vq, vk, vv = (to_dev(a) for a in wl.varlen_attn_inputs(vcfg))
    gq, gk = (to_dev(a) for a in wl.norm_weights(vcfg))
    norm = ("token", 1e-6, gq, gk)
    cfg, q, k, v, cq, ck, cv, valid = _inputs()
    vd = torch.from_numpy(valid).cuda()
    grids = list(vcfg["grids"])

    vout, out8, cout = torch.empty_like(vq), torch.empty_like(q), torch.empty_like(cq)
    big = 64 << 20
    vws, ws8, cws = (torch.empty(big, dtype=torch.uint8, device="cuda") for _ in range(3))
    vref = B.dit_attn_varlen_forward(vq, vk, vv, grids, vcfg["split"], norm=norm, workspace=vws).clone()
    ref8 = B.dit_attn_forward(q, k, v, cfg["grid"], cfg["split"], flags=B.DIT_FLAG_QK_FP8, workspace=ws8).clone()
    cref = B.dit_cross_attn_forward(cq, ck, cv, vd, workspace=cws).clone()  # leaves its tiles in cws
    lx, lw, lb = (to_dev(a) for a in wl.linear_inputs(wl.CONFIGS["proj_small"]))
    lref = B.dit_linear_forward(lx, lw, lb).clone()
    lout = torch.empty_like(lref)
    torch.cuda.synchronize()

    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            B.dit_attn_varlen_forward(vq, vk, vv, grids, vcfg["split"], norm=norm, out=vout, workspace=vws, stream=side)
            B.dit_attn_forward(q, k, v, cfg["grid"], cfg["split"], flags=B.DIT_FLAG_QK_FP8, out=out8, workspace=ws8,
                               stream=side)
            B.dit_cross_attn_forward(cq, ck, cv, None, flags=B.DIT_FLAG_KV_RESIDENT, out=cout, workspace=cws,
                                     stream=side)
            B.dit_linear_forward(lx, lw, lb, out=lout, stream=side)
    torch.cuda.synchronize()
    for rep in range(3):
        for t in (vout, out8, cout, lout):
            t.fill_(-3.0)
        vws.fill_(rep)  # rebuilt by every replay; cws keeps the resident tiles and is left alone
        ws8.fill_(rep)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(vout, vref), "packed requests, replay %d" % rep
        assert torch.equal(out8, ref8), "8-bit scores, replay %d" % rep
        assert torch.equal(cout, cref), "resident cross-attention, replay %d" % rep
        assert torch.equal(lout, lref), "projection, replay %d" % rep
