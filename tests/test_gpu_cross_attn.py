"""GPU parity of dit_cross_attn_forward (through the C ABI) against the CPU fp64 oracle."""
import numpy as np
import pytest

import oracle
from paper_2601_20655_amd import binding as B
from paper_2601_20655_amd import workloads as wl
from gpu_util import compare, to_dev, to_f64

pytestmark = pytest.mark.gpu


def run_cross(q, k, v, valid, **kw):
    import torch

    vd = torch.from_numpy(valid).cuda() if valid is not None else None
    res = B.dit_cross_attn_forward(to_dev(q), to_dev(k), to_dev(v), vd, **kw)
    torch.cuda.synchronize()
    return res


SHAPES = {
    "auto": 0,
    "pipe_qb1_4w": B.DIT_FLAG_PIPELINED_SCHEDULE | B.DIT_FLAG_SMALL_WORKGROUP,
    "pipe_qb1_8w": B.DIT_FLAG_PIPELINED_SCHEDULE | B.DIT_FLAG_BIG_WORKGROUP,
    "pipe_qb2_4w": B.DIT_FLAG_PIPELINED_SCHEDULE | B.DIT_FLAG_WIDE_QTILE,
    "chain_4w": B.DIT_FLAG_SMALL_WORKGROUP,
    "chain_8w": B.DIT_FLAG_BIG_WORKGROUP,
    "simple_qb1": B.DIT_FLAG_SIMPLE_SCHEDULE,
    "simple_qb2": B.DIT_FLAG_SIMPLE_SCHEDULE | B.DIT_FLAG_WIDE_QTILE,
}


@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("wide", sorted(SHAPES))
def test_small_cross_with_masks(D, wide):
    import torch

    cfg = dict(B=3, Lq=333, n_text=512, n_image=257, H=2, D=D, dtype="bf16", min_text=16, seed=31 + D)
    q, k, v, valid, text_len = wl.cross_attn_inputs(cfg)
    valid[2, :] = 0
    valid[2, 700] = 1  # a request with a single valid key: output = that value row
    ref, ref_lse = oracle.cross_attn(q, k, v, valid, want_lse=True)
    flags = SHAPES[wide]
    out, lse = run_cross(q, k, v, valid, flags=flags, out_dtype=torch.float32, want_lse=True)
    compare(to_f64(out), ref, what="cross D=%d wide=%s" % (D, wide))
    assert np.max(np.abs(to_f64(lse) - ref_lse)) < 5e-3
    out = run_cross(q, k, v, valid, flags=flags)
    compare(to_f64(out), ref, bf16_out=True, what="cross D=%d wide=%s bf16 out" % (D, wide))
    # no mask at all
    ref2 = oracle.cross_attn(q, k, v, None)
    out2 = run_cross(q, k, v, None, flags=flags, out_dtype=torch.float32)
    compare(to_f64(out2), ref2, what="cross no mask")


def test_fully_masked_request_and_garbage_under_mask():
    import torch

    cfg = dict(B=2, Lq=70, n_text=100, n_image=29, H=2, D=128, dtype="bf16", min_text=5, seed=5)
    q, k, v, valid, _ = wl.cross_attn_inputs(cfg)
    valid[1, :] = 0
    # huge finite garbage under the mask must not leak into request 0
    kb = wl.bf16_bits_to_f32(k).copy(); vb = wl.bf16_bits_to_f32(v).copy()
    kb[0, valid[0] == 0] = 3.0e4; vb[0, valid[0] == 0] = -3.0e4
    k2, v2 = wl.f32_to_bf16_bits(kb), wl.f32_to_bf16_bits(vb)
    ref, ref_lse = oracle.cross_attn(q, k2, v2, valid, want_lse=True)
    assert np.all(np.isneginf(ref_lse[1]))
    for name, flags in sorted(SHAPES.items()):
        out, lse = run_cross(q, k2, v2, valid, out_dtype=torch.float32, want_lse=True, flags=flags)
        o = to_f64(out)
        compare(o[0], ref[0], what="garbage under mask, %s" % name)
        assert np.all(o[1] == 0.0)
        assert np.all(np.isneginf(to_f64(lse)[1]))


def test_full_size_cross_sampled_rows():
    """4 requests x 32,760 queries x 769 keys x 40 heads, default flags; sampled rows of every head."""
    import torch

    cfg = wl.CONFIGS["cross_14b"]
    q, k, v, valid, text_len = wl.cross_attn_inputs(cfg)
    rows = wl.sample_rows(cfg["Lq"], cfg["seed"], edge=64, n_random=128)
    ref = oracle.cross_attn(q, k, v, valid, rows=rows)
    out = run_cross(q, k, v, valid)
    compare(to_f64(out[:, torch.from_numpy(rows).cuda()]), ref, bf16_out=True, what="cross_14b bf16 out")
    del out
    out = run_cross(q, k, v, valid, out_dtype=torch.float32)
    compare(to_f64(out[:, torch.from_numpy(rows).cuda()]), ref, what="cross_14b f32 out")


@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("n_text,n_image", [(200, 57), (128, 64), (7, 300), (512, 257)])
def test_decoupled_cross_attention(D, n_text, n_image):
    """Two softmaxes (text keys, image keys) added: splits on and off tile boundaries, padded text,
    one request whose text is fully masked, one whose image part is fully masked."""
    import torch

    cfg = dict(B=4, Lq=300, n_text=n_text, n_image=n_image, H=2, D=D, dtype="bf16", min_text=1, seed=900 + D + n_text)
    q, k, v, valid, text_len = wl.cross_attn_inputs(cfg)
    valid[2, :n_text] = 0          # request 2: only the image sequence attends
    valid[3, n_text:] = 0          # request 3: only the text sequence attends
    ref = oracle.cross_attn_decoupled(q, k, v, n_text, valid)
    for flags in (0, B.DIT_FLAG_QK_F16 | B.DIT_FLAG_PV_BF16):
        out = run_cross(q, k, v, valid, out_dtype=torch.float32, split=n_text, flags=flags)
        compare(to_f64(out), ref, what="decoupled D=%d split=%d flags=%d" % (D, n_text, flags))
    out = run_cross(q, k, v, valid, split=n_text)
    compare(to_f64(out), ref, bf16_out=True, what="decoupled D=%d split=%d bf16 out" % (D, n_text))
    # no mask at all, and a split at the end (= joint softmax)
    ref2 = oracle.cross_attn_decoupled(q, k, v, n_text, None)
    compare(to_f64(run_cross(q, k, v, None, out_dtype=torch.float32, split=n_text)), ref2, what="decoupled no mask")
    ref3 = oracle.cross_attn(q, k, v, valid)
    compare(to_f64(run_cross(q, k, v, valid, out_dtype=torch.float32, split=n_text + n_image)), ref3,
            what="split at Lk is the joint softmax")


def test_decoupled_rejects_lse():
    import torch

    cfg = dict(B=1, Lq=64, n_text=64, n_image=64, H=1, D=128, dtype="bf16", min_text=1, seed=5)
    q, k, v, valid, _ = wl.cross_attn_inputs(cfg)
    with pytest.raises(B.DitError) as e:
        run_cross(q, k, v, valid, split=64, want_lse=True)
    assert e.value.status == B.DIT_ERR_UNSUPPORTED


def test_full_size_decoupled_cross_sampled_rows():
    """cross_14b shape with the text / image keys as two softmaxes (split at 512)."""
    import torch

    cfg = wl.CONFIGS["cross_14b"]
    q, k, v, valid, text_len = wl.cross_attn_inputs(cfg)
    rows = wl.sample_rows(cfg["Lq"], cfg["seed"], edge=64, n_random=128)
    ref = oracle.cross_attn_decoupled(q, k, v, cfg["n_text"], valid, rows=rows)
    out = run_cross(q, k, v, valid, out_dtype=torch.float32, split=cfg["n_text"])
    compare(to_f64(out[:, torch.from_numpy(rows).cuda()]), ref, what="cross_14b decoupled f32 out")
    del out
    out = run_cross(q, k, v, valid, split=cfg["n_text"])
    compare(to_f64(out[:, torch.from_numpy(rows).cuda()]), ref, bf16_out=True, what="cross_14b decoupled bf16 out")


@pytest.mark.parametrize("split", [0, 300])
@pytest.mark.parametrize("shape", [0, B.DIT_FLAG_PIPELINED_SCHEDULE])
def test_scattered_key_masks_are_compacted(split, shape):
    """Validity scattered over the keys instead of a padded tail: every third key, a request with
    two isolated keys in different tiles, a request with one whole tile valid in the middle, and a
    request with every key valid.  The library packs the valid keys densely into tiles (the order of
    keys does not matter to attention); output and log-sum-exp against the oracle on all rows, and a
    second call on the resident tiles with the mask pointer gone."""
    import torch

    if split and shape:
        pytest.skip("the decoupled form has no pipelined kernel")
    cfg = dict(B=4, Lq=150, n_text=300, n_image=215, H=2, D=128, dtype="bf16", min_text=16, seed=401)
    q, k, v, valid, _ = wl.cross_attn_inputs(cfg)
    Lk = k.shape[1]
    valid[:] = 0
    valid[0, ::3] = 1
    valid[1, 70] = valid[1, 400] = 1
    valid[2, 320:384] = 1
    valid[3, :] = 1
    if split:  # every key group of every request keeps at least one key
        valid[1, 10] = 1
        valid[2, 5] = 1
    ws = torch.empty(64 << 20, dtype=torch.uint8, device="cuda")
    want_lse = split == 0
    res = run_cross(q, k, v, valid, flags=shape, split=split, workspace=ws, out_dtype=torch.float32, want_lse=want_lse)
    if split:
        ref = oracle.cross_attn_decoupled(q, k, v, split, valid)
        compare(to_f64(res), ref, what="scattered masks, decoupled")
    else:
        ref, ref_lse = oracle.cross_attn(q, k, v, valid, want_lse=True)
        out, lse = res
        compare(to_f64(out), ref, what="scattered masks, joint, flags %d" % shape)
        assert np.max(np.abs(to_f64(lse) - ref_lse)) < 5e-3
    q2 = wl.cross_attn_inputs(cfg, seed=402)[0]
    nan = torch.full((cfg["B"], Lk, cfg["H"], cfg["D"]), float("nan"), dtype=torch.bfloat16, device="cuda")
    out2 = B.dit_cross_attn_forward(to_dev(q2), nan, nan, None, flags=shape | B.DIT_FLAG_KV_RESIDENT, split=split,
                                    workspace=ws, out_dtype=torch.float32)
    torch.cuda.synchronize()
    ref2 = oracle.cross_attn_decoupled(q2, k, v, split, valid) if split else oracle.cross_attn(q2, k, v, valid)
    compare(to_f64(out2), ref2, what="scattered masks, resident call")


@pytest.mark.parametrize("D,shape", [(64, "chain_4w"), (128, "chain_4w"), (128, "chain_8w")])
def test_chained_query_tiles_all_rows(D, shape):
    """Enough query tiles that the default kernel's workgroups take two or three in a row (about five
    workgroups per compute unit), with requests of 0, 1, 2 and 3 key tiles -- odd and even numbers of steps,
    so that the wrap-around of the key-tile stream starts the next query tile in either K' buffer -- and a
    ragged last query tile.  Every row of every request against the oracle, output and log-sum-exp."""
    import torch

    # 202 query tiles x 4 requests x 6 heads over 256 compute units: chains of three (the last one shorter);
    # 151 x 4 x 6: chains of two
    Lq = 128 * 201 + 37 if shape == "chain_4w" else 256 * 150 + 37
    H = 6
    cfg = dict(B=4, Lq=Lq, n_text=150, n_image=42, H=H, D=D, dtype="bf16", min_text=5, seed=77 + D)
    q, k, v, valid, _ = wl.cross_attn_inputs(cfg)
    valid[:] = 0
    valid[1, 3:43] = 1                   # 40 keys: one tile
    valid[2, 0:150:2] = 1                # 75 scattered keys + 25 below: two tiles
    valid[2, 150:175] = 1
    valid[3, :] = 1                      # 192 keys: three full tiles
    ref, ref_lse = oracle.cross_attn(q, k, v, valid, want_lse=True)
    out, lse = run_cross(q, k, v, valid, out_dtype=torch.float32, want_lse=True, flags=SHAPES[shape])
    o, l = to_f64(out), to_f64(lse)
    assert np.all(o[0] == 0.0) and np.all(np.isneginf(l[0]))
    for b in (1, 2, 3):
        compare(o[b], ref[b], what="chained, request %d, %s" % (b, shape))
        assert np.allclose(l[b], ref_lse[b], rtol=0, atol=2e-3)


def _mask_from_lengths(kv_len, second_start, Lk):
    valid = np.zeros((kv_len.shape[0], Lk), dtype=np.uint8)
    for b, (l0, l1) in enumerate(kv_len):
        valid[b, :l0] = 1
        valid[b, second_start:second_start + l1] = 1
    return valid


@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("shape", ["auto", "chain_8w", "pipe_qb1_4w", "simple_qb1"])
def test_key_counts_instead_of_mask(D, shape):
    """dit_cross_attn_forward_lengths: two counts per request instead of a byte mask.  Against the oracle on the
    mask the counts stand for, and bit for bit against the mask form of the library (same keys, same order)."""
    import torch

    n_text, n_image = 200, 77
    cfg = dict(B=5, Lq=300, n_text=n_text, n_image=n_image, H=3, D=D, dtype="bf16", min_text=5, seed=31 + D)
    q, k, v, _, _ = wl.cross_attn_inputs(cfg)
    kv_len = np.array([[200, 77], [1, 0], [0, 0], [64, 64], [130, 5]], dtype=np.int32)
    valid = _mask_from_lengths(kv_len, n_text, n_text + n_image)
    ref, ref_lse = oracle.cross_attn(q, k, v, valid, want_lse=True)
    flags = SHAPES[shape]
    dq, dk, dv = to_dev(q), to_dev(k), to_dev(v)
    out, lse = B.dit_cross_attn_forward_lengths(dq, dk, dv, torch.from_numpy(kv_len).cuda(), n_text, flags=flags,
                                                out_dtype=torch.float32, want_lse=True)
    torch.cuda.synchronize()
    o, l = to_f64(out), to_f64(lse)
    for b in range(5):
        if kv_len[b].sum() == 0:
            assert np.all(o[b] == 0.0) and np.all(np.isneginf(l[b]))
        else:
            compare(o[b], ref[b], what="key counts, request %d, %s" % (b, shape))
            assert np.allclose(l[b], ref_lse[b], rtol=0, atol=2e-3)
    out_m = run_cross(q, k, v, valid, flags=flags, out_dtype=torch.float32)
    assert torch.equal(out, out_m)
    # counts outside their range are clamped, never read out of bounds
    wild = torch.tensor([[10 ** 6, 10 ** 6], [-5, 3], [0, 0], [64, 64], [130, 5]], dtype=torch.int32).cuda()
    out_w = B.dit_cross_attn_forward_lengths(dq, dk, dv, wild, n_text, flags=flags, out_dtype=torch.float32)
    torch.cuda.synchronize()
    clamped = _mask_from_lengths(np.array([[200, 77], [0, 3], [0, 0], [64, 64], [130, 5]]), n_text, n_text + n_image)
    compare(to_f64(out_w)[1], oracle.cross_attn(q, k, v, clamped)[1], what="clamped counts")
    assert torch.equal(out_w[0], out[0])


@pytest.mark.parametrize("D", [64, 128])
def test_key_counts_decoupled_and_resident(D):
    """The decoupled form (a softmax per sequence) from counts, then new queries against the tiles that call left."""
    import torch

    n_text, n_image = 150, 70
    cfg = dict(B=3, Lq=200, n_text=n_text, n_image=n_image, H=2, D=D, dtype="bf16", min_text=5, seed=5 + D)
    q, k, v, _, _ = wl.cross_attn_inputs(cfg)
    kv_len = np.array([[150, 70], [33, 0], [0, 65]], dtype=np.int32)
    valid = _mask_from_lengths(kv_len, n_text, n_text + n_image)
    ref = oracle.cross_attn_decoupled(q, k, v, n_text, valid)
    dlen = torch.from_numpy(kv_len).cuda()
    ws = torch.empty(64 << 20, dtype=torch.uint8, device="cuda")
    out = B.dit_cross_attn_forward_lengths(to_dev(q), to_dev(k), to_dev(v), dlen, n_text, split=n_text,
                                           out_dtype=torch.float32, workspace=ws)
    torch.cuda.synchronize()
    compare(to_f64(out), ref, what="decoupled from key counts")
    with pytest.raises(B.DitError):  # the second range of the decoupled form starts at the split
        B.dit_cross_attn_forward_lengths(to_dev(q), to_dev(k), to_dev(v), dlen, n_text - 1, split=n_text, workspace=ws)
    q2 = wl.f32_to_bf16_bits(wl.bf16_bits_to_f32(q)[:, ::-1].copy())
    nan = torch.full_like(to_dev(k), float("nan"))
    out2 = B.dit_cross_attn_forward_lengths(to_dev(q2), nan, nan, None, n_text, split=n_text, workspace=ws,
                                            flags=B.DIT_FLAG_KV_RESIDENT, out_dtype=torch.float32)
    torch.cuda.synchronize()
    compare(to_f64(out2), oracle.cross_attn_decoupled(q2, k, v, n_text, valid), what="resident tiles from key counts")
