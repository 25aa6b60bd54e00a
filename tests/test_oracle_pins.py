"""Pins for the CPU fp64 oracle: facts fixed by mathematics, not by the oracle itself.

Each test would fail for a plausible mistake somewhere in oracle/dit_oracle.c (a dropped
term, wrong sign, wrong index, transposed operand, wrong section order, mask leak).
The brute-force comparator below is an independent formulation: positions by nested
loops, rotation by complex multiplication, scores as Re<zq, conj zk>, softmax by an
explicit normalised-exponential loop in Python floats / numpy longdouble.
"""
import cmath
import itertools
import json
import math
import os
import sys

import numpy as np
import pytest

import oracle

SPLITS = {4: (2, 2, 0), 6: (2, 2, 2), 8: (4, 2, 2), 64: (22, 20, 22)}


def brute_self_attn(q, k, v, grid, split, origin=(0, 0, 0), base=10000.0, scale=None):
    """q, k, v: float arrays [L, D] of ONE head. Returns out [L, D], lse [L], probs [L, L]."""
    L, D = q.shape
    scale = 1.0 / math.sqrt(D) if scale is None else scale
    pos = [(origin[0] + t, origin[1] + h, origin[2] + w)
           for t in range(grid[0]) for h in range(grid[1]) for w in range(grid[2])]
    assert len(pos) == L

    def to_complex(x, p):
        z, o = [], 0
        for a in range(3):
            for i in range(split[a] // 2):
                w = base ** (-2.0 * i / split[a])
                z.append(complex(x[o + 2 * i], x[o + 2 * i + 1]) * cmath.exp(1j * p[a] * w))
            o += split[a]
        return z

    zq = [to_complex(q[n], pos[n]) for n in range(L)]
    zk = [to_complex(k[n], pos[n]) for n in range(L)]
    out = np.zeros((L, D))
    lse = np.zeros(L)
    probs = np.zeros((L, L))
    for n in range(L):
        s = [scale * sum((a * b.conjugate()).real for a, b in zip(zq[n], zk[m])) for m in range(L)]
        mx = max(s)
        e = [math.exp(x - mx) for x in s]
        z = math.fsum(e)
        for m in range(L):
            probs[n, m] = e[m] / z
            out[n] += (e[m] / z) * v[m]
        lse[n] = mx + math.log(z)
    return out, lse, probs


@pytest.mark.parametrize("grid,D", [((1, 1, 1), 4), ((1, 1, 2), 6), ((2, 2, 2), 8), ((2, 3, 4), 8),
                                    ((2, 3, 4), 64), ((3, 2, 2), 6)])
def test_p1_brute_force_tiny_grids(grid, D, rng):
    L, H = int(np.prod(grid)), 2
    q, k, v = (rng.standard_normal((1, L, H, D)) for _ in range(3))
    split = SPLITS[D]
    out, lse = oracle.self_attn(q, k, v, grid, split, want_lse=True)
    for h in range(H):
        bo, bl, _ = brute_self_attn(q[0, :, h], k[0, :, h], v[0, :, h], grid, split)
        np.testing.assert_allclose(out[0, :, h], bo, rtol=0, atol=1e-12)
        np.testing.assert_allclose(lse[0, h], bl, rtol=0, atol=1e-12)


def test_p1_brute_force_origin_scale_base(rng):
    grid, D, split = (2, 2, 3), 8, (2, 4, 2)
    L = 12
    q, k, v = (rng.standard_normal((1, L, 1, D)) for _ in range(3))
    out = oracle.self_attn(q, k, v, grid, split, origin=(3, -2, 5), base=100.0, scale=0.37)
    bo, _, _ = brute_self_attn(q[0, :, 0], k[0, :, 0], v[0, :, 0], grid, split, origin=(3, -2, 5),
                               base=100.0, scale=0.37)
    np.testing.assert_allclose(out[0, :, 0], bo, rtol=0, atol=1e-12)


def test_closed_form_two_tokens():
    """L=2, D=2, one axis: scores are 1/sqrt(2) * [cos(0), cos(1 rad)] for row 0 by hand."""
    q = np.zeros((1, 2, 1, 2)); k = np.zeros((1, 2, 1, 2)); v = np.zeros((1, 2, 1, 2))
    q[0, :, 0] = [[1.0, 0.0], [0.0, 2.0]]
    k[0, :, 0] = [[1.0, 0.0], [1.0, 0.0]]
    v[0, :, 0] = [[1.0, 10.0], [3.0, -10.0]]
    out, lse = oracle.self_attn(q, k, v, (2, 1, 1), (2, 0, 0), want_lse=True)
    sc = 1.0 / math.sqrt(2.0)
    # row 0: q at angle 0; key 0 at angle 0, key 1 rotated by +1 rad -> dot = cos(1)
    s0 = np.array([sc * 1.0, sc * math.cos(1.0)])
    # row 1: q = 2j rotated by +1 rad; key0 = 1 -> Re(2j e^{j} * 1) = -2 sin 1; key1 = e^{j} -> Re(2j) = 0
    s1 = np.array([sc * (-2.0 * math.sin(1.0)), 0.0])
    for n, s in enumerate((s0, s1)):
        p = np.exp(s) / np.exp(s).sum()
        np.testing.assert_allclose(out[0, n, 0], p[0] * v[0, 0, 0] + p[1] * v[0, 1, 0], atol=1e-14)
        assert abs(lse[0, 0, n] - math.log(np.exp(s).sum())) < 1e-14


def test_p2_softmax_rows_sum_to_one(rng):
    grid, D = (3, 4, 5), 8
    L = 60
    q, k, v = (rng.standard_normal((2, L, 3, D)) * 3 for _ in range(3))
    _, probs = oracle.self_attn(q, k, v, grid, SPLITS[8], probs_of=(1, 2))
    assert probs.shape == (L, L)
    assert np.all(probs >= 0)
    assert np.max(np.abs(probs.sum(axis=1) - 1.0)) < 1e-14
    qc, kc, vc = rng.standard_normal((2, 7, 2, 8)), rng.standard_normal((2, 9, 2, 8)), rng.standard_normal((2, 9, 2, 8))
    valid = np.array([[1, 0, 1, 1, 0, 0, 1, 1, 1], [0, 0, 0, 0, 1, 0, 0, 0, 0]], dtype=np.uint8)
    _, pc = oracle.cross_attn(qc, kc, vc, valid, probs_of=(0, 1))
    assert np.max(np.abs(pc.sum(axis=1) - 1.0)) < 1e-14
    assert np.all(pc[:, valid[0] == 0] == 0.0)


def test_p3_constant_v(rng):
    grid, D = (2, 3, 4), 8
    L = 24
    q, k = (rng.standard_normal((1, L, 2, D)) * 2 for _ in range(2))
    c = rng.standard_normal(D)
    v = np.broadcast_to(c, (1, L, 2, D)).copy()
    out = oracle.self_attn(q, k, v, grid, SPLITS[8])
    np.testing.assert_allclose(out, np.broadcast_to(c, out.shape), atol=1e-14)
    valid = (rng.random((1, L)) < 0.5).astype(np.uint8)
    valid[0, 3] = 1
    outc = oracle.cross_attn(q, k, v, valid)
    np.testing.assert_allclose(outc, np.broadcast_to(c, outc.shape), atol=1e-14)


def test_p4_rope_shift_invariance(rng):
    grid, D = (3, 4, 5), 64
    L = 60
    q, k, v = (rng.standard_normal((1, L, 2, D)) for _ in range(3))
    a = oracle.self_attn(q, k, v, grid, SPLITS[64], origin=(0, 0, 0))
    b = oracle.self_attn(q, k, v, grid, SPLITS[64], origin=(7, -3, 11))
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-10)
    # but not invariant to a shift of the keys alone (positions matter): shift q/k differently
    pos0 = oracle.token_positions(grid)
    kr0 = oracle.rope3d(k[0, :, 0], pos0, SPLITS[64])
    kr1 = oracle.rope3d(k[0, :, 0], pos0 + np.array([1, 0, 0]), SPLITS[64])
    assert np.max(np.abs(kr0 - kr1)) > 1e-3


def test_p5_single_key(rng):
    q, k, v = (rng.standard_normal((1, 1, 3, 8)) for _ in range(3))
    out, lse = oracle.self_attn(q, k, v, (1, 1, 1), SPLITS[8], want_lse=True)
    np.testing.assert_allclose(out, v, atol=0)
    # lse = the single score; position 0 means no rotation
    s = (q * k).sum(-1)[0, 0] / math.sqrt(8)
    np.testing.assert_allclose(lse[0, :, 0], s, atol=1e-14)


def test_p6_zero_query_gives_mean_of_valid_values(rng):
    grid, D = (2, 2, 5), 8
    L = 20
    k, v = (rng.standard_normal((1, L, 2, D)) for _ in range(2))
    q = np.zeros_like(k)
    out, lse = oracle.self_attn(q, k, v, grid, SPLITS[8], want_lse=True)
    np.testing.assert_allclose(out, np.broadcast_to(v.mean(axis=1, keepdims=True), out.shape), atol=1e-14)
    np.testing.assert_allclose(lse, math.log(L), atol=1e-14)
    valid = np.zeros((1, L), dtype=np.uint8)
    valid[0, [1, 4, 5, 17]] = 1
    outc, lsec = oracle.cross_attn(q, k, v, valid, want_lse=True)
    want = v[:, [1, 4, 5, 17]].mean(axis=1, keepdims=True)
    np.testing.assert_allclose(outc, np.broadcast_to(want, outc.shape), atol=1e-14)
    np.testing.assert_allclose(lsec, math.log(4), atol=1e-14)


def test_p7_dominant_key(rng):
    Lq, Lk, D = 5, 11, 8
    q = rng.standard_normal((1, Lq, 1, D))
    k = rng.standard_normal((1, Lk, 1, D)) * 0.01
    v = rng.standard_normal((1, Lk, 1, D))
    for n in range(Lq):
        m = (3 * n + 1) % Lk
        kk = k.copy()
        kk[0, m, 0] = 200.0 * q[0, n, 0]  # aligned with +q: must win (a sign error would pick the opposite)
        out = oracle.cross_attn(q, kk, v, rows=[n])
        np.testing.assert_allclose(out[0, 0, 0], v[0, m, 0], atol=1e-9)
        kk[0, m, 0] = -200.0 * q[0, n, 0]
        out = oracle.cross_attn(q, kk, v, rows=[n])
        assert np.max(np.abs(out[0, 0, 0] - v[0, m, 0])) > 1e-3


def test_p8_rope_isometry_and_identity(rng):
    D, split = 64, SPLITS[64]
    x = rng.standard_normal((50, D))
    pos = rng.integers(-40, 90, size=(50, 3))
    y = oracle.rope3d(x, pos, split)
    np.testing.assert_allclose(np.linalg.norm(y, axis=1), np.linalg.norm(x, axis=1), rtol=1e-13)
    # every pair keeps its own norm (rotation acts pairwise on (2i, 2i+1))
    np.testing.assert_allclose(np.hypot(y[:, 0::2], y[:, 1::2]), np.hypot(x[:, 0::2], x[:, 1::2]), rtol=1e-12)
    z = oracle.rope3d(x, np.zeros((50, 3), dtype=np.int64), split)
    assert np.array_equal(z, x)
    # first pair of every section has omega = 1: rotating by position p is a rotation by p radians
    p = np.array([[2, 0, 0]])
    e = np.zeros((1, D)); e[0, 0] = 1.0
    r = oracle.rope3d(e, p, split)
    np.testing.assert_allclose(r[0, :2], [math.cos(2.0), math.sin(2.0)], atol=1e-15)
    e = np.zeros((1, D)); e[0, 22] = 1.0  # first channel of the h section for split 22/20/22
    r = oracle.rope3d(e, np.array([[5, 3, 9]]), split)
    np.testing.assert_allclose(r[0, 22:24], [math.cos(3.0), math.sin(3.0)], atol=1e-15)
    e = np.zeros((1, D)); e[0, 43] = 1.0  # second channel of the first w pair: j * e^{j 9}
    r = oracle.rope3d(e, np.array([[5, 3, 9]]), split)
    np.testing.assert_allclose(r[0, 42:44], [-math.sin(9.0), math.cos(9.0)], atol=1e-15)
    # last pair of the t section: omega = base^(-2*10/22)
    e = np.zeros((1, D)); e[0, 20] = 1.0
    r = oracle.rope3d(e, np.array([[4, 0, 0]]), split)
    phi = 4.0 * 10000.0 ** (-20.0 / 22.0)
    np.testing.assert_allclose(r[0, 20:22], [math.cos(phi), math.sin(phi)], atol=1e-15)


def test_p9_reduces_to_1d_rope_closed_form(rng):
    """Split (D,0,0) on an (L,1,1) grid: score(n,m) = scale * Re sum_i q_i conj(k_i) e^{j (n-m) w_i}."""
    L, D = 9, 8
    q, k, v = (rng.standard_normal((1, L, 1, D)) for _ in range(3))
    _, lse, probs = oracle.self_attn(q, k, v, (L, 1, 1), (D, 0, 0), want_lse=True, probs_of=(0, 0))
    w = 10000.0 ** (-2.0 * np.arange(D // 2) / D)
    zq = q[0, :, 0, 0::2] + 1j * q[0, :, 0, 1::2]
    zk = k[0, :, 0, 0::2] + 1j * k[0, :, 0, 1::2]
    n = np.arange(L)
    phase = np.exp(1j * (n[:, None, None] - n[None, :, None]) * w[None, None, :])
    s = (zq[:, None, :] * np.conj(zk)[None, :, :] * phase).real.sum(-1) / math.sqrt(D)
    want = np.exp(s - s.max(1, keepdims=True))
    want /= want.sum(1, keepdims=True)
    np.testing.assert_allclose(probs, want, atol=1e-13)
    np.testing.assert_allclose(lse[0, 0], np.log(np.exp(s).sum(1)), atol=1e-12)
    # the same tokens laid along w with split (0,0,D) must give the same result
    _, probs_w = oracle.self_attn(q, k, v, (1, 1, L), (0, 0, D), probs_of=(0, 0))
    np.testing.assert_allclose(probs_w, probs, atol=1e-14)


def test_p10_axis_separability_and_section_order(rng):
    D, split = 8, (4, 2, 2)
    x = rng.standard_normal((1, D))
    base_pos = np.array([[3, 4, 5]])
    y0 = oracle.rope3d(x, base_pos, split)
    for axis, sl in enumerate((slice(0, 4), slice(4, 6), slice(6, 8))):
        p = base_pos.copy(); p[0, axis] += 2
        y1 = oracle.rope3d(x, p, split)
        changed = np.abs(y1 - y0) > 1e-12
        assert changed[0, sl].any()
        mask = np.ones(D, bool); mask[sl] = False
        assert not changed[0, mask].any()
    # swapping the h and w axes of the grid together with their sections and the token order
    grid = (2, 3, 4)
    L = 24
    q, k, v = (rng.standard_normal((1, L, 1, D)) for _ in range(3))
    out = oracle.self_attn(q, k, v, grid, (4, 2, 2))
    perm = np.arange(L).reshape(2, 3, 4).transpose(0, 2, 1).reshape(-1)  # new token order (t, w, h)
    chan = np.array([0, 1, 2, 3, 6, 7, 4, 5])
    q2, k2 = (a[:, perm][..., chan] for a in (q, k))
    v2 = v[:, perm]
    out2 = oracle.self_attn(q2, k2, v2, (2, 4, 3), (4, 2, 2))
    np.testing.assert_allclose(out2, out[:, perm], atol=1e-13)


def test_p11_permutation_properties_cross(rng):
    B, Lq, Lk, H, D = 2, 6, 13, 2, 8
    q = rng.standard_normal((B, Lq, H, D)); k = rng.standard_normal((B, Lk, H, D)); v = rng.standard_normal((B, Lk, H, D))
    valid = (rng.random((B, Lk)) < 0.7).astype(np.uint8); valid[:, 0] = 1
    out = oracle.cross_attn(q, k, v, valid)
    pk = rng.permutation(Lk)
    out_k = oracle.cross_attn(q, k[:, pk], v[:, pk], valid[:, pk])
    np.testing.assert_allclose(out_k, out, atol=1e-14)
    pq = rng.permutation(Lq)
    out_q = oracle.cross_attn(q[:, pq], k, v, valid)
    np.testing.assert_allclose(out_q, out[:, pq], atol=0)
    # heads and batches are independent: swapping heads swaps outputs
    out_h = oracle.cross_attn(q[:, :, ::-1], k[:, :, ::-1], v[:, :, ::-1], valid)
    np.testing.assert_allclose(out_h, out[:, :, ::-1], atol=0)
    # rows= selects exactly those rows
    sel = oracle.cross_attn(q, k, v, valid, rows=[4, 1])
    np.testing.assert_allclose(sel, out[:, [4, 1]], atol=0)


def test_p12_mask_equals_compaction(rng):
    B, Lq, Lk, H, D = 1, 5, 17, 2, 8
    q = rng.standard_normal((B, Lq, H, D)); k = rng.standard_normal((B, Lk, H, D)); v = rng.standard_normal((B, Lk, H, D))
    valid = np.zeros((B, Lk), dtype=np.uint8); idx = [0, 2, 3, 9, 16]; valid[0, idx] = 1
    k2, v2 = k.copy(), v.copy()
    k2[0, valid[0] == 0] = 1e30; v2[0, valid[0] == 0] = -1e30  # garbage under the mask must not leak
    out, lse = oracle.cross_attn(q, k2, v2, valid, want_lse=True)
    outc, lsec = oracle.cross_attn(q, k[:, idx], v[:, idx], None, want_lse=True)
    np.testing.assert_allclose(out, outc, atol=1e-14)
    np.testing.assert_allclose(lse, lsec, atol=1e-14)
    # fully masked request: zeros and lse = -inf
    valid0 = np.zeros((B, Lk), dtype=np.uint8)
    out0, lse0 = oracle.cross_attn(q, k, v, valid0, want_lse=True)
    assert np.all(out0 == 0.0) and np.all(np.isneginf(lse0))


def test_p13_lse_and_merge(rng):
    B, Lq, Lk, H, D = 1, 4, 12, 1, 8
    q = rng.standard_normal((B, Lq, H, D)) * 2; k = rng.standard_normal((B, Lk, H, D)); v = rng.standard_normal((B, Lk, H, D))
    out, lse = oracle.cross_attn(q, k, v, None, want_lse=True, scale=0.5)
    s = 0.5 * np.einsum("nd,md->nm", q[0, :, 0].astype(np.longdouble), k[0, :, 0].astype(np.longdouble))
    np.testing.assert_allclose(lse[0, 0], np.log(np.exp(s).sum(1)).astype(np.float64), atol=1e-14)
    va = np.zeros((B, Lk), np.uint8); va[0, :5] = 1
    vb = 1 - va
    oa, la = oracle.cross_attn(q, k, v, va, want_lse=True, scale=0.5)
    ob, lb = oracle.cross_attn(q, k, v, vb, want_lse=True, scale=0.5)
    wa = np.exp(la - lse)[0, 0][None, :, None, None]; wb = np.exp(lb - lse)[0, 0][None, :, None, None]
    np.testing.assert_allclose(wa * oa + wb * ob, out, atol=1e-14)


def test_dtype_widening_is_exact(rng):
    """bf16 bit patterns and float32 inputs are widened, never rounded."""
    from paper_2601_20655_amd import workloads as wl

    grid, D = (2, 2, 3), 8
    L = 12
    x = [rng.standard_normal((1, L, 2, D)).astype(np.float32) for _ in range(3)]
    bits = [wl.f32_to_bf16_bits(a) for a in x]
    wide = [wl.bf16_bits_to_f32(b).astype(np.float64) for b in bits]
    a = oracle.self_attn(*bits, grid, SPLITS[8])
    b = oracle.self_attn(*wide, grid, SPLITS[8])
    c = oracle.self_attn(*[w.astype(np.float32) for w in wide], grid, SPLITS[8])
    assert np.array_equal(a, b) and np.array_equal(a, c)
    # bf16 rounding helper: ties to even on known patterns
    t = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.0e-39], dtype=np.float32)  # 1+2^-8 ties down, 1+3*2^-8 ties up
    got = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(t))
    np.testing.assert_array_equal(got[:4], np.array([1.0, 1.0, 1.015625, -2.5], dtype=np.float32))


def test_bad_arguments_are_rejected(rng):
    q = rng.standard_normal((1, 4, 1, 8))
    with pytest.raises(ValueError):
        oracle.self_attn(q, q, q, (2, 2, 1), (4, 2, 1))  # odd section / wrong sum
    with pytest.raises(ValueError):
        oracle.self_attn(q, q, q, (2, 2, 1), (4, 2, 2), rows=[4])
    with pytest.raises(ValueError):
        oracle.cross_attn(q, q, q, rows=[-1])


def brute_decoupled(q, k, v, split, valid, scale):
    """One head, pure loops: two explicit softmaxes over the two key ranges, outputs added."""
    Lq, D = q.shape
    out = np.zeros((Lq, D))
    for n in range(Lq):
        for lo, hi in ((0, split), (split, k.shape[0])):
            keys = [m for m in range(lo, hi) if valid[m]]
            if not keys:
                continue
            s = [scale * float(np.dot(q[n], k[m])) for m in keys]
            mx = max(s)
            e = [math.exp(x - mx) for x in s]
            z = math.fsum(e)
            for w, m in zip(e, keys):
                out[n] += (w / z) * v[m]
    return out


def test_decoupled_cross_attention_pins(rng):
    B, Lq, Lk, H, D, split = 2, 5, 13, 2, 8, 6
    q = rng.standard_normal((B, Lq, H, D)); k = rng.standard_normal((B, Lk, H, D)); v = rng.standard_normal((B, Lk, H, D))
    valid = np.ones((B, Lk), np.uint8); valid[0, [1, 4, 9]] = 0; valid[1, split:] = 0   # request 1: second group empty
    out = oracle.cross_attn_decoupled(q, k, v, split, valid, scale=0.4)
    for b in range(B):
        for h in range(H):
            np.testing.assert_allclose(out[b, :, h], brute_decoupled(q[b, :, h], k[b, :, h], v[b, :, h], split, valid[b], 0.4),
                                       atol=1e-13)
    # an empty second group leaves the joint softmax over the first
    np.testing.assert_allclose(out[1], oracle.cross_attn(q[1:], k[1:, :split], v[1:, :split], valid[1:, :split], scale=0.4)[0], atol=0)
    # split at either end is the joint softmax over everything
    joint = oracle.cross_attn(q, k, v, valid, scale=0.4)
    np.testing.assert_allclose(oracle.cross_attn_decoupled(q, k, v, Lk, valid, scale=0.4), joint, atol=0)
    np.testing.assert_allclose(oracle.cross_attn_decoupled(q, k, v, 0, valid, scale=0.4), joint, atol=0)
    # constant values: each non-empty group returns c, so the sum is (number of non-empty groups) * c
    c = rng.standard_normal(D)
    vc = np.broadcast_to(c, v.shape).copy()
    oc = oracle.cross_attn_decoupled(q, k, vc, split, valid)
    np.testing.assert_allclose(oc[0], np.broadcast_to(2 * c, oc[0].shape), atol=1e-14)
    np.testing.assert_allclose(oc[1], np.broadcast_to(c, oc[1].shape), atol=1e-14)
    # q = 0: uniform weights inside each group -> mean of group A + mean of group B (valid keys only)
    o0 = oracle.cross_attn_decoupled(np.zeros_like(q), k, v, split, valid)
    a_idx = [m for m in range(split) if valid[0, m]]; b_idx = [m for m in range(split, Lk) if valid[0, m]]
    want = v[0, a_idx].mean(axis=0) + v[0, b_idx].mean(axis=0)
    np.testing.assert_allclose(o0[0], np.broadcast_to(want, o0[0].shape), atol=1e-14)
    # it is NOT the joint softmax in general
    assert np.max(np.abs(out[0] - joint[0])) > 1e-2


def test_packed_requests_equal_block_diagonal_attention(rng):
    """Packed requests: attention over ALL packed tokens with a block-diagonal mask (a token sees
    its own request only) and per-request positions, written out with numpy on complex pairs."""
    grids = [(2, 2, 3), (1, 1, 1), (1, 3, 2), (2, 1, 2)]
    D, H, split, base, scale = 8, 2, (4, 2, 2), 100.0, 0.3
    N = sum(int(np.prod(g)) for g in grids)
    q, k, v = (rng.standard_normal((N, H, D)) for _ in range(3))
    out, lse = oracle.self_attn_packed(q, k, v, grids, split, origin=(1, 2, 3), base=base, scale=scale, want_lse=True)
    # positions and request ids of the packed tokens
    pos, rid = [], []
    for i, (T, Hg, Wg) in enumerate(grids):
        for t in range(T):
            for h in range(Hg):
                for w in range(Wg):
                    pos.append((1 + t, 2 + h, 3 + w))
                    rid.append(i)
    pos, rid = np.array(pos, dtype=np.float64), np.array(rid)
    omega = np.concatenate([base ** (-2.0 * np.arange(split[a] // 2) / split[a]) for a in range(3)])
    axis = np.concatenate([np.full(split[a] // 2, a) for a in range(3)])
    phase = np.exp(1j * pos[:, axis] * omega[None, :])  # [N, D/2]
    for h in range(H):
        zq = (q[:, h, 0::2] + 1j * q[:, h, 1::2]) * phase
        zk = (k[:, h, 0::2] + 1j * k[:, h, 1::2]) * phase
        s = scale * (zq @ zk.conj().T).real
        s[rid[:, None] != rid[None, :]] = -np.inf
        mx = s.max(axis=1, keepdims=True)
        e = np.exp(s - mx)
        z = e.sum(axis=1, keepdims=True)
        np.testing.assert_allclose(out[:, h], (e / z) @ v[:, h], rtol=0, atol=1e-12)
        np.testing.assert_allclose(lse[h], (mx + np.log(z))[:, 0], rtol=0, atol=1e-12)
    # one request alone is the plain call
    one = oracle.self_attn_packed(q[:12], k[:12], v[:12], grids[:1], split, base=base, scale=scale)
    np.testing.assert_array_equal(one, oracle.self_attn(q[None, :12], k[None, :12], v[None, :12], grids[0], split,
                                                        base=base, scale=scale)[0])


def test_qk_rmsnorm_pins(rng):
    # worked example by hand: x = (3, 4): mean square 12.5, y = x / sqrt(12.5)
    y = oracle.qk_rmsnorm(np.array([[[3.0, 4.0]]]), eps=0.0)
    np.testing.assert_allclose(y[0, 0], [0.848528137423857, 1.131370849898476], rtol=0, atol=1e-15)
    # with eps: x = (1, 1, 1, 1), eps = 3 -> 1 / sqrt(1 + 3) = 0.5; gamma scales channel-wise
    y = oracle.qk_rmsnorm(np.ones((1, 1, 4)), gamma=np.array([[1.0, 2.0, -1.0, 0.0]]), eps=3.0)
    np.testing.assert_allclose(y[0, 0], [0.5, 1.0, -0.5, 0.0], rtol=0, atol=1e-15)
    # zero rows stay zero (no division by zero with eps > 0)
    assert np.all(oracle.qk_rmsnorm(np.zeros((2, 3, 8)), eps=1e-6) == 0.0)
    x = rng.standard_normal((5, 3, 16)) * 7.0
    g = rng.standard_normal((3, 16))
    for mode in ("head", "token"):
        y = oracle.qk_rmsnorm(x, eps=0.0, mode=mode)
        ax = -1 if mode == "head" else (-2, -1)
        np.testing.assert_allclose(np.mean(y * y, axis=ax), 1.0, rtol=1e-13)           # unit mean square
        np.testing.assert_allclose(oracle.qk_rmsnorm(-3.5 * x, eps=0.0, mode=mode), -y, rtol=1e-13)  # scale-free
        np.testing.assert_allclose(oracle.qk_rmsnorm(x, g, 0.0, mode), y * g, rtol=1e-13)
    # "token" mode is "head" mode on the flattened row, and both agree for one head
    np.testing.assert_allclose(oracle.qk_rmsnorm(x, g, 1e-3, "token").reshape(5, 1, 48),
                               oracle.qk_rmsnorm(x.reshape(5, 1, 48), g.reshape(1, 48), 1e-3, "head"), rtol=1e-14)
    # library routine on the same numbers
    import torch

    t = torch.nn.functional.rms_norm(torch.from_numpy(x), (16,), torch.from_numpy(g[1]), eps=1e-5).numpy()
    np.testing.assert_allclose(oracle.qk_rmsnorm(x, np.broadcast_to(g[1], (3, 16)), 1e-5, "head"), t, rtol=1e-12)
    # bf16 bit patterns are decoded exactly: 0x3FC0 = 1.5, 0xC000 = -2.0
    np.testing.assert_array_equal(oracle.as_f64(np.array([0x3FC0, 0xC000, 0x0000], dtype=np.uint16)), [1.5, -2.0, 0.0])


def test_normed_attention_pins(rng):
    """Normalise-then-attend: with gamma = 1 and eps = 0 the scores depend on directions only, so
    scaling q rows and k rows by arbitrary positive factors changes nothing; and a brute-force
    evaluation on pre-normalised rows agrees."""
    grid, D, H = (2, 2, 3), 8, 2
    L = 12
    q, k, v = (rng.standard_normal((1, L, H, D)) for _ in range(3))
    a = oracle.self_attn_normed(q, k, v, grid, SPLITS[D], eps=0.0)
    fq = rng.uniform(0.1, 9.0, size=(1, L, H, 1))
    fk = rng.uniform(0.1, 9.0, size=(1, L, H, 1))
    b = oracle.self_attn_normed(q * fq, k * fk, v, grid, SPLITS[D], eps=0.0)
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-12)
    g = rng.standard_normal((H, D))
    c = oracle.self_attn_normed(q, k, v, grid, SPLITS[D], q_gamma=g, k_gamma=2 * g, eps=1e-2, mode="token")
    for h in range(H):
        msq = np.mean(q[0] ** 2, axis=(1, 2))[:, None]
        msk = np.mean(k[0] ** 2, axis=(1, 2))[:, None]
        qn = q[0, :, h] / np.sqrt(msq + 1e-2) * g[h]
        kn = k[0, :, h] / np.sqrt(msk + 1e-2) * 2 * g[h]
        ref, _, _ = brute_self_attn(qn, kn, v[0, :, h], grid, SPLITS[D])
        np.testing.assert_allclose(c[0, :, h], ref, rtol=0, atol=1e-12)


GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def test_hand_worked_cases_from_golden_folder():
    """Cases with exact, pencil-and-paper expected values (derivations in the fixture)."""
    cases = json.load(open(os.path.join(GOLDEN, "hand_worked_cases.json")))
    for name, c in cases.items():
        if c["kind"] in ("cross", "decoupled"):
            q = np.array(c["q"], dtype=np.float64)[None, :, None, :]
            k = np.array(c["k"], dtype=np.float64)[None, :, None, :]
            v = np.array(c["v"], dtype=np.float64)[None, :, None, :]
            valid = np.array(c["valid"], dtype=np.uint8)[None]
            if c["kind"] == "cross":
                out, lse = oracle.cross_attn(q, k, v, valid, scale=c["scale"], want_lse=True)
                np.testing.assert_allclose(lse[0, 0], c["lse"], rtol=0, atol=1e-14, err_msg=name)
            else:
                out = oracle.cross_attn_decoupled(q, k, v, c["split"], valid, scale=c["scale"])
            np.testing.assert_allclose(out[0, :, 0], c["out"], rtol=0, atol=1e-15, err_msg=name)
        elif c["kind"] == "packed":
            q, k, v = (np.array(c[n], dtype=np.float64)[:, None, :] for n in ("q", "k", "v"))
            out = oracle.self_attn_packed(q, k, v, [tuple(g) for g in c["grids"]], tuple(c["split"]))
            np.testing.assert_allclose(out[:, 0], c["out"], rtol=0, atol=1e-15, err_msg=name)
        elif c["kind"] == "rmsnorm":
            x = np.array(c["x"], dtype=np.float64)[None, None, :]
            for cc in c["cases"]:
                g = None if cc["gamma"] is None else np.array(cc["gamma"])[None]
                y = oracle.qk_rmsnorm(x, g, cc["eps"], "head")
                np.testing.assert_allclose(y[0, 0], cc["y"], rtol=0, atol=2e-16, err_msg=name)
        else:
            raise AssertionError("unknown case kind in %s" % name)


def test_oracle_matches_its_stored_regression_values():
    """The stored file was written by tests/golden/make_golden.py from the oracle alone; a change
    of the oracle's arithmetic shows up here first."""
    sys.path.insert(0, GOLDEN)
    import make_golden

    stored = [l.rstrip("\n") for l in open(os.path.join(GOLDEN, "oracle_tiny_regression.txt")) if not l.startswith("#")]
    now = make_golden.values()
    assert len(stored) == len(now)
    for a, b in zip(stored, now):
        ta, tb = a.split(), b.split()
        assert ta[:4] == tb[:4]
        fa = np.array([float(x) for x in ta if "e" in x and x[0] in "-0123456789"])
        fb = np.array([float(x) for x in tb if "e" in x and x[0] in "-0123456789"])
        np.testing.assert_allclose(fa, fb, rtol=1e-12, atol=1e-15)


# ---- the 8-bit score operands (E4M3) ----

def e4m3_code_values():
    """All finite E4M3 values, decoded from the format's definition: sign, 4 exponent bits (bias 7),
    3 mantissa bits; exponent field 0 = subnormal m/8 * 2^-6; field 15 with mantissa 7 = NaN."""
    vals = []
    for code in range(256):
        s, e, m = code >> 7, (code >> 3) & 15, code & 7
        if e == 15 and m == 7:
            continue
        mag = (m / 8.0) * 2.0 ** -6 if e == 0 else (1.0 + m / 8.0) * 2.0 ** (e - 7)
        vals.append((-mag if s else mag, m))
    return vals


def test_e4m3_round_pins(rng):
    vals = e4m3_code_values()
    mags = sorted({abs(x) for x, _ in vals})
    assert len(mags) == 127 and mags[0] == 0.0 and mags[1] == 2.0 ** -9 and mags[-1] == 448.0
    # every code value is a fixed point; a point between two neighbours goes to the nearer one
    allv = np.array([x for x, _ in vals])
    assert np.array_equal(oracle.e4m3_round(allv), allv)
    lo, hi = np.array(mags[:-1]), np.array(mags[1:])
    assert np.array_equal(oracle.e4m3_round(lo + 0.25 * (hi - lo)), lo)
    assert np.array_equal(oracle.e4m3_round(-(lo + 0.75 * (hi - lo))), -hi)
    # ties go to the neighbour with the even mantissa
    mant = {abs(x): m for x, m in vals}
    tie = oracle.e4m3_round(0.5 * (lo + hi))
    for t, a, b in zip(tie, lo, hi):
        assert t == (a if mant[a] % 2 == 0 else b)
    # hand values: step 2^-5 below 0.5, step 2 between 16 and 32, saturation, the smallest tie
    assert np.array_equal(oracle.e4m3_round([0.3, 17.0, 19.0, 500.0, -1e9, 2.0 ** -10, 3 * 2.0 ** -10]),
                          [0.3125, 16.0, 20.0, 448.0, -448.0, 0.0, 2.0 ** -8])
    # an independent library routine: torch's cast to float8_e4m3fn
    import torch

    x = np.concatenate([rng.normal(size=20000) * s for s in (1e-3, 0.05, 1.0, 30.0, 150.0)]).astype(np.float32)
    x = x[np.abs(x) <= 448.0]
    ref = torch.from_numpy(x).to(torch.float8_e4m3fn).to(torch.float64).numpy()
    assert np.array_equal(oracle.e4m3_round(x.astype(np.float64)), ref)


def test_e4m3_quantise_rows_pins(rng):
    # values with at most 4 significant bits, within 2^14 of the row's largest: unchanged
    x = np.array([[3.0, -0.75, 1.5, 0.09375, 0.0, 13.0 * 2.0 ** -12], [-15.0 * 2.0 ** 40, 2.0 ** 30, 9.0 * 2.0 ** 35, 0, 0, 0]])
    assert np.array_equal(oracle.e4m3_quantise_rows(x), x)
    assert np.array_equal(oracle.e4m3_quantise_rows(np.zeros((2, 5))), np.zeros((2, 5)))
    # a power of two in front of a row changes nothing else; rows do not influence each other
    y = rng.normal(size=(7, 64))
    qy = oracle.e4m3_quantise_rows(y)
    assert np.array_equal(oracle.e4m3_quantise_rows(y * 2.0 ** -17), qy * 2.0 ** -17)
    assert np.array_equal(oracle.e4m3_quantise_rows(y[3:4]), qy[3:4])
    # the scaled row tops out in [128, 256): elements round with 4 significant bits (relative error
    # at most 2^-4) down to 2^-6 / 256 of the largest; the largest element itself keeps that bound
    big = np.abs(y) >= np.max(np.abs(y), axis=1, keepdims=True) * 2.0 ** -13
    assert np.all(np.abs(qy - y)[big] <= 2.0 ** -4 * np.abs(y)[big])
    # hand-worked row: largest 5.3 -> factor 2^5 (169.6 in [128, 256)), steps 16/32 = 0.5 in [4, 8),
    # 2/32 = 0.0625 in [0.5, 1), subnormal step 2^-9 / 32 below 2^-6 / 32
    assert np.array_equal(oracle.e4m3_quantise_rows(np.array([[5.3, 0.7, 2.0 ** -13]])),
                          [[5.5, 0.6875, 2.0 ** -13]])
    # (1.4 * 2^-15 * 32 = 0.7 * 2^-9 -> one subnormal step; 0.4 * 2^-14 * 32 = 0.4 * 2^-9 -> zero)
    assert np.array_equal(oracle.e4m3_quantise_rows(np.array([[5.3, 2.0 ** -15 * 1.4, 2.0 ** -14 * 0.4]])),
                          [[5.5, 2.0 ** -14, 0.0]])


def test_self_attn_fp8_scores_pins(rng, monkeypatch):
    grid, split, D = (2, 3, 20), (22, 20, 22), 64
    L = int(np.prod(grid))
    q, k, v = (rng.normal(size=(1, L, 2, D)) for _ in range(3))
    kw = dict(origin=(3, -1, 2), base=300.0, scale=0.2)
    exact = oracle.self_attn(q, k, v, grid, split, **kw)
    # with the rounding taken out, the routine is the plain definition (rotation, scale, base-2 softmax)
    import oracle.dit_oracle as impl

    with monkeypatch.context() as mp:
        mp.setattr(impl, "e4m3_quantise_rows", lambda x: np.asarray(x, dtype=np.float64))
        assert np.max(np.abs(oracle.self_attn_fp8_scores(q, k, v, grid, split, **kw) - exact)) < 1e-12
    # with it, the result moves by what the rounding model predicts: relative operand error of RMS
    # 2^-4 / sqrt(3) * 0.7355 on both sides, score spread sigma_s = scale * sqrt(D) for unit inputs
    got = oracle.self_attn_fp8_scores(q, k, v, grid, split, **kw)
    err = np.sqrt(np.mean((got - exact) ** 2)) / np.sqrt(np.mean(exact ** 2))
    predicted = 2.0 ** -4 / math.sqrt(3.0) * 0.7355 * math.sqrt(2.0) * (0.2 * math.sqrt(D))
    assert 0.6 * predicted < err < 1.4 * predicted, (err, predicted)
    # a single key: the output is that value row whatever the scores round to
    one = oracle.self_attn_fp8_scores(q[:, :1], k[:, :1], v[:, :1], (1, 1, 1), split)
    assert np.array_equal(one, v[:, :1])


def test_linear_pins(rng):
    """y = x w^T + bias with w stored [out, in]: brute force by loops in Python floats, the
    identity and one-hot weights (which catch a transposed operand), a rectangular shape (which
    catches swapped M/N), additivity in the bias, and exact widening of 16-bit inputs."""
    M, N, K = 5, 3, 7
    x, w, b = rng.normal(size=(M, K)), rng.normal(size=(N, K)), rng.normal(size=N)
    y = oracle.linear(x, w, b)
    assert y.shape == (M, N) and y.dtype == np.float64
    for m in range(M):
        for n in range(N):
            acc = math.fsum(float(x[m, k]) * float(w[n, k]) for k in range(K)) + float(b[n])
            assert abs(y[m, n] - acc) < 1e-13
    # one-hot rows of w pick columns of x; w[n, k] = 1 means output n reads input k
    sel = np.zeros((N, K))
    sel[0, 4] = sel[1, 0] = sel[2, 6] = 1.0
    assert np.array_equal(oracle.linear(x, sel), x[:, [4, 0, 6]])
    assert np.array_equal(oracle.linear(x, np.eye(K)), x)
    assert np.max(np.abs(oracle.linear(x, w) + b[None, :] - y)) < 1e-14
    # bf16 bit patterns widen exactly: 0x3FC0 = 1.5, 0xC000 = -2, 0x3E80 = 0.25
    xb = np.array([[0x3FC0, 0xC000]], dtype=np.uint16)
    wb = np.array([[0x3E80, 0x3FC0], [0xC000, 0x3E80]], dtype=np.uint16)
    assert np.array_equal(oracle.linear(xb, wb, np.array([0x3FC0, 0x0000], dtype=np.uint16)),
                          np.array([[1.5 * 0.25 - 2 * 1.5 + 1.5, -3.0 - 0.5]]))
