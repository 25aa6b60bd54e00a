"""Seeded synthetic workloads for the DiT attention hot path.

This module only *generates inputs* (shapes, N(0,1) values, bf16 bit patterns, key-padding
masks, sampled row lists).  It holds none of the attention arithmetic, so both the GPU
library's tests and the CPU oracle's tests can be fed from it.

The tensors stand in for the activations of a Wan2.1-class video diffusion transformer
(the Diffusion stage of the paper's image-to-video workflow, Sec. 2.4): same shapes, same
dense (T,Hg,Wg) position lattice, unit-variance values.  No trained weights are involved.
"""
import numpy as np

# name -> description of the five reference shapes
CONFIGS = {
    "tiny": dict(kind="self", B=1, grid=(4, 8, 8), H=4, D=64, split=(22, 20, 22), dtype="f32",
                 seed=20655 + 1),
    "dit_1p3b": dict(kind="self", B=1, grid=(21, 30, 52), H=12, D=128, split=(44, 42, 42),
                     dtype="bf16", seed=20655 + 2),
    "dit_14b": dict(kind="self", B=1, grid=(21, 30, 52), H=40, D=128, split=(44, 42, 42),
                    dtype="bf16", seed=20655 + 3),
    "dit_14b_hires": dict(kind="self", B=1, grid=(21, 45, 80), H=40, D=128, split=(44, 42, 42),
                          dtype="bf16", seed=20655 + 4),
    "cross_14b": dict(kind="cross", B=4, Lq=32760, n_text=512, n_image=257, H=40, D=128,
                      dtype="bf16", min_text=16, seed=20655 + 5),
    # mid-size shape for an all-rows comparison that spans several tiles and a ragged tail
    "mid": dict(kind="self", B=1, grid=(4, 30, 52), H=4, D=128, split=(44, 42, 42),
                dtype="bf16", seed=20655 + 6),
    # several requests of different grids packed along the token axis (batched serving)
    "varlen_small": dict(kind="varlen", grids=((2, 5, 7), (3, 16, 20), (1, 1, 1), (4, 9, 13), (2, 16, 16),
                                               (1, 8, 8)),
                         H=4, D=128, split=(44, 42, 42), dtype="bf16", seed=20655 + 7),
    "varlen_small_d64": dict(kind="varlen", grids=((3, 7, 9), (1, 3, 5), (5, 12, 11)),
                             H=3, D=64, split=(22, 20, 22), dtype="f32", seed=20655 + 8),
    # a mixed batch at 14B width: 720p and 480p clips of 81, 49 and 33 frames plus a still image
    "varlen_14b": dict(kind="varlen", grids=((13, 30, 52), (21, 45, 80), (1, 45, 80), (21, 30, 52), (9, 45, 80),
                                             (13, 30, 52), (21, 30, 52)),
                       H=40, D=128, split=(44, 42, 42), dtype="bf16", seed=20655 + 9),
    # the dense projections either side of attention at 14B width (5,120 = 40 heads x 128): the fused
    # q/k/v projection (three weights stacked along the output axis) and the output projection
    "qkv_proj_14b": dict(kind="linear", M=32760, N=3 * 5120, K=5120, seed=20655 + 10),
    "out_proj_14b": dict(kind="linear", M=32760, N=5120, K=5120, seed=20655 + 11),
    # the front of a block at 14B width: the q/k/v projection of 32,760 token rows, then self-attention on its output
    "qkv_attn_14b": dict(kind="qkv_attn", grid=(21, 30, 52), split=(44, 42, 42), H=40, D=128, K=5120,
                         seed=20655 + 13),
    # all-elements comparison: two full tiles and a ragged one along both M and N, three K steps
    "proj_small": dict(kind="linear", M=600, N=520, K=192, seed=20655 + 12),
}


def f32_to_bf16_bits(x):
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return rounded.astype(np.uint16)


def bf16_bits_to_f32(b):
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal(shape, seed, stream, dtype="bf16", gain=1.0):
    """iid N(0, gain^2) tensor; stream separates q/k/v.  bf16 -> uint16 bit patterns."""
    rng = np.random.default_rng([int(seed), int(stream)])
    x = rng.standard_normal(size=shape, dtype=np.float32)
    if gain != 1.0:
        x *= np.float32(gain)
    if dtype == "bf16":
        return f32_to_bf16_bits(x)
    if dtype == "f32":
        return x
    raise ValueError(dtype)


def self_attn_inputs(cfg, seed=None, gain=1.0, dtype=None):
    """q, k, v of shape [B, L, H, D] for a self-attention config dict."""
    T, Hg, Wg = cfg["grid"]
    shape = (cfg["B"], T * Hg * Wg, cfg["H"], cfg["D"])
    seed = cfg["seed"] if seed is None else seed
    dtype = cfg["dtype"] if dtype is None else dtype
    return tuple(normal(shape, seed, s, dtype, gain if s < 2 else 1.0) for s in range(3))


def varlen_attn_inputs(cfg, seed=None, dtype=None):
    """q, k, v of shape [sum of T*Hg*Wg over cfg["grids"], H, D], requests back to back."""
    n = sum(t * h * w for t, h, w in cfg["grids"])
    shape = (n, cfg["H"], cfg["D"])
    seed = cfg["seed"] if seed is None else seed
    dtype = cfg["dtype"] if dtype is None else dtype
    return tuple(normal(shape, seed, s, dtype) for s in range(3))


def norm_weights(cfg, seed=None):
    """Channel weights of the q and k normalisation layers, [H, D] float32 each, 1 + 0.25 N(0,1)
    (trained weights of such layers sit around one)."""
    seed = cfg["seed"] if seed is None else seed
    shape = (cfg["H"], cfg["D"])
    return tuple((1.0 + 0.25 * normal(shape, seed, s, "f32")).astype(np.float32) for s in (7, 8))


def cross_attn_inputs(cfg, seed=None, dtype=None):
    """q [B,Lq,H,D], k, v [B,Lk,H,D], kv_valid [B,Lk] uint8, text_len [B].

    Keys [0, n_text) are text tokens of which the first text_len[b] are valid
    (text_len ~ U{min_text..n_text}); keys [n_text, n_text+n_image) are image tokens,
    always valid.
    """
    seed = cfg["seed"] if seed is None else seed
    dtype = cfg["dtype"] if dtype is None else dtype
    B, H, D = cfg["B"], cfg["H"], cfg["D"]
    Lk = cfg["n_text"] + cfg["n_image"]
    q = normal((B, cfg["Lq"], H, D), seed, 0, dtype)
    k = normal((B, Lk, H, D), seed, 1, dtype)
    v = normal((B, Lk, H, D), seed, 2, dtype)
    rng = np.random.default_rng([int(seed), 3])
    text_len = rng.integers(cfg["min_text"], cfg["n_text"] + 1, size=B)
    valid = np.zeros((B, Lk), dtype=np.uint8)
    for b in range(B):
        valid[b, : text_len[b]] = 1
        valid[b, cfg["n_text"]:] = 1
    return q, k, v, valid, text_len


def linear_inputs(cfg, seed=None):
    """x [M, K] ~ N(0, 1), w [N, K] ~ N(0, 1/K) (so outputs have unit variance, as after a
    normalisation layer and a variance-preserving initialisation), bias [N] ~ N(0, 0.1^2); bf16 bits."""
    seed = cfg["seed"] if seed is None else seed
    x = normal((cfg["M"], cfg["K"]), seed, 0)
    w = normal((cfg["N"], cfg["K"]), seed, 1, gain=cfg["K"] ** -0.5)
    b = normal((cfg["N"],), seed, 2, gain=0.1)
    return x, w, b


def sample_rows(L, seed, edge=64, n_random=128):
    """First `edge` rows, last `edge` rows and n_random seeded rows in between (sorted, unique)."""
    if L <= 2 * edge + n_random:
        return np.arange(L, dtype=np.int64)
    rng = np.random.default_rng([int(seed), 7])
    mid = rng.choice(np.arange(edge, L - edge), size=n_random, replace=False)
    return np.unique(np.concatenate([np.arange(edge), np.arange(L - edge, L), mid])).astype(np.int64)
