"""CPU pin of tests/fp8_error_model.py, the statistics the 8-bit-score GPU tests are judged with: applied to
oracle.self_attn_fp8_scores (the E4M3 rounding written out in numpy, itself pinned against the format's code
table in test_oracle_pins.py) versus the plain definition oracle.self_attn, the predicted per-element standard
deviation must describe the actual differences -- normalised RMS close to 1, largest normalised error inside
the Gaussian tail -- on a uniform-softmax case, a long-sequence case and a peaky one.  A wrong step size
(e.g. 2 instead of 3 mantissa bits, a missing row factor, a forgotten ln 2) moves the RMS by 2x or more."""
import numpy as np
import pytest

import oracle
import fp8_error_model as em
from paper_2601_20655_amd import workloads as wl

CASES = {
    "tiny": (wl.CONFIGS["tiny"], 1.0, {}),
    "long": (dict(wl.CONFIGS["mid"], grid=(1, 30, 52), H=2), 1.0, dict(origin=(2, -3, 1))),
    "peaky": (dict(B=1, grid=(3, 9, 17), H=2, D=128, split=(44, 42, 42), dtype="bf16", seed=4242), 2.0,
              dict(scale=0.11)),
}


@pytest.mark.parametrize("name", sorted(CASES))
def test_model_describes_the_quantiser(name):
    cfg, gain, kw = CASES[name]
    q, k, v = wl.self_attn_inputs(cfg, gain=gain)
    ref = oracle.self_attn(q, k, v, cfg["grid"], cfg["split"], **kw)
    quantised = oracle.self_attn_fp8_scores(q, k, v, cfg["grid"], cfg["split"], **kw)
    pred = em.predicted_std_self(q, k, v, cfg["grid"], cfg["split"], **kw)
    assert np.all(pred > 0)
    z = (quantised - ref) / pred
    assert 0.9 <= np.sqrt(np.mean(z * z)) <= 1.1
    assert np.abs(z).max() <= em.gaussian_tail_z(z.size)


def test_step_sizes():
    # a row whose largest magnitude is 200 needs no factor: steps 16 at [128, 256), 1/8 at [1, 2), 2^-9 below 2^-6
    x = np.array([[200.0, 1.5, 0.001, 0.0, -130.0]])
    assert np.array_equal(em.e4m3_step(x), [[16.0, 0.125, 2.0 ** -9, 2.0 ** -9, 16.0]])
    # the same row scaled by 2^-10 has the same steps scaled by 2^-10
    assert np.array_equal(em.e4m3_step(x * 2.0 ** -10), em.e4m3_step(x) * 2.0 ** -10)
    # every e4m3 value is a multiple of its own step and its neighbours are one step away
    vals = np.array([[240.0, 3.5, 0.4375, 2.0 ** -6]])
    assert np.array_equal(oracle.e4m3_round(vals), vals)
    assert np.array_equal(oracle.e4m3_round(vals + 0.49 * em.e4m3_step(vals)), vals)
    assert np.all(oracle.e4m3_round(vals + 0.51 * em.e4m3_step(vals)) > vals)
