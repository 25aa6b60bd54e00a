"""Predicted size of the error the 8-bit score operands (library flag DIT_FLAG_QK_FP8) leave in each output
element -- test-side statistics, not an oracle: nothing here produces an expected VALUE, only the scale an
error may have, derived from the operand format alone.

The format (a reading of this repository, the paper has no 8-bit path): q' = rope(q) * scale * log2(e) and
k' = rope(k) are rounded per ROW: the row is multiplied by the power of two that brings its largest magnitude
into [128, 256), rounded to nearest-even E4M3 (3 stored mantissa bits, normal numbers down to 2^-6, below
that a fixed step of 2^-9), and the power of two is undone inside the matrix instruction.

Propagation, first order, rounding errors independent and uniform within half a step:
  * an operand x carries an error of variance step(x)^2 / 12, step(x) = spacing of E4M3 at x (after the row factor);
  * a base-2 score t_nj = sum_c q'_nc k'_jc carries
        var(t_nj) = sum_c ( step(q'_nc)^2 k'_jc^2 + q'_nc^2 step(k'_jc)^2 ) / 12;
  * an output element moves by  sum_j p_nj (v_jc - o_nc) ln2 dt_nj,  so, taking the score errors of
    different keys of one row as uncorrelated (the q-side errors are shared between keys, but their cross
    terms carry the random signs of k'_jc k'_j'c and vanish on average),
        var(o_nc) = ln2^2 sum_j p_nj^2 var(t_nj) (v_jc - o_nc)^2.
The tests check both that the measured errors HAVE this size (their RMS, element by element normalised, is
close to 1: the 8-bit path ran, and nothing else adds error) and that none exceeds it by more than a
Gaussian tail allows for the number of elements compared.
"""
import numpy as np

import oracle

LN2 = float(np.log(2.0))
LOG2E = float(np.log2(np.e))


def e4m3_step(x):
    """Spacing of the E4M3 grid at each element of x once its row (last axis) has been multiplied by the power
    of two that brings the row's largest magnitude into [128, 256); returned in x's own units."""
    x = np.abs(np.asarray(x, dtype=np.float64))
    amax = x.max(axis=-1, keepdims=True)
    _, ex = np.frexp(amax)                       # amax in [2^(ex-1), 2^ex)
    row_e = np.where(amax > 0, 8 - ex, 0)        # amax * 2^row_e in [128, 256)
    xs = np.ldexp(x, row_e)
    _, e = np.frexp(np.maximum(xs, 2.0 ** -6))   # xs in [2^(e-1), 2^e), clamped into the normal range
    return np.ldexp(1.0, (e - 1 - 3) - row_e)


def predicted_std(qr, kr, v, scale, rows=None, chunk=1024, want_lse=False):
    """One (sequence, head): qr [L, D] and kr [Lk, D] are the rotated (and, where used, normalised) q and k in
    float64, v [Lk, D].  Returns the predicted standard deviation of the error of out[rows, :] ([len(rows), D]);
    with want_lse also that of the rows' log-sum-exp ([len(rows)])."""
    qp = np.asarray(qr, dtype=np.float64) * (scale * LOG2E)
    kp = np.asarray(kr, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    if rows is not None:
        qp = qp[rows]
    sq2, sk2 = e4m3_step(qp) ** 2 / 12.0, e4m3_step(kp) ** 2 / 12.0
    out = np.empty((qp.shape[0], v.shape[1]))
    lse = np.empty(qp.shape[0])
    v2 = v * v
    for i in range(0, qp.shape[0], chunk):
        t = qp[i:i + chunk] @ kp.T
        p = np.exp2(t - t.max(axis=1, keepdims=True))
        p /= p.sum(axis=1, keepdims=True)
        o = p @ v
        wk = p * p * ((qp[i:i + chunk] ** 2) @ sk2.T)          # k-side rounding: independent from key to key
        w = wk + p * p * (sq2[i:i + chunk] @ (kp * kp).T)      # + q-side, keys taken as uncorrelated
        var = w @ v2 - 2.0 * o * (w @ v) + o * o * w.sum(axis=1, keepdims=True)
        out[i:i + chunk] = LN2 * np.sqrt(np.maximum(var, 0.0))
        # The log-sum-exp moves by sum_j p_nj ln2 dt_nj.  Here the q-side errors of a row do NOT average out
        # over its keys (for the outputs they do, because sum_j p_nj (v_jc - o_nc) = 0): the channel-c error of
        # q'_n multiplies the p-weighted mean key sum_j p_nj k'_jc, which points along q'_n.  Exact q-side term:
        kbar = p @ kp
        lse[i:i + chunk] = LN2 * np.sqrt(wk.sum(axis=1) + (sq2[i:i + chunk] * kbar * kbar).sum(axis=1))
    return (out, lse) if want_lse else out


def predicted_std_self(q, k, v, grid, split, origin=(0, 0, 0), base=10000.0, scale=0.0, rows=None,
                       q_rot_in=None, k_rot_in=None, want_lse=False):
    """[B, L, H, D] inputs of a self-attention call -> predicted error std of out[:, rows] ([B, n, H, D]);
    with want_lse also of lse[:, :, rows] ([B, H, n]).
    q_rot_in / k_rot_in: float64 arrays to rotate instead of q / k (normalised q and k)."""
    qf = oracle.as_f64(q) if q_rot_in is None else q_rot_in
    kf = oracle.as_f64(k) if k_rot_in is None else k_rot_in
    vf = oracle.as_f64(v)
    B, L, H, D = qf.shape
    if scale <= 0:
        scale = 1.0 / np.sqrt(D)
    pos = oracle.token_positions(grid, origin)
    n = L if rows is None else len(rows)
    out = np.empty((B, n, H, D))
    lse = np.empty((B, H, n))
    for b in range(B):
        for h in range(H):
            out[b, :, h], lse[b, h] = predicted_std(oracle.rope3d(qf[b, :, h], pos, split, base),
                                                    oracle.rope3d(kf[b, :, h], pos, split, base), vf[b, :, h], scale,
                                                    rows, want_lse=True)
    return (out, lse) if want_lse else out


def gaussian_tail_z(n_elements, expected_exceedances=1e-2):
    """z such that n independent standard normal values hold about `expected_exceedances` beyond +-z."""
    from scipy.stats import norm

    return float(norm.isf(expected_exceedances / (2.0 * n_elements)))
