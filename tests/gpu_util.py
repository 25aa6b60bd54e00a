"""Helpers for the GPU parity tests: move seeded inputs to the device, run the library through
the C ABI binding, compare with the CPU fp64 oracle."""
import numpy as np

TOL = 2e-2  # max |err| <= TOL * RMS(oracle output), the parity bar for 16-bit operands


def to_dev(a):
    import torch

    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).cuda()
    return torch.from_numpy(a).cuda()


def to_f64(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def bf16_half_ulp(x):
    """Half a bf16 unit in the last place at |x| (8 significant bits)."""
    ax = np.maximum(np.abs(x), 1e-38)
    return 2.0 ** (np.floor(np.log2(ax)) - 8)


def compare(gpu, ref, bf16_out=False, tol=TOL, what=""):
    """max|gpu - ref| / RMS(ref); for bf16 outputs the final cast's half-ulp is allowed on top."""
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert gpu.shape == ref.shape, (gpu.shape, ref.shape)
    assert np.all(np.isfinite(gpu)), "%s: non-finite GPU output" % what
    rms = float(np.sqrt(np.mean(ref * ref)))
    err = np.abs(gpu - ref)
    ratio = float(err.max() / rms) if rms > 0 else float(err.max())
    print("%s: max|err|/RMS = %.3e over %d elements (RMS %.4e, bf16_out=%s)" % (what, ratio, ref.size, rms, bf16_out))
    allow = tol * rms + (bf16_half_ulp(ref) if bf16_out else 0.0)
    bad = err > allow
    assert not bad.any(), "%s: %d of %d elements beyond tolerance, max|err|/RMS = %.3e" % (
        what, int(bad.sum()), ref.size, ratio)
    return ratio
