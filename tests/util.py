"""Helpers shared by the GPU parity tests."""
import numpy as np

# Tolerance of the path, as the stated bar defines it: max_i |gpu_i - oracle_i| / max_i |oracle_i| per
# tensor (a tensor-normalised bound, not an element-wise relative error; the oracle is fp64).
TOL = {"fp32": 1e-5, "bf16": 2e-2}
# A second measure beside it, so that an error spread over many small entries cannot hide under the
# tensor maximum: ||gpu - oracle||_2 / ||oracle||_2.  Rounding noise is about as large relative to the
# root mean square as relative to the maximum (both scale with the tensor), so it gets half the bar
# in bf16 and the same bar in fp32.
TOL_RMS = {"fp32": 1e-5, "bf16": 1e-2}


def rel_err(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.all(np.isfinite(got)), "non-finite values in the GPU result"
    den = np.abs(ref).max()
    return float(np.abs(got - ref).max() / (den if den > 0 else 1.0))


def rms_err(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    den = np.sqrt(np.mean(ref * ref))
    return float(np.sqrt(np.mean((got - ref) ** 2)) / (den if den > 0 else 1.0))


def to_dev(a, bf16):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return t.to(torch.bfloat16) if bf16 else t


def to_host(t):
    return t.detach().float().cpu().numpy()
