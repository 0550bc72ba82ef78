"""Helpers shared by the GPU parity tests."""
import numpy as np

# tolerance of the path: max_i |gpu_i - oracle_i| / max_i |oracle_i| per tensor
TOL = {"fp32": 1e-5, "bf16": 2e-2}


def rel_err(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.all(np.isfinite(got)), "non-finite values in the GPU result"
    den = np.abs(ref).max()
    return float(np.abs(got - ref).max() / (den if den > 0 else 1.0))


def to_dev(a, bf16):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return t.to(torch.bfloat16) if bf16 else t


def to_host(t):
    return t.detach().float().cpu().numpy()
