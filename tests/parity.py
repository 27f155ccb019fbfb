"""Acceptance rules shared by the GPU parity tests (comparison only, no method arithmetic)."""
import numpy as np

EPS0 = float(np.float32(2.1))   # the library stores eps0 as fp32; the oracle is given the same value


def sqdist(Xr, Y, idx):
    diff = np.asarray(Xr, dtype=np.float64) - np.asarray(Y, dtype=np.float64)[idx]
    return np.einsum("ij,ij->i", diff, diff)


def check_assignment(a_gpu, a_ref, Xr, Y, min_agree=0.999, gap=1e-4):
    """>= 99.9 % of the assignments agree, and wherever they differ the two centroids are a
    near-tie for that point: their fp64 distances differ by at most 1e-4 relative."""
    a_gpu = np.asarray(a_gpu)
    a_ref = np.asarray(a_ref)
    assert a_gpu.shape == a_ref.shape
    diff = np.nonzero(a_gpu != a_ref)[0]
    agree = 1.0 - len(diff) / max(len(a_ref), 1)
    assert agree >= min_agree, f"agreement {agree:.6f} < {min_agree}"
    if len(diff):
        Xd = np.asarray(Xr, dtype=np.float64)[diff]
        dg = sqdist(Xd, Y, a_gpu[diff])
        dr = sqdist(Xd, Y, a_ref[diff])
        rel = np.abs(dg - dr) / np.maximum(np.minimum(dg, dr), 1e-300)
        assert rel.max() <= gap, f"disagreement that is no near-tie: rel gap {rel.max():.3e} at point {diff[rel.argmax()]}"
    return agree


def rel_l2(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))
