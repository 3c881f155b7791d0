"""Helpers shared by the GPU parity tests."""
import numpy as np


def rel_l2(got, ref):
    ref = np.asarray(ref, dtype=np.float64).ravel()
    got = np.asarray(got, dtype=np.float64).ravel()
    return float(np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-30))


def tol_for(cfg):
    """BASELINE tolerance: relative error 2e-2 with bf16 inputs, 1e-5 for the fp32 workload."""
    return 2e-2 if cfg.dtype == "bf16" else 1e-5


def sample_masks(N, rng, extra=()):
    """All-ones, a few single tensors, random dense and sparse masks (never empty)."""
    masks = [np.ones(N, dtype=np.uint8)]
    for j in sorted(set([0, 1, 2, 3, N // 2, N - 4, N - 2, N - 1]) | set(extra)):
        m = np.zeros(N, dtype=np.uint8)
        m[j] = 1
        masks.append(m)
    for p in (0.1, 0.5, 0.9):
        m = (rng.random(N) < p).astype(np.uint8)
        if not m.any():
            m[rng.integers(0, N)] = 1
        masks.append(m)
    return masks
