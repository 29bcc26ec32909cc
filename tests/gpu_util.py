"""Helpers for the GPU parity tests."""
import numpy as np

from paper_2207_08393_amd.runner import ModuleRunner, SenseRunner  # noqa: F401


def rel_l2(a, b):
    a = np.asarray(a).astype(np.complex128 if np.iscomplexobj(a) else np.float64)
    b = np.asarray(b).astype(a.dtype)
    return float(np.linalg.norm((a - b).ravel()) / max(np.linalg.norm(b.ravel()), 1e-300))


def run_sense_normal(geom, x, S, M):
    r = SenseRunner(geom, x, S, M)
    r.run()
    return r.result()
