import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (runs the HIP library)")


def rel_err(a, b):
    """(Frobenius relative error, max-abs error relative to max|b|) of a against the reference b."""
    import numpy as np
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    nb = np.linalg.norm(b)
    mb = np.abs(b).max() if b.size else 0.0
    fro = np.linalg.norm(a - b) / nb if nb > 0 else np.linalg.norm(a - b)
    mx = np.abs(a - b).max() / mb if mb > 0 else (np.abs(a - b).max() if a.size else 0.0)
    return fro, mx


def assert_close(a, b, tol, what=""):
    """Both relative measures must stay within tol: Frobenius norm of the
    difference over that of the reference, and largest absolute difference
    over the largest reference magnitude."""
    fro, mx = rel_err(a, b)
    assert fro <= tol and mx <= tol, f"{what}: fro_rel={fro:.3e} max_rel={mx:.3e} tol={tol:.1e}"
