"""Helpers shared by the GPU parity tests: error measures against the oracle and
the tolerance the library documents for a whole step (include/qn.h, "Accuracy")."""
import numpy as np

import oracle

EPS_C_STREAM = 2e-7      # Gram matrix of the matrix-core streaming pass (n > 16384)
EPS_C_SMALL = 1e-14      # fp64 vector kernel (n <= 16384)
GRAM_SMALL_ROWS = 16384


def rel(a, b):
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    d = np.linalg.norm(a - b)
    s = np.linalg.norm(b)
    return d / s if s > 0 else d


def assert_close(got, want, tol, k=2.0, what=""):
    """Relative L2 <= tol and, element by element, |got - want| <= k tol max|want|
    (one wrong row among 1e8 moves the norm by nothing, but not the maximum)."""
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    r = rel(got, want)
    assert r <= tol, f"{what} relative L2 {r:.3e} > {tol:.1e}"
    scale = np.abs(want).max() if want.size else 0.0
    worst = np.abs(got - want).max() if want.size else 0.0
    assert worst <= k * tol * scale, (f"{what} max |got - want| = {worst:.3e} at "
                                      f"{int(np.abs(got - want).argmax())} > {k * tol * scale:.3e}")


def step_tolerance(ref, th_np, gr_np, tau, base):
    """base + the first-order bound of qn.h on what the rounding of the Gram matrix
    does to theta_new, relative to ||theta_new||; every quantity is the oracle's:
        tau eps_C (1 + max_{k<=j} ||Theta v_k|| / sigma_k) (sigma_1^2 ||c|| + ||w||) / sigma_j
    """
    j = int(ref["j"])
    norm = np.linalg.norm(ref["theta_new"])
    if j <= 0 or norm == 0:
        return base
    n = th_np.shape[1]
    eps = EPS_C_SMALL if n <= GRAM_SMALL_ROWS else EPS_C_STREAM
    sig = np.asarray(ref["sigma"], np.float64)
    V = np.asarray(ref["V"], np.float64)            # V[k] = v_k
    Ct, _ = oracle.gram_accumulate(th_np)           # Theta^T Theta
    gain = max(np.sqrt(max(V[k] @ Ct @ V[k], 0.0)) / sig[k] for k in range(j))
    amp = (1.0 + gain) * (sig[0] ** 2 * np.linalg.norm(ref["c"]) + np.linalg.norm(ref["w"])) / sig[j - 1]
    return base + abs(tau) * eps * amp / norm
