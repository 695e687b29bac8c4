"""What Section 2 fixes about the step, checked on the GPU path directly against
closed forms (no oracle involved): on an exact quadratic whose workers span the
whole space the step is Newton's and lands on the minimiser; with curvature s*I
the step is Newton's on the span of the workers' spread and averaged SGD off it."""
import numpy as np
import pytest
import torch

import paper_1709_05069_amd as qn

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _spd(n, rng, lo=0.5, hi=4.0):
    Q, _ = np.linalg.qr(rng.standard_normal((n, n)))
    return (Q * np.linspace(lo, hi, n)) @ Q.T


def _rel(a, b):
    return np.linalg.norm(np.asarray(a, np.float64) - b) / np.linalg.norm(b)


@pytest.mark.parametrize("m", [2, 3, 4, 8, 17, 32, 33, 64])
def test_exact_quadratic_with_n_equal_m_minus_1_lands_on_the_minimiser(m):
    # J = 0.5 x^T A x - b^T x, grad_k = A theta_k - b, n = m - 1 and workers in
    # general position: G = A Theta is square and invertible on the centred
    # space, so eq. (4) gives Theta G^-1 g_bar = theta_bar - x* and eq. (2) with
    # tau = 1 gives x*; with tau = 1/4 a quarter of the way there.
    rng = np.random.default_rng(100 + m)
    n = m - 1
    A = _spd(n, rng)
    b = rng.standard_normal(n)
    th64 = rng.standard_normal(n)[None, :] + 0.3 * rng.standard_normal((m, n))
    # the stored (fp32) parameters define the problem; gradients exact for them
    th32 = th64.astype(np.float32)
    gr32 = (th32.astype(np.float64) @ A.T - b[None, :]).astype(np.float32)
    xstar = np.linalg.solve(A, b)
    th, gr = torch.tensor(th32, device=DEV), torch.tensor(gr32, device=DEV)
    tb = th32.astype(np.float64).mean(0)
    # the fp32 rounding of the gradients (2^-24 relative) is the only inexactness
    # of the secant system: its solution moves by about cond * 2^-24 * |g| / spread
    tol = 2e-4
    for tau in (1.0, 0.25):
        out, j = qn.qn_update(th, gr, tau, 1e-6)
        torch.cuda.synchronize()
        assert int(j.item()) == n
        want = tb - tau * (tb - xstar)
        assert _rel(out.cpu().numpy(), want) <= tol, (m, tau)


@pytest.mark.parametrize("n,m,storage", [(50, 5, torch.float32), (100_000, 8, torch.float32),
                                         (300_001, 32, torch.float32), (200_000, 16, torch.bfloat16)])
def test_isotropic_curvature_gives_newton_on_the_span_and_sgd_off_it(n, m, storage):
    # A = s I: G = s Theta exactly, so on span(Theta) the operator of eq. (4)
    # divides by s and elsewhere it is the identity
    rng = np.random.default_rng(21 + m)
    s, tau = 4.0, 1.0
    th = torch.tensor(rng.standard_normal(n)[None, :] + 0.1 * rng.standard_normal((m, n)),
                      dtype=storage, device=DEV)
    b = torch.tensor(rng.standard_normal(n), dtype=storage, device=DEV)
    # fp32 storage rounds s*theta - b by 2^-24, bf16 storage by 2^-9: the closed form
    # holds to the resolution of the stored gradients
    gr = (s * th.double() - b.double()).to(storage)
    gr64, th64 = gr.double().cpu().numpy(), th.double().cpu().numpy()
    tb, gb = th64.mean(0), gr64.mean(0)
    Q, _ = np.linalg.qr((th64 - tb).T)
    Q = Q[:, :m - 1]
    on = Q @ (Q.T @ gb)
    expect = tb - tau * ((gb - on) + on / s)
    out, j = qn.qn_update(th, gr, tau, 1e-6)
    torch.cuda.synchronize()
    assert int(j.item()) == m - 1
    tol = 1e-5 if storage == torch.float32 else 4e-3
    assert _rel(out.cpu().numpy(), expect) <= tol
    assert np.abs(out.cpu().numpy() - expect).max() <= 4 * tol * np.abs(expect).max()
