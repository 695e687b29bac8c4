"""GPU parity for the step size capped by 1 / sigma_max (Section 3, closing
discussion): qn_tau_bound and qn_update_bounded against the oracle's two
readings of the estimate."""
from dataclasses import replace

import numpy as np
import pytest
import torch

import oracle
import paper_1709_05069_amd as qn
from paper_1709_05069_amd import synth
from parity_util import assert_close

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
MODES = [qn.BOUND_SIGMA1, qn.BOUND_SECANT]


def rel(a, b):
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    return np.linalg.norm(a - b) / np.linalg.norm(b)


def oracle_bounded(th_np, gr_np, tau, lam, mode):
    """The oracle's step with the capped tau, through its chunked forms."""
    m, n = th_np.shape
    C, w = oracle.gram_accumulate(gr_np)
    co = oracle.coefficients(C, w, lam)
    Ct, _ = oracle.gram_accumulate(th_np)
    t_eff, smax = oracle.tau_bounded_from_gram(tau, mode, Ct, co["sigma"], co["V"], co["j"])
    if n * m <= 2_000_000:    # the two oracle forms agree before either is used
        tb, gb = oracle.row_means(th_np), oracle.row_means(gr_np)
        Theta, G = oracle.centre(th_np, tb), oracle.centre(gr_np, gb)
        t_lit, s_lit = oracle.tau_bounded_literal(tau, mode, Theta, G, co["sigma"], co["V"], co["j"])
        assert abs(t_lit - t_eff) <= 1e-9 * abs(t_eff) and abs(s_lit - smax) <= 1e-9 * smax
    theta_new = oracle.apply_closed_form(th_np, gr_np, co["c"], t_eff)
    return theta_new, co["j"], t_eff, smax


CASES = [("tiny_exact", 4096, None), ("small_mlp", 60_000, None), ("resnet50", 50_001, None),
         ("gpt2_small", 40_000, None), ("gpt2_small", 12_000, 48), ("stress_1b_bf16", 40_000, None)]


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("name,n,m", CASES)
def test_update_bounded_matches_oracle(name, n, m, mode):
    wl = synth.WORKLOADS[name].scaled(n)
    if m is not None:
        wl = replace(wl, m=m)
    th, gr = synth.make_worker_states(wl, DEV)
    th_np, gr_np = synth.to_numpy_stored(th), synth.to_numpy_stored(gr)
    lam = float(np.float32(wl.lam))
    tol = 1e-5 if wl.storage == "f32" else 1e-3
    seen = set()
    for tau in (1e4, 1e-7):          # far above and far below any cap
        tau32 = float(np.float32(tau))
        want, j, t_eff, smax = oracle_bounded(th_np, gr_np, tau32, lam, mode)
        out, jd, td = qn.qn_update_bounded(th, gr, tau, wl.lam, mode)
        torch.cuda.synchronize()
        assert int(jd.item()) == j
        capped = t_eff < tau32
        seen.add(capped)
        if capped:
            assert abs(float(td.item()) - t_eff) <= 1e-5 * t_eff
        else:
            assert float(td.item()) == tau32          # untouched, bit for bit
        assert_close(out.cpu().numpy(), want, tol)
        if capped:   # the step theta_new - theta_bar on its own (resolvable in fp32 here)
            tb = oracle.row_means(th_np)
            assert rel(out.cpu().numpy().astype(np.float64) - tb, want - tb) <= 1e-3
    assert seen == {True, False}


def _engineered(n, m, svals, seed, spread):
    rng = np.random.default_rng(seed)
    U, _ = np.linalg.qr(rng.standard_normal((n, m - 1)))
    M = rng.standard_normal((m, m))
    M[:, 0] = 1.0
    W = np.linalg.qr(M)[0][:, 1:]
    G = (U * np.asarray(svals)) @ W.T
    grads = (G + rng.standard_normal(n)[:, None]).T.astype(np.float32)
    Y = (U * np.asarray(spread)) @ W.T                    # Theta v_k = spread_k U_k
    thetas = (Y + rng.standard_normal(n)[:, None]).T.astype(np.float32)
    return np.ascontiguousarray(thetas), np.ascontiguousarray(grads)


@pytest.mark.parametrize("lam,expect_j", [(0.6, 2), (0.2, 5), (0.01, 7)])
def test_tau_bound_piece_on_engineered_secant_quotients(lam, expect_j):
    # sigma_k = 5 * 0.7^k, ||Theta v_k|| = spread_k: the quotients are known in
    # closed form and the largest among the first j moves with the cutoff
    n, m = 20_000, 8
    svals = 5.0 * 0.7 ** np.arange(m - 1)
    spread = np.array([2.0, 4.0, 0.5, 0.25, 0.1, 0.2, 0.04])
    thetas, grads = _engineered(n, m, svals, 91, spread)
    th, gr = torch.tensor(thetas, device=DEV), torch.tensor(grads, device=DEV)
    C, w = qn.qn_gram(gr)
    Ct, _ = qn.qn_gram(th)
    sigma, V, c, j = qn.qn_eig(C, w, lam)
    assert int(j.item()) == expect_j
    quots = (svals / spread)[:expect_j]
    quot = quots.max()
    # Theta^T Theta is good to ~1e-7 of its norm (fp32 products), so a small
    # ||Theta v_k||^2 carries a relative error ~1e-7 (spread_max / spread_k)^2
    tol = 1e-6 * (spread.max() / spread[int(quots.argmax())]) ** 2
    t, smax = qn.qn_tau_bound(sigma, V, j, Ct, 100.0, qn.BOUND_SECANT)
    assert abs(float(smax.item()) - quot) <= tol * quot
    assert abs(float(t.item()) - 1.0 / quot) <= tol / quot
    t1, smax1 = qn.qn_tau_bound(sigma, V, j, None, 100.0, qn.BOUND_SIGMA1)
    assert abs(float(smax1.item()) - 5.0) <= 1e-5 and abs(float(t1.item()) - 0.2) <= 1e-6
    # the oracle on the same stored inputs
    _, j_o, t_o, s_o = oracle_bounded(thetas, grads, 100.0, float(np.float32(lam)), oracle.BOUND_SECANT)
    assert j_o == expect_j and abs(float(smax.item()) - s_o) <= tol * s_o
    assert abs(float(t.item()) - t_o) <= tol * t_o
    # below the cap tau passes through bit for bit
    t, _ = qn.qn_tau_bound(sigma, V, j, Ct, 1e-3, qn.BOUND_SECANT)
    assert float(t.item()) == float(np.float32(1e-3))


def test_bounded_degenerate_cases():
    wl = synth.WORKLOADS["small_mlp"].scaled(10_000)
    th, gr = synth.make_worker_states(wl, DEV)
    plain, _ = qn.qn_update(th, gr, 0.5, 1.5)                     # lambda > 1: j = 0
    out, j, t = qn.qn_update_bounded(th, gr, 0.5, 1.5, qn.BOUND_SECANT)
    assert int(j.item()) == 0 and float(t.item()) == 0.5 and torch.equal(out, plain)
    # sigma_1 is still an estimate at j = 0
    out, j, t = qn.qn_update_bounded(th, gr, 1e6, 1.5, qn.BOUND_SIGMA1)
    C, w = qn.qn_gram(gr)
    sigma, _, _, _ = qn.qn_eig(C, w, 1.5)
    assert int(j.item()) == 0
    assert abs(float(t.item()) - 1.0 / float(sigma[0].item())) <= 1e-6 / float(sigma[0].item())
    # a non-finite gradient: j = -1, tau untouched
    bad = gr.clone()
    bad[2, 7] = float("inf")
    for mode in MODES:
        out, j, t = qn.qn_update_bounded(th, bad, 0.5, wl.lam, mode)
        assert int(j.item()) == -1 and float(t.item()) == 0.5
    # identical thetas: ||Theta v_k|| = 0, infinite estimate, the step is theta_bar
    same = th[:1].expand_as(th).contiguous()
    out, j, t = qn.qn_update_bounded(same, gr, 0.5, wl.lam, qn.BOUND_SECANT)
    assert int(j.item()) == wl.m - 1 and float(t.item()) == 0.0
    assert torch.equal(out, same[0])
    with pytest.raises(qn.QnError):
        qn.qn_update_bounded(th, gr, 0.5, wl.lam, 3)              # unknown mode
