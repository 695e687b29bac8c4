"""GPU parity for the operator of eq. (3)/(4) on arbitrary vectors (qn_hinv and
its pieces) against the oracle's literal evaluation (explicit u_k, y_k)."""
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


def rel(a, b):
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    return np.linalg.norm(a - b) / np.linalg.norm(b)


def oracle_pieces(th_np, gr_np, lam):
    tb, gb = oracle.row_means(th_np), oracle.row_means(gr_np)
    Theta, G = oracle.centre(th_np, tb), oracle.centre(gr_np, gb)
    mu, V, _ = oracle.jacobi_eigh(oracle.gram(G))
    sigma = oracle.sigma_from_mu(mu)
    return Theta, G, sigma, V, oracle.select_j(sigma, lam), tb, gb


CASES = [("tiny_exact", 4096, None, 0.01), ("small_mlp", 30_001, None, 0.05),
         ("resnet50", 50_000, None, 0.01), ("gpt2_small", 40_000, None, 0.01),
         ("gpt2_small", 9_999, 23, 0.01), ("stress_1b_bf16", 40_000, None, 0.02),
         ("stress_1b_bf16", 12_345, 9, 0.02), ("gpt2_small", 20_000, 64, 0.01),
         ("stress_1b_bf16", 16_001, 40, 0.02)]


@pytest.mark.parametrize("name,n,m,lam", CASES)
def test_hinv_matches_literal_eq4_on_random_vectors(name, n, m, lam):
    wl = synth.WORKLOADS[name].scaled(n)
    if m is not None:
        wl = replace(wl, m=m)
    th, gr = synth.make_worker_states(wl, DEV)
    th_np, gr_np = synth.to_numpy_stored(th), synth.to_numpy_stored(gr)
    lam32 = float(np.float32(lam))
    Theta, G, sigma, V, j, tb, gb = oracle_pieces(th_np, gr_np, lam32)
    rng = np.random.default_rng(n)
    # a vector with a sizeable component inside span{u_k}: mix of G's columns
    z = (rng.standard_normal(n) * np.abs(gb).mean()
         + (rng.standard_normal(wl.m) @ G) * 3.0).astype(np.float32)
    zd = torch.tensor(z, device=DEV)
    out, jd = qn.qn_hinv(th, gr, zd, lam)
    torch.cuda.synchronize()
    ref = oracle.apply_Hinv_literal(Theta, G, sigma, V, j, z.astype(np.float64))
    assert int(jd.item()) == j
    tol = 1e-5 if wl.storage == "f32" else 1e-3
    assert_close(out.cpu().numpy(), ref, tol, k=4.0)
    # what the operator changed (out - z) is right on its own
    assert rel(out.cpu().numpy().astype(np.float64) - z, ref - z) <= 1e-4
    # G^T z
    w = qn.qn_gemv_t(gr, zd)
    assert rel(w.cpu().numpy(), oracle.gemv_t(G, z.astype(np.float64))) <= 1e-5
    # the pieces compose to the fused operator: the same bits with 16-bit storage;
    # with fp32 storage the fused call keeps c in double for the apply pass, the
    # pieces hand over its fp32 rounding
    C, wg = qn.qn_gram(gr)
    s2, V2, _, j2 = qn.qn_eig(C, wg, lam)
    c = qn.qn_coef(s2, V2, j2, w)
    out2 = qn.qn_hinv_apply(th, gr, zd, c)
    if wl.storage == "f32":
        assert_close(out2.cpu().numpy(), out.cpu().numpy(), 1e-6, k=8.0)
    else:
        assert torch.equal(out, out2)


def _engineered(n, m, svals, seed):
    rng = np.random.default_rng(seed)
    U, _ = np.linalg.qr(rng.standard_normal((n, m - 1)))
    M = rng.standard_normal((m, m))
    M[:, 0] = 1.0
    W = np.linalg.qr(M)[0][:, 1:]
    G = (U * np.asarray(svals)) @ W.T
    grads = (G + rng.standard_normal(n)[:, None]).T.astype(np.float32)
    thetas = (rng.standard_normal(n)[None, :] + (rng.standard_normal((m, m - 1)) @ U.T) * 0.7
              + 0.05 * rng.standard_normal((m, n))).astype(np.float32)
    return np.ascontiguousarray(thetas), np.ascontiguousarray(grads)


@pytest.mark.parametrize("lam,expect_j", [(0.3, 2), (0.05, 5), (1e-3, 7)])
def test_both_branches_of_eq3_on_the_gpu(lam, expect_j):
    n, m = 30_000, 8
    thetas, grads = _engineered(n, m, 5.0 * 0.5 ** np.arange(m - 1), 77)
    lam32 = float(np.float32(lam))
    Theta, G, sigma, V, j, _, _ = oracle_pieces(thetas, grads, lam32)
    assert j == expect_j
    th, gr = torch.tensor(thetas, device=DEV), torch.tensor(grads, device=DEV)
    # The Gram matrix is accurate to ~1e-7 of its norm (fp32 products), so a
    # coefficient along v_k carries a relative error ~1e-7 (sigma_1/sigma_k)^2:
    # the method's own conditioning, bounded by 1/lambda^2 through the cutoff.
    amp = (sigma[0] / sigma[j - 1]) ** 2
    for k in range(m - 1):
        z = (V[k] @ G).astype(np.float32)                       # G v_k
        out, jd = qn.qn_hinv(th, gr, torch.tensor(z, device=DEV), lam)
        got = out.cpu().numpy().astype(np.float64)
        assert int(jd.item()) == j
        want = V[k] @ Theta if k < j else z.astype(np.float64)   # Theta v_k, or untouched
        scale = np.linalg.norm(z) + np.linalg.norm(want)
        assert np.linalg.norm(got - want) <= 1e-6 * amp * scale, f"k={k}"
    # a vector orthogonal to u_1..u_j passes through unchanged
    rng = np.random.default_rng(5)
    Uj = np.stack([(V[k] @ G) / sigma[k] for k in range(j)], 1)
    z = rng.standard_normal(n)
    z -= Uj @ (Uj.T @ z)
    z32 = z.astype(np.float32)
    out, _ = qn.qn_hinv(th, gr, torch.tensor(z32, device=DEV), lam)
    assert np.linalg.norm(out.cpu().numpy() - z32) <= 1e-6 * amp * np.linalg.norm(z32)


def test_update_is_eq2_with_the_operator_applied_to_gbar():
    wl = synth.WORKLOADS["gpt2_small"].scaled(120_000)
    th, gr = synth.make_worker_states(wl, DEV)
    upd, j = qn.qn_update(th, gr, 0.7, wl.lam)
    g_bar = gr.double().mean(0).float().contiguous()          # inputs only
    theta_bar = th.double().mean(0)
    h, j2 = qn.qn_hinv(th, gr, g_bar, wl.lam)
    assert int(j.item()) == int(j2.item())
    want = (theta_bar - 0.7 * h.double()).cpu().numpy()
    assert rel(upd.cpu().numpy(), want) <= 1e-5


def test_hinv_j0_and_nonfinite():
    wl = synth.WORKLOADS["small_mlp"].scaled(10_000)
    th, gr = synth.make_worker_states(wl, DEV)
    z = torch.randn(10_000, device=DEV)
    out, j = qn.qn_hinv(th, gr, z, 1.5)                        # lambda > 1: identity
    assert int(j.item()) == 0 and torch.equal(out, z)
    bad = gr.clone()
    bad[1, 5] = float("nan")
    out, j = qn.qn_hinv(th, bad, z, wl.lam)
    assert int(j.item()) == -1
    keep = torch.ones(10_000, dtype=torch.bool, device=DEV)
    keep[5] = False
    assert torch.equal(out[keep], z[keep])


@pytest.mark.parametrize("name,n,m", [("gpt2_small", 33_000, 32), ("gpt2_small", 9_001, 64),
                                      ("stress_1b_bf16", 20_480, 32), ("stress_1b_bf16", 7_777, 12),
                                      ("small_mlp", 300, 8), ("gpt2_small", 50_000, 4),
                                      ("stress_1b_bf16", 30_000, 8), ("stress_1b_bf16", 9_000, 3)])
def test_z_at_any_alignment_gives_the_same_bits(name, n, m):
    # z rides through the Gram pass in its own LDS slot, fetched with 16-byte or
    # 4-byte direct-to-LDS loads depending on its address: same values, same bits
    wl = replace(synth.WORKLOADS[name].scaled(n), m=m)
    th, gr = synth.make_worker_states(wl, DEV)
    g = torch.Generator(device=DEV)
    g.manual_seed(n)
    buf = torch.randn(n + 3, device=DEV, generator=g)
    z0 = buf[:n].clone()
    w0 = qn.qn_gemv_t(gr, z0)
    out0, j0 = qn.qn_hinv(th, gr, z0, wl.lam)
    for off in (1, 2, 3):
        zo = torch.empty(n + 3, device=DEV)[off:off + n]
        zo.copy_(z0)
        assert zo.data_ptr() % 16 != 0
        assert torch.equal(qn.qn_gemv_t(gr, zo), w0)
        out, j = qn.qn_hinv(th, gr, zo, wl.lam)
        assert int(j.item()) == int(j0.item()) and torch.equal(out, out0)
    G = oracle.centre(synth.to_numpy_stored(gr), oracle.row_means(synth.to_numpy_stored(gr)))
    assert rel(w0.cpu().numpy(), oracle.gemv_t(G, z0.cpu().numpy().astype(np.float64))) <= 1e-5
