"""GPU parity: the HIP library (through its C ABI) against the CPU oracle,
element by element on the same seeded inputs.

Tolerances:
  j                       exact
  theta_new               relative L2 <= 1e-5 (fp32 storage), <= 1e-3 (bf16 storage),
                          and element by element |got - want| <= 2 tol max|want|
internal, stricter than the headline needs:
  C, w                    Frobenius / L2 relative <= 1e-5
  c                       relative L2 <= 1e-4
  correction (Theta-G)c   relative L2 <= 1e-4
"""
import numpy as np
import pytest
import torch

import oracle
import paper_1709_05069_amd as qn
from paper_1709_05069_amd import synth
from parity_util import rel, assert_close

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def gen(name, n, m=None):
    wl = synth.WORKLOADS[name].scaled(n)
    if m is not None:
        from dataclasses import replace
        wl = replace(wl, m=m)
    th, gr = synth.make_worker_states(wl, DEV)
    return wl, th, gr, synth.to_numpy_stored(th), synth.to_numpy_stored(gr)


def oracle_full(th_np, gr_np, tau, lam):
    n = th_np.shape[1]
    if n * th_np.shape[0] <= 2_000_000:
        lit = oracle.update_literal(th_np, gr_np, tau, lam)
    else:
        lit = None
    st = oracle.update_streaming(th_np, gr_np, tau, lam)
    if lit is not None:   # the two oracle modes agree before either is used
        assert lit["j"] == st["j"]
        assert rel(lit["theta_new"], st["theta_new"]) <= 1e-11
    return st


# ----------------------------------------------------------------- Gram ----
GRAM_CASES = [
    ("tiny_exact", 4096, 4), ("tiny_exact", 1, 2), ("tiny_exact", 130, 1),
    ("small_mlp", 777, 3), ("small_mlp", 5000, 8), ("small_mlp", 127, 15),
    ("resnet50", 100003, 16), ("resnet50", 66001, 17), ("gpt2_small", 200000, 32),
    ("gpt2_small", 129, 32), ("gpt2_small", 50001, 31), ("stress_1b_bf16", 70000, 32),
    ("stress_1b_bf16", 4097, 8), ("stress_1b_bf16", 33333, 20),
    # more than 32 workers: the 4x4 tiling
    ("gpt2_small", 60000, 64), ("gpt2_small", 30001, 33), ("resnet50", 20480, 48),
    ("stress_1b_bf16", 40000, 64), ("stress_1b_bf16", 20003, 47),
    ("gpt2_small", 20001, 64), ("stress_1b_bf16", 10001, 64),      # unaligned columns, four sets
    # few workers at larger n: row blocks packed side by side in the column lanes
    ("gpt2_small", 100_000, 8), ("gpt2_small", 70_001, 4), ("gpt2_small", 50_000, 2),
    ("gpt2_small", 30_000, 5), ("stress_1b_bf16", 50_000, 5), ("stress_1b_bf16", 40_001, 3),
    ("stress_1b_bf16", 65_536, 8),
]


@pytest.mark.parametrize("name,n,m", GRAM_CASES)
def test_gram_matches_oracle(name, n, m):
    wl, th, gr, th_np, gr_np = gen(name, n, m)
    C, w = qn.qn_gram(gr)
    torch.cuda.synchronize()
    Co, wo = oracle.gram_accumulate(gr_np)
    C, w = C.cpu().numpy(), w.cpu().numpy()
    if m == 1:
        assert np.all(C == 0) and np.all(w == 0) and np.all(Co == 0)
        return
    assert rel(C, Co) <= 1e-5
    assert rel(w, wo) <= 1e-5
    assert np.array_equal(C, C.T)
    assert np.abs(C.sum(0)).max() <= 1e-9 * np.abs(C).max()      # G 1 = 0


def test_gram_unaligned_columns_and_leading_dimension():
    # odd n with ld = n: columns 1.. are not 16-byte aligned (element-wise path);
    # a row shard of a wider matrix: ld > n, base offset by 5 rows
    wl, th, gr, th_np, gr_np = gen("resnet50", 30001, 16)
    C, w = qn.qn_gram(gr)
    Co, wo = oracle.gram_accumulate(gr_np)
    assert rel(C.cpu().numpy(), Co) <= 1e-5 and rel(w.cpu().numpy(), wo) <= 1e-5
    for r0, rows in ((5, 20000), (8, 16384), (0, 127)):
        Cs, ws = qn.qn_gram(gr[:, r0:r0 + rows])
        Cso, wso = oracle.gram_accumulate(gr_np[:, r0:r0 + rows])
        assert rel(Cs.cpu().numpy(), Cso) <= 1e-5
        assert rel(ws.cpu().numpy(), wso) <= 1e-5


def test_gram_is_additive_over_row_shards():
    # centring is per row, so C and w of the whole are the sums over row shards
    wl, th, gr, _, _ = gen("gpt2_small", 300000, 32)
    C, w = qn.qn_gram(gr)
    Cs = torch.zeros_like(C)
    ws = torch.zeros_like(w)
    for r0 in range(0, 300000, 75008):
        c1, w1 = qn.qn_gram(gr[:, r0:r0 + 75008])
        Cs += c1
        ws += w1
    assert rel(Cs.cpu().numpy(), C.cpu().numpy()) <= 1e-6
    assert rel(ws.cpu().numpy(), w.cpu().numpy()) <= 1e-6


# ------------------------------------------------------------------ eig ----
def _engineered_C(m, svals, seed):
    rng = np.random.default_rng(seed)
    M = rng.standard_normal((m, m))
    M[:, 0] = 1.0
    Q, _ = np.linalg.qr(M)
    W = Q[:, 1:]
    s = np.asarray(svals, float)
    C = (W * s ** 2) @ W.T
    w = W @ (rng.standard_normal(m - 1) * s)
    return C, w


@pytest.mark.parametrize("m,lam", [(2, 0.5), (3, 0.3), (4, 0.5), (7, 0.2), (8, 0.6),
                                   (16, 0.35), (17, 0.9), (31, 0.05), (32, 0.5),
                                   (32, 1e-3), (32, 1.5), (24, 0.1), (25, 0.1), (33, 0.3), (40, 0.2), (48, 0.05), (49, 0.1),
                                   (64, 0.5), (64, 1e-3)])
def test_eig_select_matches_oracle_on_engineered_spectra(m, lam):
    svals = np.geomspace(1.0, 0.02, m - 1) * 3.7
    C, w = _engineered_C(m, svals, 40 + m)
    ref = oracle.coefficients(C, w, np.float32(lam))
    Cd = torch.tensor(C, device=DEV)
    wd = torch.tensor(w, device=DEV)
    sigma, V, c, j = qn.qn_eig(Cd, wd, lam)
    torch.cuda.synchronize()
    sigma, V, c, j = sigma.cpu().numpy(), V.cpu().numpy(), c.cpu().numpy(), int(j.item())
    # the cutoff margin of this case is wide, so "same j" is well posed
    margin = np.min(np.abs(ref["sigma"][:m - 1] / ref["sigma"][0] - lam))
    assert margin > 1e-6
    assert j == ref["j"]
    assert 0 <= j <= m - 1
    assert np.abs(sigma[:m - 1] - ref["sigma"][:m - 1]).max() <= 1e-11 * ref["sigma"][0]
    assert sigma[m - 1] <= 1e-6 * sigma[0]
    assert np.all(np.diff(sigma) <= 0)
    Vc = V.T
    assert np.abs(Vc.T @ Vc - np.eye(m)).max() <= 1e-12
    assert np.abs(C @ Vc - Vc * sigma ** 2).max() <= 1e-12 * sigma[0] ** 2
    if j > 0:
        assert rel(c, ref["c"]) <= 1e-6
        assert abs(c.sum()) <= 1e-6 * np.abs(c).max()
    else:
        assert np.all(c == 0)


def test_eig_degenerate_inputs():
    m = 8
    z = torch.zeros((m, m), dtype=torch.float64, device=DEV)
    zw = torch.zeros(m, dtype=torch.float64, device=DEV)
    sigma, V, c, j = qn.qn_eig(z, zw, 0.1)
    assert int(j.item()) == 0 and torch.all(c == 0) and torch.all(sigma == 0)
    bad = z.clone()
    bad[2, 3] = float("nan")
    sigma, V, c, j = qn.qn_eig(bad, zw, 0.1)
    assert int(j.item()) == -1 and torch.all(c == 0)
    one = torch.zeros((1, 1), dtype=torch.float64, device=DEV)
    sigma, V, c, j = qn.qn_eig(one, zw[:1].contiguous(), 0.1)
    assert int(j.item()) == 0 and float(c[0]) == 0.0


# ---------------------------------------------------------------- apply ----
APPLY_CASES = [
    ("tiny_exact", 4096, 4), ("tiny_exact", 3, 2), ("small_mlp", 1001, 8),
    ("small_mlp", 70001, 5), ("resnet50", 100000, 16), ("gpt2_small", 65537, 32),
    ("gpt2_small", 40000, 1), ("stress_1b_bf16", 50000, 32),
    ("stress_1b_bf16", 12345, 8), ("stress_1b_bf16", 8200, 23),
    ("gpt2_small", 30000, 64), ("gpt2_small", 10001, 40), ("stress_1b_bf16", 16008, 64),
    # the direct kernel with its capped grid (several row groups per thread)
    ("small_mlp", 3_000_001, 8), ("stress_1b_bf16", 5_000_003, 4),
]


@pytest.mark.parametrize("name,n,m", APPLY_CASES)
def test_apply_matches_oracle(name, n, m):
    wl, th, gr, th_np, gr_np = gen(name, n, m)
    rng = np.random.default_rng(n + m)
    c = rng.standard_normal(m).astype(np.float32)       # arbitrary, not centred
    out = qn.qn_apply(th, gr, torch.tensor(c, device=DEV), wl.tau)
    torch.cuda.synchronize()
    ref = oracle.apply_closed_form(th_np, gr_np, c.astype(np.float64), wl.tau)
    assert_close(out.cpu().numpy(), ref, 2e-6, k=4.0)
    # the correction alone (difference to the SGD form) is also right
    sgd = oracle.apply_closed_form(th_np, gr_np, np.zeros(m), wl.tau)
    if m > 1:
        # bf16 storage sums the stored values in fp32 (no pivot differences): the
        # correction on its own is good to the storage type's 1e-3, not to 1e-4
        tol = 1e-4 if wl.storage == "f32" else 1e-3
        assert rel(out.cpu().numpy().astype(np.float64) - sgd, ref - sgd) <= tol


def test_apply_shards_and_unaligned():
    wl, th, gr, th_np, gr_np = gen("resnet50", 40003, 16)
    c = np.linspace(-1, 1, 16).astype(np.float32)
    cd = torch.tensor(c, device=DEV)
    ref = oracle.apply_closed_form(th_np, gr_np, c.astype(np.float64), 0.7)
    out = qn.qn_apply(th, gr, cd, 0.7)                   # odd n: element-wise path
    assert_close(out.cpu().numpy(), ref, 2e-6, k=4.0)
    for r0, rows in ((3, 30000), (4, 1025), (16, 16)):
        o = qn.qn_apply(th[:, r0:r0 + rows], gr[:, r0:r0 + rows], cd, 0.7)
        assert_close(o.cpu().numpy(), ref[r0:r0 + rows], 2e-6, k=4.0)


# ----------------------------------------------------------- whole step ----
UPDATE_CASES = [
    ("tiny_exact", 4096, None),           # configs[0] at full size
    ("small_mlp", 1_200_000, None),       # configs[1] at full size
    ("resnet50", 300_001, None), ("gpt2_small", 250_000, None),
    ("stress_1b_bf16", 200_000, None), ("small_mlp", 50_000, 3),
    ("gpt2_small", 10_000, 27), ("gpt2_small", 50_000, 64), ("stress_1b_bf16", 30_000, 48),
    ("resnet50", 20_000, 33),
]


@pytest.mark.parametrize("name,n,m", UPDATE_CASES)
def test_update_matches_oracle(name, n, m):
    wl, th, gr, th_np, gr_np = gen(name, n, m)
    ref = oracle_full(th_np, gr_np, wl.tau, np.float32(wl.lam))
    out, j = qn.qn_update(th, gr, wl.tau, wl.lam)
    torch.cuda.synchronize()
    out = out.cpu().numpy()
    assert int(j.item()) == ref["j"] == wl.m - 1
    tol = 1e-5 if wl.storage == "f32" else 1e-3
    assert_close(out, ref["theta_new"], tol)
    # internal parity of the pieces
    C, w = qn.qn_gram(gr)
    sigma, V, c, j2 = qn.qn_eig(C, w, wl.lam)
    assert int(j2.item()) == ref["j"]
    assert rel(C.cpu().numpy(), ref["C"]) <= 1e-5
    assert rel(w.cpu().numpy(), ref["w"]) <= 1e-5
    assert rel(c.cpu().numpy(), ref["c"]) <= 1e-4
    sgd = oracle.apply_closed_form(th_np, gr_np, np.zeros(wl.m), wl.tau)
    assert rel(out.astype(np.float64) - sgd, ref["theta_new"] - sgd) <= 1e-4
    # composing the three entry points gives the fused step: the same bits with
    # 16-bit storage; with fp32 storage qn_update hands the apply pass c in double
    # where the pieces pass its fp32 rounding, so to fp32 rounding of the result
    out2 = qn.qn_apply(th, gr, c, wl.tau)
    if wl.storage == "f32":
        assert_close(out2.cpu().numpy(), out, 2e-7, k=8.0)
    else:
        assert torch.equal(out2.cpu(), torch.from_numpy(out))


def test_update_is_bitwise_reproducible():
    wl, th, gr, _, _ = gen("gpt2_small", 500_000)
    a, ja = qn.qn_update(th, gr, wl.tau, wl.lam)
    b, jb = qn.qn_update(th, gr, wl.tau, wl.lam)
    torch.cuda.synchronize()
    assert torch.equal(a, b) and int(ja.item()) == int(jb.item())


def test_update_j0_cases_are_averaged_sgd():
    wl, th, gr, th_np, gr_np = gen("small_mlp", 20_000)
    sgd = oracle.apply_closed_form(th_np, gr_np, np.zeros(wl.m), wl.tau)
    out, j = qn.qn_update(th, gr, wl.tau, 1.5)            # lambda > 1
    assert int(j.item()) == 0 and rel(out.cpu().numpy(), sgd) <= 1e-6
    same = gr[:1].repeat(wl.m, 1).contiguous()            # identical gradients
    out, j = qn.qn_update(th, same, wl.tau, wl.lam)
    ref = oracle.update_streaming(th_np, synth.to_numpy_stored(same), wl.tau, wl.lam)
    assert int(j.item()) == 0 == ref["j"]
    assert rel(out.cpu().numpy(), ref["theta_new"]) <= 1e-6
    out, j = qn.qn_update(th[:1], gr[:1], wl.tau, wl.lam)  # one worker
    assert int(j.item()) == 0
    assert rel(out.cpu().numpy(), th_np[0].astype(np.float64)
               - wl.tau * gr_np[0].astype(np.float64)) <= 1e-6


def test_update_nonfinite_input_reports_minus_one():
    wl, th, gr, th_np, gr_np = gen("small_mlp", 10_000)
    gr = gr.clone()
    gr[3, 77] = float("inf")
    out, j = qn.qn_update(th, gr, wl.tau, wl.lam)
    torch.cuda.synchronize()
    assert int(j.item()) == -1
    o = out.cpu().numpy()
    ok = np.ones(10_000, bool)
    ok[77] = False
    gr_np = synth.to_numpy_stored(gr)
    sgd = oracle.apply_closed_form(th_np[:, ok], gr_np[:, ok], np.zeros(wl.m), wl.tau)
    assert rel(o[ok], sgd) <= 1e-6 and not np.isfinite(o[77])


def test_cutoff_below_full_rank_on_engineered_workers():
    # worker deviations confined to a few directions with a geometric spectrum:
    # exercises j < m - 1 through the whole pipeline
    rng = np.random.default_rng(9)
    n, m = 60_000, 16
    U, _ = np.linalg.qr(rng.standard_normal((n, m - 1)))
    M = rng.standard_normal((m, m))
    M[:, 0] = 1.0
    W = np.linalg.qr(M)[0][:, 1:]
    s = 2.0 * 0.6 ** np.arange(m - 1)
    G = (U * s) @ W.T
    grads = (G + rng.standard_normal(n)[:, None]).T.astype(np.float32)
    thetas = (rng.standard_normal(n)[None, :]
              + 1e-2 * rng.standard_normal((m, n))).astype(np.float32)
    thetas, grads = np.ascontiguousarray(thetas), np.ascontiguousarray(grads)
    for lam, tau in ((0.5, 1.0), (0.1, 0.3), (0.012, 1.0)):
        ref = oracle.update_streaming(thetas, grads, tau, np.float32(lam))
        assert 0 < ref["j"] < m - 1
        out, j = qn.qn_update(torch.tensor(thetas, device=DEV),
                              torch.tensor(grads, device=DEV), tau, lam)
        assert int(j.item()) == ref["j"]
        assert_close(out.cpu().numpy(), ref["theta_new"], 1e-5)


# ------------------------------------------------ harder inputs, fused path ----
def _engineered_states(n, m, svals, seed, g_offset=0.0, g_scale=1.0):
    """Worker states whose centred gradient matrix has the given singular values
    (times g_scale), on top of a common gradient g_offset + N(0,1)."""
    rng = np.random.default_rng(seed)
    U, _ = np.linalg.qr(rng.standard_normal((n, m - 1)))
    M = rng.standard_normal((m, m))
    M[:, 0] = 1.0
    W = np.linalg.qr(M)[0][:, 1:]
    G = (U * np.asarray(svals)) @ W.T
    grads = ((G + rng.standard_normal(n)[:, None] + g_offset) * g_scale).T.astype(np.float32)
    thetas = (rng.standard_normal(n)[None, :] + 0.05 * rng.standard_normal((m, n))).astype(np.float32)
    return np.ascontiguousarray(thetas), np.ascontiguousarray(grads)


@pytest.mark.parametrize("m,lam,expect_j", [(32, 0.5, 6), (32, 0.1, 18), (32, 0.03, 27),
                                            (64, 0.25, 22), (12, 0.3, 4)])
def test_update_cutoff_inside_the_fused_step(m, lam, expect_j):
    # geometric spectrum: the cutoff falls strictly inside it, so the fused step
    # (raw accumulators -> eigen kernel -> apply) has to drop directions
    n = 40_000
    svals = 3.0 * np.geomspace(1.0, 0.02, m - 1)
    thetas, grads = _engineered_states(n, m, svals, 100 + m)
    ref = oracle_full(thetas, grads, 0.8, np.float32(lam))
    assert ref["j"] == expect_j
    margin = np.min(np.abs(ref["sigma"][:m - 1] / ref["sigma"][0] - np.float32(lam)))
    assert margin > 1e-4
    th, gr = torch.tensor(thetas, device=DEV), torch.tensor(grads, device=DEV)
    out, j = qn.qn_update(th, gr, 0.8, lam)
    assert int(j.item()) == expect_j
    assert_close(out.cpu().numpy(), ref["theta_new"], 1e-5)
    # the step on its own; the coefficient along v_k carries ~1e-7 (sigma_1/sigma_k)^2
    tb = oracle.row_means(thetas)
    amp = (ref["sigma"][0] / ref["sigma"][expect_j - 1]) ** 2
    assert rel(out.cpu().numpy().astype(np.float64) - tb, ref["theta_new"] - tb) <= 1e-6 * max(amp, 10.0)


@pytest.mark.parametrize("g_offset,g_scale", [(1e3, 1.0), (0.0, 1e-12), (0.0, 1e12), (50.0, 1e-6)])
def test_update_with_large_common_gradient_and_extreme_scales(g_offset, g_scale):
    # a common gradient a million times the centred part (the raw Gram would lose
    # everything; the pivot-shifted one must not), and gradient scales whose
    # squares are still inside the fp32 range
    n, m = 30_000, 16
    svals = 1e-3 * np.geomspace(1.0, 0.2, m - 1) * np.sqrt(n)
    thetas, grads = _engineered_states(n, m, svals, 7, g_offset, g_scale)
    ref = oracle_full(thetas, grads, 1e-3 / g_scale, np.float32(0.05))
    assert ref["j"] == m - 1
    th, gr = torch.tensor(thetas, device=DEV), torch.tensor(grads, device=DEV)
    C, w = qn.qn_gram(gr)
    assert rel(C.cpu().numpy(), ref["C"]) <= 1e-5 and rel(w.cpu().numpy(), ref["w"]) <= 1e-5
    out, j = qn.qn_update(th, gr, 1e-3 / g_scale, 0.05)
    assert int(j.item()) == m - 1
    assert_close(out.cpu().numpy(), ref["theta_new"], 1e-5)


def test_gradient_magnitudes_outside_the_fp32_range_of_their_squares():
    # documented in qn.h: centred entries below ~1e-19 underflow in the Gram pass
    # (j = 0: averaged SGD), above ~1e19 they overflow (j = -1: c = 0, the SGD form)
    n, m = 20_000, 8
    svals = np.geomspace(1.0, 0.3, m - 1) * np.sqrt(n)
    for scale, want_j in ((1e-25, 0), (1e25, -1)):
        thetas, grads = _engineered_states(n, m, svals, 3, 0.0, scale)
        th, gr = torch.tensor(thetas, device=DEV), torch.tensor(grads, device=DEV)
        tau = 1e-3 / scale
        out, j = qn.qn_update(th, gr, tau, 0.05)
        assert int(j.item()) == want_j
        sgd = oracle.apply_closed_form(thetas, grads, np.zeros(m), np.float32(tau))
        assert rel(out.cpu().numpy(), sgd) <= 2e-6
