"""GPU parity for IEEE binary16 storage (the *_ex entry points with QN_F16):
Gram, apply, the whole step and the operator against the oracle, which widens
the same stored half-precision values exactly."""
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
TOL = 1e-4      # half precision stores 11 significant bits; the arithmetic is fp32/fp64


def rel(a, b):
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    return np.linalg.norm(a - b) / np.linalg.norm(b)


def gen(name, n, m):
    wl = replace(synth.WORKLOADS[name].scaled(n), m=m, storage="f16")
    th, gr = synth.make_worker_states(wl, DEV)
    assert th.dtype == torch.float16
    th_np, gr_np = synth.to_numpy_stored(th), synth.to_numpy_stored(gr)
    assert th_np.dtype == np.float16
    return wl, th, gr, th_np, gr_np


CASES = [("small_mlp", 60_000, 8), ("small_mlp", 4_097, 3), ("resnet50", 100_000, 16),
         ("gpt2_small", 70_000, 32), ("gpt2_small", 20_001, 32), ("gpt2_small", 513, 17),
         ("gpt2_small", 30_000, 48), ("gpt2_small", 16_384, 64), ("tiny_exact", 7, 2)]


@pytest.mark.parametrize("name,n,m", CASES)
def test_f16_gram_update_and_operator_match_the_oracle(name, n, m):
    wl, th, gr, th_np, gr_np = gen(name, n, m)
    lam = float(np.float32(wl.lam))
    C, w = qn.qn_gram(gr)
    Co, wo = oracle.gram_accumulate(gr_np)
    assert rel(C.cpu().numpy(), Co) <= 1e-5 and rel(w.cpu().numpy(), wo) <= 1e-5
    ref = oracle.update_streaming(th_np, gr_np, wl.tau, lam)
    margin = np.min(np.abs(ref["sigma"][:m - 1] / ref["sigma"][0] - lam))
    out, j = qn.qn_update(th, gr, wl.tau, wl.lam)
    if margin > 1e-5:
        assert int(j.item()) == ref["j"]
        assert_close(out.cpu().numpy(), ref["theta_new"], TOL)
    # apply with an arbitrary coefficient vector
    rng = np.random.default_rng(n + m)
    c = rng.standard_normal(m).astype(np.float32)
    got = qn.qn_apply(th, gr, torch.tensor(c, device=DEV), wl.tau)
    want = oracle.apply_closed_form(th_np, gr_np, c.astype(np.float64), wl.tau)
    assert rel(got.cpu().numpy(), want) <= 1e-5
    # the operator on a random vector
    z = torch.randn(n, device=DEV)
    h, jh = qn.qn_hinv(th, gr, z, wl.lam)
    if margin > 1e-5:
        tb, gb = oracle.row_means(th_np), oracle.row_means(gr_np)
        href = oracle.apply_Hinv_literal(oracle.centre(th_np, tb), oracle.centre(gr_np, gb),
                                         ref["sigma"], ref["V"], ref["j"],
                                         z.cpu().numpy().astype(np.float64))
        assert int(jh.item()) == ref["j"] and rel(h.cpu().numpy(), href) <= TOL


def test_f16_unaligned_shards_and_subnormal_values():
    wl, th, gr, th_np, gr_np = gen("resnet50", 40_003, 16)
    # values in half precision's subnormal range (multiples of 2^-24) widen exactly
    g = torch.Generator(device=DEV)
    g.manual_seed(1)
    gr[:, :100] = (torch.randint(-900, 900, (16, 100), device=DEV, generator=g).float() * 2.0 ** -24).half()
    gr_np = synth.to_numpy_stored(gr)
    assert np.any((np.abs(gr_np[:, :100].astype(np.float64)) < 6.1e-5) & (gr_np[:, :100] != 0))
    for r0, rows in ((0, 40_003), (3, 30_000), (5, 1_025), (8, 16)):
        Cs, ws = qn.qn_gram(gr[:, r0:r0 + rows])
        Co, wo = oracle.gram_accumulate(np.ascontiguousarray(gr_np[:, r0:r0 + rows]))
        assert rel(Cs.cpu().numpy(), Co) <= 1e-5 and rel(ws.cpu().numpy(), wo) <= 1e-5
        ref = oracle.update_streaming(np.ascontiguousarray(th_np[:, r0:r0 + rows]),
                                      np.ascontiguousarray(gr_np[:, r0:r0 + rows]), 0.7, np.float32(0.01))
        out, j = qn.qn_update(th[:, r0:r0 + rows], gr[:, r0:r0 + rows], 0.7, 0.01)
        assert int(j.item()) == ref["j"]
        assert_close(out.cpu().numpy(), ref["theta_new"], TOL)
