"""Closed loop on the synthetic quadratic (stand-in for the paper's Section 3
comparison of DistNewton-m with SGD): every server step of the loop is checked
against the oracle on the same worker states, and the qualitative claims are
asserted: the quasi-Newton server beats the largest stable SGD step, more
workers help, SGD at the same step length diverges."""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_1709_05069_amd import closed_loop, synth

pytestmark = pytest.mark.gpu


def test_every_server_step_of_the_loop_matches_the_oracle():
    worst = {"err": 0.0, "steps": 0}

    def check(it, thetas, grads, theta_new, j):
        ref = oracle.update_streaming(synth.to_numpy_stored(thetas),
                                      synth.to_numpy_stored(grads), 1.0,
                                      float(np.float32(0.1)))
        margin = np.min(np.abs(ref["sigma"][:-1] / ref["sigma"][0] - np.float32(0.1)))
        assert margin > 1e-4
        assert j == ref["j"]
        got = theta_new.cpu().numpy().astype(np.float64)
        err = np.linalg.norm(got - ref["theta_new"]) / np.linalg.norm(ref["theta_new"])
        worst["err"] = max(worst["err"], err)
        worst["steps"] += 1

    hist, js = closed_loop.run(n=20_000, m=16, iters=12, server="qn", on_step=check)
    assert worst["steps"] == 12 and worst["err"] <= 1e-5
    assert all(j == 4 for j in js)            # the four stiff directions are trusted
    assert hist[-1] < hist[0]


def test_quasi_newton_server_beats_stable_sgd_and_more_workers_help():
    kw = dict(n=50_000, iters=40)
    qn16, _ = closed_loop.run(server="qn", m=16, tau=1.0, **kw)
    qn8, _ = closed_loop.run(server="qn", m=8, tau=1.0, **kw)
    sgd_safe, _ = closed_loop.run(server="sgd", m=16, tau=0.095, **kw)
    sgd_big, _ = closed_loop.run(server="sgd", m=16, tau=1.0, **kw)
    assert qn16[-1] < 0.6 * sgd_safe[-1]
    assert qn16[-1] <= qn8[-1] * 1.05
    assert (not math.isfinite(sgd_big[-1])) or sgd_big[-1] > 1e6 * sgd_big[0]
    # too few workers to resolve the stiff directions (m - 1 < 4): no benefit
    qn4, _ = closed_loop.run(server="qn", m=4, tau=1.0, **kw)
    assert (not math.isfinite(qn4[-1])) or qn4[-1] > qn16[-1]
