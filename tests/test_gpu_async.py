"""The step after a single worker's Write (Section 2, opening sentence): the m x m
state kept between steps against qn_gram of the current matrix, and the whole
step against the oracle on the current worker states, over sequences of Writes
by arbitrary workers -- the pivot worker, the same worker twice, every worker."""
import ctypes
from dataclasses import replace

import numpy as np
import pytest
import torch

import oracle
import paper_1709_05069_amd as qn
from paper_1709_05069_amd import synth, _lib
from parity_util import rel, assert_close

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

CASES = [
    # name, n, m, storage, sequence of writing workers
    ("gpt2_small", 50_000, 32, "f32", [5, 0, 1, 1, 31, 2, 0]),
    ("gpt2_small", 20_003, 64, "f32", [63, 0, 1, 0, 17]),
    ("resnet50", 70_001, 16, "f32", [0, 0, 1, 15, 8]),
    ("small_mlp", 12_345, 8, "f32", [3, 0, 7]),
    ("tiny_exact", 4096, 4, "f32", [0, 1, 2, 3, 0]),
    ("small_mlp", 999, 3, "f32", [2, 0, 1]),
    ("small_mlp", 5, 2, "f32", [0, 1, 0]),
    ("stress_1b_bf16", 60_000, 32, "bf16", [0, 9, 31, 1]),
    ("stress_1b_bf16", 30_001, 48, "bf16", [47, 0, 1]),
    ("gpt2_small", 40_000, 64, "f16", [1, 0, 63]),
    ("gpt2_small", 25_007, 20, "f16", [19, 0, 0, 7]),
    ("gpt2_small", 100_000, 1, "f32", [0, 0]),
    # long enough that the column pass runs with its capped grid (every thread
    # takes several row groups), for each blocks-per-unit setting
    ("gpt2_small", 2_000_003, 32, "f32", [7, 0]),
    ("resnet50", 1_500_001, 16, "f32", [0, 15]),
    ("small_mlp", 3_000_002, 4, "f32", [3, 0]),
    ("small_mlp", 2_500_000, 8, "f32", [1]),
    ("stress_1b_bf16", 3_000_008, 8, "bf16", [0, 5]),
    ("stress_1b_bf16", 2_000_001, 32, "bf16", [31]),
]


def _rewrite(wl, th, gr, worker, step):
    """A fresh (theta_k, grad_k) for one worker: another draw of the same recipe."""
    wl2 = replace(wl, seed=1000 + 17 * step + worker)
    th2, gr2 = synth.make_worker_states(wl2, DEV)
    src = (worker + 1 + step) % wl.m
    th[worker].copy_(th2[src])
    gr[worker].copy_(gr2[src])


@pytest.mark.parametrize("name,n,m,storage,writes", CASES)
def test_state_follows_single_worker_writes(name, n, m, storage, writes):
    wl = replace(synth.WORKLOADS[name].scaled(n), m=m, storage=storage)
    th, gr = synth.make_worker_states(wl, DEV)
    st = qn.GramState(gr)
    C, w = st.gram()
    Cf, wf = qn.qn_gram(gr)
    if m > 1:
        assert rel(C.cpu().numpy(), Cf.cpu().numpy()) <= 1e-12      # the same pass, re-expressed
        assert rel(w.cpu().numpy(), wf.cpu().numpy()) <= 1e-9
    tol = 1e-5 if storage == "f32" else (1e-3 if storage == "bf16" else 1e-4)
    lam32 = np.float32(wl.lam)
    for step, worker in enumerate(writes):
        _rewrite(wl, th, gr, worker, step)
        out, j = st.update(th, gr, worker, wl.tau, wl.lam)
        torch.cuda.synchronize()
        th_np, gr_np = synth.to_numpy_stored(th), synth.to_numpy_stored(gr)
        # the state is the Gram matrix of the current gradients
        C, w = st.gram()
        Co, wo = oracle.gram_accumulate(gr_np)
        if m > 1:
            assert rel(C.cpu().numpy(), Co) <= 1e-6, (step, worker)
            assert rel(w.cpu().numpy(), wo) <= 1e-6, (step, worker)
            Cf, wf = qn.qn_gram(gr)
            assert rel(C.cpu().numpy(), Cf.cpu().numpy()) <= 1e-5
        else:
            assert torch.all(C == 0) and torch.all(w == 0)
        # and the step is the oracle's step on the current worker states
        ref = oracle.update_streaming(th_np, gr_np, wl.tau, lam32)
        margin = (np.min(np.abs(ref["sigma"][:max(m - 1, 1)] / ref["sigma"][0] - lam32))
                  if ref["sigma"][0] > 0 else 1.0)
        assert margin > 1e-4
        assert int(j.item()) == ref["j"], (step, worker)
        assert_close(out.cpu().numpy(), ref["theta_new"], tol, what=f"step {step} worker {worker}")
        full, jf = qn.qn_update(th, gr, wl.tau, wl.lam)
        assert int(jf.item()) == ref["j"]
        assert_close(out.cpu().numpy(), full.cpu().numpy(), 10 * tol if storage != "f32" else 2e-6)


def test_state_write_without_step_and_several_columns_changed():
    wl = replace(synth.WORKLOADS["gpt2_small"].scaled(33_333), m=24)
    th, gr = synth.make_worker_states(wl, DEV)
    st = qn.GramState(gr)
    for step, worker in enumerate([4, 0, 23]):       # three Writes, then bring the state up to date
        _rewrite(wl, th, gr, worker, step)
    for worker in (0, 23, 4):                        # any order
        st.write(gr, worker)
    C, w = st.gram()
    Co, wo = oracle.gram_accumulate(synth.to_numpy_stored(gr))
    assert rel(C.cpu().numpy(), Co) <= 1e-6 and rel(w.cpu().numpy(), wo) <= 1e-6
    # deterministic: the same sequence gives the same bits
    th2, gr2 = synth.make_worker_states(wl, DEV)
    st2 = qn.GramState(gr2)
    for step, worker in enumerate([4, 0, 23]):
        _rewrite(wl, th2, gr2, worker, step)
    for worker in (0, 23, 4):
        st2.write(gr2, worker)
    C2, w2 = st2.gram()
    assert torch.equal(C, C2) and torch.equal(w, w2)


def test_state_entry_points_check_their_arguments():
    L = _lib.load()
    p = 0x1000
    big = 1 << 30
    assert L.qn_gram_state_bytes() >= (64 * 64 + 64) * 8
    assert L.qn_gram_state_init_ws(p, 0, 10, 4, 10, None, p, big, None) == -1          # no state
    assert L.qn_gram_state_write_ws(p, 0, 10, 4, 10, 4, p, p, big, None) == -1         # worker >= m
    assert L.qn_gram_state_write_ws(p, 0, 10, 4, 10, -1, p, p, big, None) == -1
    assert L.qn_gram_state_get(p, 65, p, p, None) == -1
    assert L.qn_update_async_ws(p, p, 0, 10, 4, 10, 0, 1.0, 0.0, p, p, p, p, big, None) == -1
    wl = synth.WORKLOADS["small_mlp"].scaled(1000)
    th, gr = synth.make_worker_states(wl, DEV)
    st = qn.GramState(gr)
    with pytest.raises(qn.QnError):
        st.write(gr[:, :500], 0)                      # not the matrix the state was made from
    with pytest.raises(qn.QnError):
        st.write(gr, wl.m)
    # too small a workspace is refused before anything is enqueued
    state = torch.empty(L.qn_gram_state_bytes(), dtype=torch.uint8, device=DEV)
    ws = torch.empty(1024, dtype=torch.uint8, device=DEV)
    m, n = gr.shape
    assert L.qn_gram_state_init_ws(gr.data_ptr(), 0, n, m, n, state.data_ptr(), ws.data_ptr(),
                                   1024, None) == -5
