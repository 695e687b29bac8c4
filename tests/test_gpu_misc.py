"""GPU tests of the library's plumbing: streams, tracing, probes, graph capture
and the binding's argument checks."""
import numpy as np
import pytest
import torch

import paper_1709_05069_amd as qn
from paper_1709_05069_amd import synth, _lib

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _inputs(n=70_000, name="gpt2_small"):
    wl = synth.WORKLOADS[name].scaled(n)
    th, gr = synth.make_worker_states(wl, DEV)
    return wl, th, gr


def test_trace_counts_every_kernel_once_per_update():
    wl, th, gr = _inputs()
    qn.trace_begin(64)
    for _ in range(3):
        qn.qn_update(th, gr, wl.tau, wl.lam)
    tr = qn.trace_end()
    assert set(tr) == set(qn.KERNEL_NAMES)
    for name, (ms, cnt) in tr.items():
        # the pieces' projection kernel (the fused step projects inside the eigen
        # kernel), the coefficient piece, the capped step
        if name in ("gram_project", "coef", "tau_bound"):
            assert cnt == 0
        else:
            assert cnt == 3 and ms > 0.0
    with pytest.raises(qn.QnError):
        qn.trace_end()                       # not tracing any more
    # more launches than slots: the surplus is simply not timed
    qn.trace_begin(2)
    qn.qn_update(th, gr, wl.tau, wl.lam)
    tr = qn.trace_end()
    assert sum(c for _, c in tr.values()) == 2
    # the operator on an arbitrary vector: the Gram pass carries z, then the
    # eigen kernel and the apply sweep
    qn.trace_begin(64)
    qn.qn_hinv(th, gr, torch.randn(th.shape[1], device=DEV), wl.lam)
    tr = qn.trace_end()
    assert tr["gram_stage1"][1] == 1 and tr["eig_select"][1] == 1 and tr["apply_kernel"][1] == 1
    assert tr["coef"][1] == 0


def test_side_stream_gives_the_same_bits():
    wl, th, gr = _inputs()
    a, ja = qn.qn_update(th, gr, wl.tau, wl.lam)
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        b, jb = qn.qn_update(th, gr, wl.tau, wl.lam)
    s.synchronize()
    assert torch.equal(a, b) and int(ja.item()) == int(jb.item())


def test_probes_move_the_bytes_they_claim():
    src = torch.randn(1 << 20, device=DEV)
    dst = torch.zeros_like(src)
    qn.probe_copy(src, dst)
    sink = qn.probe_read(src)
    torch.cuda.synchronize()
    assert torch.equal(src, dst)
    assert sink.numel() == _lib.load().qn_probe_sink_floats()
    with pytest.raises(qn.QnError):
        qn.probe_copy(src[:1001], dst[:1001])          # not a multiple of 16 bytes


def test_latency_probe_times_its_chain():
    short = qn.probe_chain(8 * 1000)
    long = qn.probe_chain(8 * 4000)
    torch.cuda.synchronize()
    t_short, t_long = int(short[0].item()), int(long[0].item())
    assert t_short > 0 and int(short[1].item()) > 0
    # four times the links: four times the time (dependent chain, nothing else)
    assert 3.0 <= t_long / t_short <= 5.0
    # 8000 dependent fp64 multiply-adds at a few clocks each: tens of microseconds
    assert 1e-6 <= t_short / 100e6 <= 1e-3
    with pytest.raises(qn.QnError):
        qn.probe_chain(7)


def test_binding_rejects_bad_tensors():
    wl, th, gr = _inputs(5_000, "small_mlp")
    with pytest.raises(qn.QnError):
        qn.qn_update(th.cpu(), gr.cpu(), 1.0, 0.1)
    with pytest.raises(qn.QnError):
        qn.qn_update(th, gr[:, :-1], 1.0, 0.1)
    with pytest.raises(qn.QnError):
        qn.qn_update(th.double(), gr.double(), 1.0, 0.1)
    with pytest.raises(qn.QnError):
        qn.qn_update(th.t(), gr.t(), 1.0, 0.1)           # rows not contiguous
    with pytest.raises(qn.QnError):
        qn.qn_update(th, gr, 1.0, -0.5)                  # lambda <= 0: library says EINVAL
    with pytest.raises(qn.QnError):
        qn.qn_apply(th, gr, torch.zeros(3, device=DEV), 1.0)
    with pytest.raises(qn.QnError):
        qn.qn_update(th[:, :0], gr[:, :0], 1.0, 0.1)    # no rows
    big = torch.zeros((65, 64), device=DEV)
    with pytest.raises(qn.QnError):
        qn.qn_gram(big)                                  # m > QN_MAX_M


def test_update_can_be_captured_in_a_hip_graph_and_replayed():
    # after qn_init the step allocates nothing and records no memset, so a
    # caller may capture it; every replay must reproduce the eager result, also
    # with fresh inputs copied into the captured buffers between replays
    wl, th, gr = _inputs(200_000, "resnet50")
    qn.qn_init()
    ws = torch.empty(qn.workspace_bytes(wl.n, wl.m), dtype=torch.uint8, device=DEV)
    out = torch.empty(wl.n, dtype=torch.float32, device=DEV)
    j = torch.zeros(1, dtype=torch.int32, device=DEV)
    eager, je = qn.qn_update(th, gr, wl.tau, wl.lam)
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        qn.qn_update(th, gr, wl.tau, wl.lam, out, j, workspace=ws)   # warm-up on the side stream
    torch.cuda.current_stream().wait_stream(s)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        # the caller's scratch buffer: nothing is allocated under capture
        qn.qn_update(th, gr, wl.tau, wl.lam, out, j, workspace=ws)
    for rep in range(3):
        out.zero_()
        j.zero_()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager) and int(j.item()) == int(je.item())
        # eager work of the program between replays
        _ = qn.qn_gram(gr)
        torch.cuda.synchronize()
    # new inputs in the captured buffers
    wl2 = synth.WORKLOADS["resnet50"].scaled(200_000)
    from dataclasses import replace
    th2, gr2 = synth.make_worker_states(replace(wl2, seed=5), DEV)
    th.copy_(th2)
    gr.copy_(gr2)
    eager2, je2 = qn.qn_update(th, gr, wl.tau, wl.lam)
    g.replay()
    torch.cuda.synchronize()
    assert torch.equal(out, eager2) and int(j.item()) == int(je2.item())
    assert not torch.equal(eager2, eager)
