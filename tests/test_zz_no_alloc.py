"""The entry point that allocates nothing (its scratch memory is a static device
array inside the library), through the C ABI: two calls in a row, the second on a
smaller problem, each against qn_update_ex on the same inputs."""
import ctypes

import pytest
import torch

from paper_1709_05069_amd import synth, _lib

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
QN_EWORKSPACE = -5


def _states(name, n, m, seed):
    from dataclasses import replace
    wl = replace(synth.WORKLOADS[name].scaled(n), m=m, seed=seed)
    th, gr = synth.make_worker_states(wl, DEV)
    return wl, th, gr


def _call(fn, th, gr, wl, out, j):
    m, n = th.shape
    dt = {torch.float32: 0, torch.bfloat16: 1, torch.float16: 2}[th.dtype]
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    rc = fn(th.data_ptr(), gr.data_ptr(), dt, n, m, th.stride(0), wl.tau, wl.lam,
            out.data_ptr(), j.data_ptr(), stream)
    torch.cuda.synchronize()
    return rc


def test_no_alloc_entry_point_matches_qn_update_ex_on_two_calls_in_a_row():
    L = _lib.load()
    # first a problem that fills the grid (512 partials of 768 entries), then a
    # smaller one of another shape and storage type, then a tiny one on the fp64
    # Gram kernel: stale scratch from the larger calls must not leak into them
    cases = [("gpt2_small", 2_000_003, 32, 1), ("stress_1b_bf16", 300_000, 8, 2),
             ("small_mlp", 1000, 5, 3)]
    inputs = [_states(*c) for c in cases]
    outs = [(torch.empty(wl.n, dtype=torch.float32, device=DEV),
             torch.zeros(1, dtype=torch.int32, device=DEV)) for wl, _, _ in inputs]
    refs = [(torch.empty(wl.n, dtype=torch.float32, device=DEV),
             torch.zeros(1, dtype=torch.int32, device=DEV)) for wl, _, _ in inputs]
    torch.cuda.synchronize()
    # The first launch in a process makes the HIP runtime load the library's code
    # object, static array included; from then on the free device memory must not move.
    wl, th, gr = inputs[2]
    assert _call(L.qn_update_noalloc, th, gr, wl, *outs[2]) == 0
    outs[2][0].zero_()
    free_before, _ = torch.cuda.mem_get_info()
    for (wl, th, gr), (out, j) in zip(inputs, outs):          # back to back
        assert _call(L.qn_update_noalloc, th, gr, wl, out, j) == 0
    free_after, _ = torch.cuda.mem_get_info()
    assert free_after == free_before                           # no device memory was taken
    for (wl, th, gr), (ref, jr) in zip(inputs, refs):
        assert _call(L.qn_update_ex, th, gr, wl, ref, jr) == 0
    for (wl, _, _), (out, j), (ref, jr) in zip(inputs, outs, refs):
        assert int(j.item()) == int(jr.item()) == wl.m - 1
        assert torch.equal(out, ref), wl.name                 # same kernels: same bits
    # and once more in the other order
    for k in (2, 0):
        wl, th, gr = inputs[k]
        out, j = outs[k]
        out.zero_()
        assert _call(L.qn_update_noalloc, th, gr, wl, out, j) == 0
        assert torch.equal(out, refs[k][0])


def test_no_alloc_entry_point_checks_its_arguments():
    L = _lib.load()
    p = 0x1000
    assert L.qn_update_noalloc(p, p, 0, 0, 4, 0, 1.0, 0.1, p, p, None) == -1      # n < 1
    assert L.qn_update_noalloc(p, p, 0, 10, 65, 10, 1.0, 0.1, p, p, None) == -1   # m > max
    assert L.qn_update_noalloc(p, p, 5, 10, 4, 10, 1.0, 0.1, p, p, None) == -1    # dtype
    assert L.qn_update_noalloc(p, None, 0, 10, 4, 10, 1.0, 0.1, p, p, None) == -1
    # every valid problem fits the static array on this device
    assert max(L.qn_workspace_bytes(1 << 40, m, dt) for m in (16, 32, 48, 64)
               for dt in (0, 1, 2)) <= 6 * 1024 * 1024


def test_no_alloc_entry_point_under_hip_graph_capture():
    # the caller this entry point is for: a captured stream may not allocate.  Every
    # replay, with eager work of the same library between replays, gives the eager bits
    L = _lib.load()
    wl, th, gr = _states("resnet50", 300_000, 16, 4)
    out = torch.empty(wl.n, dtype=torch.float32, device=DEV)
    j = torch.zeros(1, dtype=torch.int32, device=DEV)
    ref = torch.empty_like(out)
    jr = torch.zeros_like(j)
    assert _call(L.qn_update_ex, th, gr, wl, ref, jr) == 0

    def enqueue():
        m, n = th.shape
        stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
        return L.qn_update_noalloc(th.data_ptr(), gr.data_ptr(), 0, n, m, th.stride(0), wl.tau,
                                   wl.lam, out.data_ptr(), j.data_ptr(), stream)

    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        assert enqueue() == 0                     # set-up happens outside the capture
    torch.cuda.current_stream().wait_stream(s)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        rc = enqueue()
    assert rc == 0
    other = torch.empty_like(out)
    for rep in range(3):
        out.zero_()
        j.zero_()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, ref) and int(j.item()) == int(jr.item())
        wl2, th2, gr2 = _states("small_mlp", 50_000 + rep, 8, 5 + rep)   # dirties the shared scratch
        assert _call(L.qn_update_noalloc, th2, gr2, wl2, other[:wl2.n], jr.clone()) == 0
