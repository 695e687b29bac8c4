"""Caller-owned scratch memory: the *_ws entry points through the C ABI."""
import ctypes

import numpy as np
import pytest
import torch

import paper_1709_05069_amd as qn
from paper_1709_05069_amd import synth, _lib

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
QN_EWORKSPACE = -5


def _inputs(n, name="gpt2_small", m=None, seed=0):
    from dataclasses import replace
    wl = synth.WORKLOADS[name].scaled(n)
    wl = replace(wl, seed=seed, m=m if m else wl.m)
    th, gr = synth.make_worker_states(wl, DEV)
    return wl, th, gr


def _raw_update_ws(L, th, gr, wl, out, j, ws_ptr, ws_bytes, stream):
    m, n = th.shape
    return L.qn_update_ws(th.data_ptr(), gr.data_ptr(), 0, n, m, th.stride(0), wl.tau, wl.lam,
                          out.data_ptr(), j.data_ptr(), ws_ptr, ws_bytes,
                          ctypes.c_void_p(stream.cuda_stream))


def test_workspace_size_is_what_the_problem_needs():
    L = _lib.load()
    cu = torch.cuda.get_device_properties(0).multi_processor_count
    # one 256-entry partial per block, at most 4 blocks per unit, plus the fixed part
    small = L.qn_workspace_bytes(100, 4, 0)
    assert small < 64 * 1024 + 3 * 32768 + 16 * 1024
    full = L.qn_workspace_bytes(124_000_000, 32, 0)
    assert full >= 2 * cu * 768 * 8 and full <= 2 * cu * 768 * 8 + 300 * 1024
    assert full == qn.workspace_bytes(124_000_000, 32)


def test_too_small_misaligned_or_missing_workspace_is_refused():
    L = _lib.load()
    wl, th, gr = _inputs(50_000)
    out = torch.full((wl.n,), 7.0, device=DEV)
    j = torch.full((1,), 99, dtype=torch.int32, device=DEV)
    need = L.qn_workspace_bytes(wl.n, wl.m, 0)
    buf = torch.empty(need + 512, dtype=torch.uint8, device=DEV)
    s = torch.cuda.current_stream()
    assert buf.data_ptr() % 256 == 0
    assert _raw_update_ws(L, th, gr, wl, out, j, buf.data_ptr(), need - 1, s) == QN_EWORKSPACE
    assert _raw_update_ws(L, th, gr, wl, out, j, buf.data_ptr() + 16, need, s) == QN_EWORKSPACE
    assert _raw_update_ws(L, th, gr, wl, out, j, None, need, s) == QN_EWORKSPACE
    m, n = gr.shape
    C = torch.empty((m, m), dtype=torch.float64, device=DEV)
    w = torch.empty(m, dtype=torch.float64, device=DEV)
    assert L.qn_gram_ws(gr.data_ptr(), 0, n, m, n, C.data_ptr(), w.data_ptr(), buf.data_ptr(),
                        1024, None) == QN_EWORKSPACE
    torch.cuda.synchronize()
    # nothing was enqueued: the outputs are untouched
    assert float(out.min()) == 7.0 and int(j.item()) == 99
    assert L.qn_status_string(QN_EWORKSPACE).startswith(b"workspace")
    # exactly enough is enough
    assert _raw_update_ws(L, th, gr, wl, out, j, buf.data_ptr(), need, s) == 0
    ref, jr = qn.qn_update(th, gr, wl.tau, wl.lam)
    torch.cuda.synchronize()
    assert torch.equal(out, ref) and int(j.item()) == int(jr.item())


def test_two_streams_with_two_workspaces_overlap_and_give_the_serial_bits():
    L = _lib.load()
    # two different problems, each large enough to keep the device busy for a while
    wa, tha, gra = _inputs(6_000_000, "gpt2_small", seed=1)
    wb, thb, grb = _inputs(9_000_001, "resnet50", seed=2)
    serial_a, ja = qn.qn_update(tha, gra, wa.tau, wa.lam)
    serial_b, jb = qn.qn_update(thb, grb, wb.tau, wb.lam)
    torch.cuda.synchronize()
    wsa = torch.empty(qn.workspace_bytes(wa.n, wa.m), dtype=torch.uint8, device=DEV)
    wsb = torch.empty(qn.workspace_bytes(wb.n, wb.m), dtype=torch.uint8, device=DEV)
    outa, outb = torch.empty_like(serial_a), torch.empty_like(serial_b)
    j2a = torch.zeros(1, dtype=torch.int32, device=DEV)
    j2b = torch.zeros(1, dtype=torch.int32, device=DEV)
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    for rep in range(4):
        outa.zero_()
        outb.zero_()
        torch.cuda.synchronize()
        # interleaved submission: the two steps are in flight together
        assert _raw_update_ws(L, tha, gra, wa, outa, j2a, wsa.data_ptr(), wsa.numel(), sa) == 0
        assert _raw_update_ws(L, thb, grb, wb, outb, j2b, wsb.data_ptr(), wsb.numel(), sb) == 0
        assert _raw_update_ws(L, tha, gra, wa, outa, j2a, wsa.data_ptr(), wsa.numel(), sa) == 0
        assert _raw_update_ws(L, thb, grb, wb, outb, j2b, wsb.data_ptr(), wsb.numel(), sb) == 0
        sa.synchronize()
        sb.synchronize()
        assert torch.equal(outa, serial_a) and torch.equal(outb, serial_b), rep
        assert int(j2a.item()) == int(ja.item()) and int(j2b.item()) == int(jb.item())


def test_the_binding_keeps_one_workspace_per_stream():
    wl, th, gr = _inputs(300_000)
    a, _ = qn.qn_update(th, gr, wl.tau, wl.lam)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        b, _ = qn.qn_update(th, gr, wl.tau, wl.lam)
    s.synchronize()
    torch.cuda.synchronize()
    keys = {k for k in qn.qn._WORKSPACES if k[0] == 0}
    assert len(keys) >= 2 and torch.equal(a, b)
    explicit = torch.empty(qn.workspace_bytes(wl.n, wl.m), dtype=torch.uint8, device=DEV)
    c, _ = qn.qn_update(th, gr, wl.tau, wl.lam, workspace=explicit)
    torch.cuda.synchronize()
    assert torch.equal(a, c)
    with pytest.raises(qn.QnError):
        qn.qn_update(th, gr, wl.tau, wl.lam, workspace=explicit[:1000])


def test_library_owned_workspace_gives_the_same_bits_and_survives_shutdown():
    L = _lib.load()
    wl, th, gr = _inputs(30_000, "resnet50")
    m, n = th.shape
    ref, jr = qn.qn_update(th, gr, wl.tau, wl.lam)
    out = torch.empty_like(ref)
    j = torch.zeros(1, dtype=torch.int32, device=DEV)

    def plain():
        rc = L.qn_update(th.data_ptr(), gr.data_ptr(), n, m, wl.tau, wl.lam, out.data_ptr(),
                         j.data_ptr(), ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
        assert rc == 0
        torch.cuda.synchronize()

    plain()
    assert torch.equal(out, ref) and int(j.item()) == int(jr.item())
    assert L.qn_shutdown() == 0
    out.zero_()
    plain()                                  # allocates its workspace again
    assert torch.equal(out, ref)
    assert L.qn_init() == 0
    # the other entry points that use scratch memory, both forms
    z = torch.randn(n, device=DEV)
    h, jh = qn.qn_hinv(th, gr, z, wl.lam)
    h2 = torch.empty_like(h)
    assert L.qn_hinv(th.data_ptr(), gr.data_ptr(), z.data_ptr(), n, m, wl.lam, h2.data_ptr(),
                     j.data_ptr(), None) == 0
    w = qn.qn_gemv_t(gr, z)
    w2 = torch.empty_like(w)
    assert L.qn_gemv_t_ex(gr.data_ptr(), 0, z.data_ptr(), n, m, n, w2.data_ptr(), None) == 0
    b, jb, tb = qn.qn_update_bounded(th, gr, wl.tau, wl.lam, qn.BOUND_SECANT)
    b2, t2 = torch.empty_like(b), torch.empty_like(tb)
    assert L.qn_update_bounded_ex(th.data_ptr(), gr.data_ptr(), 0, n, m, n, wl.tau, wl.lam, 2,
                                  b2.data_ptr(), j.data_ptr(), t2.data_ptr(), None) == 0
    C, wg = qn.qn_gram(gr)
    C2, wg2 = torch.empty_like(C), torch.empty_like(wg)
    assert L.qn_gram(gr.data_ptr(), n, m, C2.data_ptr(), wg2.data_ptr(), None) == 0
    torch.cuda.synchronize()
    assert torch.equal(h, h2) and torch.equal(w, w2) and torch.equal(b, b2) and torch.equal(tb, t2)
    assert torch.equal(C, C2) and torch.equal(wg, wg2)


def test_two_host_threads_with_their_own_workspaces_and_streams():
    # the *_ws entry points keep no shared state: two host threads, each with its own
    # stream and workspace, submit steps at the same time and get the serial bits
    import threading
    L = _lib.load()
    cases = [_inputs(1_500_000, "gpt2_small", seed=11), _inputs(2_000_003, "resnet50", seed=12)]
    serial = [qn.qn_update(th, gr, wl.tau, wl.lam) for wl, th, gr in cases]
    torch.cuda.synchronize()
    results, errors = [None, None], []

    def work(i):
        try:
            torch.cuda.set_device(0)
            wl, th, gr = cases[i]
            stream = torch.cuda.Stream()
            ws = torch.empty(qn.workspace_bytes(wl.n, wl.m), dtype=torch.uint8, device=DEV)
            out = torch.empty(wl.n, dtype=torch.float32, device=DEV)
            j = torch.zeros(1, dtype=torch.int32, device=DEV)
            torch.cuda.synchronize()
            for _ in range(20):
                rc = _raw_update_ws(L, th, gr, wl, out, j, ws.data_ptr(), ws.numel(), stream)
                assert rc == 0
            stream.synchronize()
            results[i] = (out, j)
        except Exception as e:            # surfaced in the main thread below
            errors.append(e)

    threads = [threading.Thread(target=work, args=(i,)) for i in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    for (out, j), (ref, jr) in zip(results, serial):
        assert torch.equal(out, ref) and int(j.item()) == int(jr.item())
