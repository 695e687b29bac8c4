"""Argument marshalling for libqn's C ABI: torch tensors in, torch tensors out.

Worker matrices are (m, n) tensors whose rows are the workers' vectors
(stride(1) == 1; stride(0) = ld >= n), dtype float32, bfloat16 or float16, on the HIP
device.  Every step of the computation runs in the library's kernels; torch
only owns the memory and the stream.
"""
import ctypes

import torch

from . import _lib

QN_F32, QN_BF16, QN_F16 = 0, 1, 2
KERNEL_NAMES = ("gram_stage1", "gram_reduce", "gram_project", "eig_select",
                "apply_kernel", "coef", "tau_bound")


class QnError(RuntimeError):
    pass


def _check(rc: int, what: str):
    if rc != 0:
        msg = _lib.load().qn_status_string(rc).decode()
        raise QnError(f"{what}: {msg} (status {rc})")


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _worker(t: torch.Tensor, name: str):
    if not t.is_cuda:
        raise QnError(f"{name} must live on the HIP device")
    if t.dim() != 2 or t.stride(1) != 1:
        raise QnError(f"{name} must have shape (m, n) with unit stride along n")
    if t.dtype == torch.float32:
        dt = QN_F32
    elif t.dtype == torch.bfloat16:
        dt = QN_BF16
    elif t.dtype == torch.float16:
        dt = QN_F16
    else:
        raise QnError(f"{name}: unsupported dtype {t.dtype}")
    m, n = t.shape
    ld = t.stride(0) if m > 1 else max(n, 1)
    return dt, m, n, ld


def _dev_out(t, shape, dtype, device, name):
    if t is None:
        return torch.empty(shape, dtype=dtype, device=device)
    if t.dtype != dtype or tuple(t.shape) != tuple(shape) or not t.is_contiguous() \
            or t.device != device:
        raise QnError(f"{name}: expected a contiguous {dtype} tensor of shape {shape}")
    return t


# Scratch memory of the library's passes: torch allocates it, one buffer per
# (device, stream) sized for the largest problem (a few MB), kept for the life of
# the process, and every call goes through the library's *_ws entry points, so the
# library itself allocates nothing.  Calls on different streams use different
# buffers and may overlap.
_WORKSPACES = {}
_MAX_ROWS = 1 << 40


def workspace_bytes(n: int, m: int, dtype: int = QN_F32) -> int:
    """Bytes of scratch memory an (n, m) problem of this element type needs."""
    return int(_lib.load().qn_workspace_bytes(int(n), int(m), int(dtype)))


def _workspace(device, stream, workspace=None):
    """(pointer, bytes) of the scratch buffer for a call on this device and stream."""
    if workspace is not None:
        if not (workspace.is_cuda and workspace.dtype == torch.uint8
                and workspace.is_contiguous() and workspace.device == device):
            raise QnError("workspace must be a contiguous uint8 tensor on the inputs' device")
        return workspace.data_ptr(), workspace.numel()
    s = torch.cuda.current_stream(device) if stream is None else stream
    key = (device.index, s.cuda_stream)
    buf = _WORKSPACES.get(key)
    if buf is None:
        with torch.cuda.device(device):
            need = max(workspace_bytes(_MAX_ROWS, 64, dt) for dt in (QN_F32, QN_BF16, QN_F16))
        if need == 0:
            raise QnError("qn_workspace_bytes failed")
        buf = torch.empty(need, dtype=torch.uint8, device=device)
        _WORKSPACES[key] = buf
    return buf.data_ptr(), buf.numel()


def qn_init():
    """Prepares the current device and this stream's scratch buffer ahead of the
    first call (nothing is allocated inside the calls after it)."""
    dev = torch.device("cuda", torch.cuda.current_device())
    _workspace(dev, None)


def qn_update(thetas, grads, tau, lam, theta_new=None, j_out=None, stream=None,
              workspace=None):
    """theta_new (n fp32) and j_out (1 int32, on device) for the whole step.
    workspace: optional uint8 device tensor of at least workspace_bytes(n, m, dtype)."""
    L = _lib.load()
    dt, m, n, ld = _worker(thetas, "thetas")
    dg, mg, ng, ldg = _worker(grads, "grads")
    if (dt, m, n, ld) != (dg, mg, ng, ldg):
        raise QnError("thetas and grads must agree in dtype, shape and stride")
    theta_new = _dev_out(theta_new, (n,), torch.float32, thetas.device, "theta_new")
    j_out = _dev_out(j_out, (1,), torch.int32, thetas.device, "j_out")
    ws, ws_bytes = _workspace(thetas.device, stream, workspace)
    _check(L.qn_update_ws(thetas.data_ptr(), grads.data_ptr(), dt, n, m, ld,
                          float(tau), float(lam), theta_new.data_ptr(),
                          j_out.data_ptr(), ws, ws_bytes, _stream(stream)), "qn_update")
    return theta_new, j_out


def qn_update_noalloc(thetas, grads, tau, lam, theta_new, j_out, stream=None):
    """The whole step through the entry point that allocates nothing: its scratch
    memory is a static device array inside the library.  The caller passes the
    outputs (theta_new: n fp32, j_out: 1 int32)."""
    L = _lib.load()
    dt, m, n, ld = _worker(thetas, "thetas")
    if (dt, m, n, ld) != _worker(grads, "grads"):
        raise QnError("thetas and grads must agree in dtype, shape and stride")
    theta_new = _dev_out(theta_new, (n,), torch.float32, thetas.device, "theta_new")
    j_out = _dev_out(j_out, (1,), torch.int32, thetas.device, "j_out")
    _check(L.qn_update_noalloc(thetas.data_ptr(), grads.data_ptr(), dt, n, m, ld,
                               float(tau), float(lam), theta_new.data_ptr(),
                               j_out.data_ptr(), _stream(stream)), "qn_update_noalloc")
    return theta_new, j_out


def qn_gram(grads, C=None, w=None, stream=None, workspace=None):
    """C = G^T G (m, m) and w = G^T g_bar (m,), float64 on device."""
    L = _lib.load()
    dt, m, n, ld = _worker(grads, "grads")
    C = _dev_out(C, (m, m), torch.float64, grads.device, "C")
    w = _dev_out(w, (m,), torch.float64, grads.device, "w")
    ws, ws_bytes = _workspace(grads.device, stream, workspace)
    _check(L.qn_gram_ws(grads.data_ptr(), dt, n, m, ld, C.data_ptr(),
                        w.data_ptr(), ws, ws_bytes, _stream(stream)), "qn_gram")
    return C, w


class GramState:
    """The m x m state of the step after single-worker Writes (qn_gram_state_*).
    Holds the device buffer; tied to the (m, n) worker matrix it was made from."""

    def __init__(self, grads, stream=None):
        L = _lib.load()
        self.dt, self.m, self.n, self.ld = _worker(grads, "grads")
        self.buf = torch.empty(int(L.qn_gram_state_bytes()), dtype=torch.uint8, device=grads.device)
        ws, ws_bytes = _workspace(grads.device, stream)
        _check(L.qn_gram_state_init_ws(grads.data_ptr(), self.dt, self.n, self.m, self.ld,
                                       self.buf.data_ptr(), ws, ws_bytes, _stream(stream)),
               "qn_gram_state_init")

    def _same(self, t, name):
        if _worker(t, name) != (self.dt, self.m, self.n, self.ld):
            raise QnError(f"{name} does not match the matrix the state was made from")

    def write(self, grads, worker, stream=None):
        """worker's row of grads has been overwritten: bring the state up to date."""
        self._same(grads, "grads")
        ws, ws_bytes = _workspace(grads.device, stream)
        _check(_lib.load().qn_gram_state_write_ws(
            grads.data_ptr(), self.dt, self.n, self.m, self.ld, int(worker),
            self.buf.data_ptr(), ws, ws_bytes, _stream(stream)), "qn_gram_state_write")

    def gram(self, stream=None):
        """(C, w) of the matrix the state describes, as qn_gram returns them."""
        C = torch.empty((self.m, self.m), dtype=torch.float64, device=self.buf.device)
        w = torch.empty(self.m, dtype=torch.float64, device=self.buf.device)
        _check(_lib.load().qn_gram_state_get(self.buf.data_ptr(), self.m, C.data_ptr(),
                                             w.data_ptr(), _stream(stream)), "qn_gram_state_get")
        return C, w

    def update(self, thetas, grads, worker, tau, lam, theta_new=None, j_out=None, stream=None):
        """The whole server step after worker's Write.  Returns (theta_new, j_out)."""
        self._same(thetas, "thetas")
        self._same(grads, "grads")
        theta_new = _dev_out(theta_new, (self.n,), torch.float32, thetas.device, "theta_new")
        j_out = _dev_out(j_out, (1,), torch.int32, thetas.device, "j_out")
        ws, ws_bytes = _workspace(thetas.device, stream)
        _check(_lib.load().qn_update_async_ws(
            thetas.data_ptr(), grads.data_ptr(), self.dt, self.n, self.m, self.ld, int(worker),
            float(tau), float(lam), self.buf.data_ptr(), theta_new.data_ptr(),
            j_out.data_ptr(), ws, ws_bytes, _stream(stream)), "qn_update_async")
        return theta_new, j_out


GRAM_AUTO, GRAM_STREAM, GRAM_SMALL = 0, 1, 2


def diag_gram(grads, path, z=None, stream=None):
    """qn_gram with the stage-1 kernel named by the caller (diagnostics): the
    matrix-core streaming pass (GRAM_STREAM) or the fp64 vector kernel
    (GRAM_SMALL).  With z (n fp32 values) w = G^T z.  Uses the library's own
    workspace."""
    L = _lib.load()
    dt, m, n, ld = _worker(grads, "grads")
    if z is not None:
        _vector(z, n, grads.device, "z")
    C = torch.empty((m, m), dtype=torch.float64, device=grads.device)
    w = torch.empty(m, dtype=torch.float64, device=grads.device)
    _check(L.qn_diag_gram_ex(grads.data_ptr(), dt, z.data_ptr() if z is not None else None,
                             n, m, ld, int(path), C.data_ptr(), w.data_ptr(),
                             _stream(stream)), "qn_diag_gram")
    return C, w


def qn_eig(C, w, lam, stream=None):
    """Returns (sigma (m,), V (m, m) with V[k] = v_k, c (m,) fp32, j (1,) int32)."""
    L = _lib.load()
    if not (C.is_cuda and w.is_cuda and C.dtype == torch.float64 and
            w.dtype == torch.float64 and C.is_contiguous() and w.is_contiguous()
            and C.dim() == 2 and C.shape[0] == C.shape[1] == w.shape[0]):
        raise QnError("C must be (m, m) and w (m,), contiguous float64 on device")
    m = C.shape[0]
    dev = C.device
    sigma = torch.empty(m, dtype=torch.float64, device=dev)
    V = torch.empty((m, m), dtype=torch.float64, device=dev)
    c = torch.empty(m, dtype=torch.float32, device=dev)
    j = torch.empty(1, dtype=torch.int32, device=dev)
    _check(L.qn_eig(C.data_ptr(), w.data_ptr(), m, float(lam), sigma.data_ptr(),
                    V.data_ptr(), c.data_ptr(), j.data_ptr(), _stream(stream)),
           "qn_eig")
    return sigma, V, c, j


def qn_apply(thetas, grads, c, tau, theta_new=None, stream=None):
    L = _lib.load()
    dt, m, n, ld = _worker(thetas, "thetas")
    dg, mg, ng, ldg = _worker(grads, "grads")
    if (dt, m, n, ld) != (dg, mg, ng, ldg):
        raise QnError("thetas and grads must agree in dtype, shape and stride")
    if not (c.is_cuda and c.dtype == torch.float32 and c.is_contiguous()
            and tuple(c.shape) == (m,)):
        raise QnError("c must be a contiguous float32 tensor of shape (m,) on device")
    theta_new = _dev_out(theta_new, (n,), torch.float32, thetas.device, "theta_new")
    _check(L.qn_apply_ex(thetas.data_ptr(), grads.data_ptr(), dt, n, m, ld,
                         c.data_ptr(), float(tau), theta_new.data_ptr(),
                         _stream(stream)), "qn_apply")
    return theta_new


def _vector(z, n, device, name):
    if not (z.is_cuda and z.dtype == torch.float32 and z.is_contiguous()
            and tuple(z.shape) == (n,) and z.device == device):
        raise QnError(f"{name} must be a contiguous float32 tensor of shape ({n},) on device")


def qn_hinv(thetas, grads, z, lam, out=None, j_out=None, stream=None):
    """Eq. (3)/(4) applied to an arbitrary vector z.  Returns (out, j_out)."""
    L = _lib.load()
    dt, m, n, ld = _worker(thetas, "thetas")
    if (dt, m, n, ld) != _worker(grads, "grads"):
        raise QnError("thetas and grads must agree in dtype, shape and stride")
    _vector(z, n, thetas.device, "z")
    out = _dev_out(out, (n,), torch.float32, thetas.device, "out")
    j_out = _dev_out(j_out, (1,), torch.int32, thetas.device, "j_out")
    ws, ws_bytes = _workspace(thetas.device, stream)
    _check(L.qn_hinv_ws(thetas.data_ptr(), grads.data_ptr(), dt, z.data_ptr(), n, m,
                        ld, float(lam), out.data_ptr(), j_out.data_ptr(), ws, ws_bytes,
                        _stream(stream)), "qn_hinv")
    return out, j_out


def qn_gemv_t(grads, z, stream=None):
    """w = G^T z (m,) float64 for the centred gradient matrix."""
    L = _lib.load()
    dt, m, n, ld = _worker(grads, "grads")
    _vector(z, n, grads.device, "z")
    w = torch.empty(m, dtype=torch.float64, device=grads.device)
    ws, ws_bytes = _workspace(grads.device, stream)
    _check(L.qn_gemv_t_ws(grads.data_ptr(), dt, z.data_ptr(), n, m, ld, w.data_ptr(),
                          ws, ws_bytes, _stream(stream)), "qn_gemv_t")
    return w


def qn_coef(sigma, V, j, w, stream=None):
    """c (m,) fp32 from qn_eig's sigma, V, the device int j and w."""
    L = _lib.load()
    m = sigma.shape[0]
    ok = (sigma.dtype == torch.float64 and V.dtype == torch.float64 and
          w.dtype == torch.float64 and j.dtype == torch.int32 and
          tuple(V.shape) == (m, m) and tuple(w.shape) == (m,) and j.numel() == 1 and
          all(t.is_cuda and t.is_contiguous() for t in (sigma, V, j, w)))
    if not ok:
        raise QnError("qn_coef: sigma (m,), V (m, m), w (m,) float64 and j (1,) int32 on device")
    c = torch.empty(m, dtype=torch.float32, device=sigma.device)
    _check(L.qn_coef(sigma.data_ptr(), V.data_ptr(), j.data_ptr(), w.data_ptr(), m,
                     c.data_ptr(), _stream(stream)), "qn_coef")
    return c


def qn_hinv_apply(thetas, grads, z, c, out=None, stream=None):
    """out = z + (Theta - G) c."""
    L = _lib.load()
    dt, m, n, ld = _worker(thetas, "thetas")
    if (dt, m, n, ld) != _worker(grads, "grads"):
        raise QnError("thetas and grads must agree in dtype, shape and stride")
    _vector(z, n, thetas.device, "z")
    if not (c.is_cuda and c.dtype == torch.float32 and c.is_contiguous()
            and tuple(c.shape) == (m,)):
        raise QnError("c must be a contiguous float32 tensor of shape (m,) on device")
    out = _dev_out(out, (n,), torch.float32, thetas.device, "out")
    _check(L.qn_hinv_apply_ex(thetas.data_ptr(), grads.data_ptr(), dt, z.data_ptr(), n,
                              m, ld, c.data_ptr(), out.data_ptr(), _stream(stream)),
           "qn_hinv_apply")
    return out


BOUND_SIGMA1, BOUND_SECANT = 1, 2


def qn_update_bounded(thetas, grads, tau, lam, mode, theta_new=None, j_out=None,
                      tau_out=None, stream=None):
    """The whole step with tau capped at 1 / sigma_max (mode: BOUND_SIGMA1 or
    BOUND_SECANT).  Returns (theta_new, j_out, tau_out (1,) fp32 on device)."""
    L = _lib.load()
    dt, m, n, ld = _worker(thetas, "thetas")
    if (dt, m, n, ld) != _worker(grads, "grads"):
        raise QnError("thetas and grads must agree in dtype, shape and stride")
    theta_new = _dev_out(theta_new, (n,), torch.float32, thetas.device, "theta_new")
    j_out = _dev_out(j_out, (1,), torch.int32, thetas.device, "j_out")
    tau_out = _dev_out(tau_out, (1,), torch.float32, thetas.device, "tau_out")
    ws, ws_bytes = _workspace(thetas.device, stream)
    _check(L.qn_update_bounded_ws(thetas.data_ptr(), grads.data_ptr(), dt, n, m, ld,
                                  float(tau), float(lam), int(mode),
                                  theta_new.data_ptr(), j_out.data_ptr(),
                                  tau_out.data_ptr(), ws, ws_bytes, _stream(stream)),
           "qn_update_bounded")
    return theta_new, j_out, tau_out


def qn_tau_bound(sigma, V, j, C_theta, tau, mode, stream=None):
    """(tau_eff (1,) fp32, sigma_max (1,) fp64) on device from qn_eig's sigma, V,
    the device int j and C_theta = Theta^T Theta (None for BOUND_SIGMA1)."""
    L = _lib.load()
    m = sigma.shape[0]
    ts = [sigma, V, j] + ([C_theta] if C_theta is not None else [])
    ok = (sigma.dtype == torch.float64 and V.dtype == torch.float64 and
          j.dtype == torch.int32 and tuple(V.shape) == (m, m) and j.numel() == 1 and
          (C_theta is None or (C_theta.dtype == torch.float64 and
                               tuple(C_theta.shape) == (m, m))) and
          all(t.is_cuda and t.is_contiguous() for t in ts))
    if not ok:
        raise QnError("qn_tau_bound: sigma (m,), V (m, m), C_theta (m, m) float64 and "
                      "j (1,) int32 on device")
    tau_out = torch.empty(1, dtype=torch.float32, device=sigma.device)
    smax = torch.empty(1, dtype=torch.float64, device=sigma.device)
    _check(L.qn_tau_bound(sigma.data_ptr(), V.data_ptr(), j.data_ptr(),
                          C_theta.data_ptr() if C_theta is not None else None, m,
                          float(tau), int(mode), tau_out.data_ptr(), smax.data_ptr(),
                          _stream(stream)), "qn_tau_bound")
    return tau_out, smax


def probe_copy(src, dst, stream=None):
    """dst = src through the library's plain copy kernel (known traffic)."""
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes:
        raise QnError("probe_copy: size mismatch")
    _check(_lib.load().qn_probe_copy(src.data_ptr(), dst.data_ptr(), nbytes,
                                     _stream(stream)), "qn_probe_copy")


def probe_read(src, stream=None):
    """Streams src once through the library's read-only kernel."""
    L = _lib.load()
    nsink = L.qn_probe_sink_floats()
    if nsink < 0:
        raise QnError("probe_read: no gfx950 device")
    sink = torch.empty(nsink, dtype=torch.float32, device=src.device)
    _check(L.qn_probe_read(src.data_ptr(), src.numel() * src.element_size(),
                           sink.data_ptr(), _stream(stream)), "qn_probe_read")
    return sink


def probe_chain(links, out=None, stream=None):
    """Enqueues the latency probe; returns the device tensor (3 x int64) holding
    100 MHz ticks, shader-counter ticks and a value of no meaning."""
    if out is None:
        out = torch.zeros(3, dtype=torch.int64, device="cuda")
    _check(_lib.load().qn_probe_chain(int(links), out.data_ptr(), _stream(stream)),
           "qn_probe_chain")
    return out


def trace_begin(max_launches: int = 4096):
    _check(_lib.load().qn_trace_begin(int(max_launches)), "qn_trace_begin")


def trace_end():
    """Returns {kernel name: (summed ms, launches)}."""
    ms = (ctypes.c_double * len(KERNEL_NAMES))()
    cnt = (ctypes.c_int * len(KERNEL_NAMES))()
    _check(_lib.load().qn_trace_end(ms, cnt), "qn_trace_end")
    return {name: (ms[i], cnt[i]) for i, name in enumerate(KERNEL_NAMES)}
