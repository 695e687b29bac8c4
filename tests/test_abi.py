"""The C ABI without a GPU: the library loads, exports every function that
include/qn.h and include/qn_diag.h declare, and its host-only entry points behave."""
import os
import re
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "qn.h")
HEADERS = sorted(f for f in os.listdir(os.path.join(ROOT, "include")) if f.endswith(".h"))


def _declared_functions(headers=HEADERS):
    names = []
    for h in headers:
        src = open(os.path.join(ROOT, "include", h)).read()
        src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
        names += re.findall(r"\b(qn_[a-z0-9_]+)\s*\(", src)
    return sorted(set(names))


@pytest.fixture(scope="module")
def lib():
    from paper_1709_05069_amd import _lib
    if not os.path.exists(_lib.LIB_PATH):
        from paper_1709_05069_amd import build
        build.build()
    return _lib.load()


def test_header_declares_the_four_entry_points_of_the_step():
    names = _declared_functions(["qn.h"])
    for required in ("qn_update", "qn_gram", "qn_eig", "qn_apply", "qn_workspace_bytes",
                     "qn_update_ws", "qn_gram_ws"):
        assert required in names
    # diagnostics live in a header of their own
    assert not [n for n in names if n.startswith(("qn_probe", "qn_trace", "qn_diag"))]
    assert HEADERS == ["qn.h", "qn_diag.h"]


def test_header_is_valid_c99(tmp_path):
    # the boundary is a C ABI: the header must compile as plain C, not only as C++
    src = tmp_path / "use_qn.c"
    src.write_text('#include "qn.h"\n#include "qn_diag.h"\n'
                   'int main(void) { return QN_MAX_M > 0 && QN_TRACE_KERNELS > 0 ? 0 : 1; }\n')
    r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror",
                        "-fsyntax-only", "-I", os.path.dirname(HEADER), str(src)],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr


def test_every_declared_symbol_is_exported(lib):
    from paper_1709_05069_amd import _lib
    names = _declared_functions()
    assert len(names) >= 15
    for name in names:
        assert hasattr(lib, name), f"libqn.so does not export {name}"
    # and the binding's signature table covers the header exactly
    assert sorted(_lib.SIGNATURES) == names


def test_status_strings(lib):
    assert lib.qn_status_string(0) == b"ok"
    seen = {lib.qn_status_string(c) for c in (0, -1, -2, -3, -4, -5)}
    assert len(seen) == 6
    assert lib.qn_status_string(-99) == b"unknown status"
    assert lib.qn_kernel_name(4) == b"apply_kernel"


def test_argument_errors_are_reported_before_any_device_work(lib):
    # null pointers / bad sizes return QN_EINVAL on the host; no GPU is needed
    # because validation precedes every HIP call
    assert lib.qn_update(None, None, 10, 4, 1.0, 0.1, None, None, None) == -1
    assert lib.qn_gram(None, 10, 4, None, None, None) == -1
    assert lib.qn_eig(None, None, 4, 0.1, None, None, None, None, None) == -1
    assert lib.qn_apply(None, None, 10, 4, None, 1.0, None, None) == -1
    # sizes and scalars (pointers are never dereferenced on the host)
    p = 0x1000
    assert lib.qn_update(p, p, 0, 4, 1.0, 0.1, p, p, None) == -1        # n < 1
    assert lib.qn_update(p, p, 10, 0, 1.0, 0.1, p, p, None) == -1       # m < 1
    assert lib.qn_update(p, p, 10, 65, 1.0, 0.1, p, p, None) == -1      # m > max
    assert lib.qn_update(p, p, 10, 4, float("nan"), 0.1, p, p, None) == -1
    assert lib.qn_update(p, p, 10, 4, 1.0, 0.0, p, p, None) == -1       # lambda <= 0
    assert lib.qn_update(p, p, 10, 4, 1.0, float("inf"), p, p, None) == -1
    assert lib.qn_update_ex(p, p, 0, 10, 4, 9, 1.0, 0.1, p, p, None) == -1   # ld < n
    assert lib.qn_update_ex(p, p, 7, 10, 4, 10, 1.0, 0.1, p, p, None) == -1  # dtype
    assert lib.qn_trace_end(None, None) == -1                            # not tracing
    # the operator, its pieces and the capped step
    assert lib.qn_hinv(p, p, None, 10, 4, 0.1, p, p, None) == -1         # z missing
    assert lib.qn_hinv_ex(p, p, 0, p, 10, 4, 10, -1.0, p, p, None) == -1  # lambda <= 0
    assert lib.qn_gemv_t_ex(p, 3, p, 10, 4, 10, p, None) == -1           # dtype
    assert lib.qn_coef(p, p, p, p, 65, p, None) == -1                    # m > max
    assert lib.qn_hinv_apply_ex(p, p, 0, p, 10, 4, 10, None, p, None) == -1   # c missing
    assert lib.qn_update_bounded_ex(p, p, 0, 10, 4, 10, 1.0, 0.1, 0, p, p, p, None) == -1  # mode
    assert lib.qn_update_bounded_ex(p, p, 0, 10, 4, 10, 1.0, 0.1, 3, p, p, p, None) == -1
    assert lib.qn_tau_bound(p, p, p, None, 4, 1.0, 2, p, p, None) == -1  # secant needs Theta^T Theta
    assert lib.qn_tau_bound(p, p, p, p, 4, float("nan"), 1, p, p, None) == -1
    assert lib.qn_probe_copy(p, p, 24, None) == -1                       # not a multiple of 16
    # the workspace forms check their other arguments the same way, first
    assert lib.qn_update_ws(p, p, 0, 0, 4, 0, 1.0, 0.1, p, p, p, 1 << 30, None) == -1
    assert lib.qn_gram_ws(p, 0, 10, 65, 10, p, p, p, 1 << 30, None) == -1
    assert lib.qn_hinv_ws(p, p, 0, None, 10, 4, 10, 0.1, p, p, p, 1 << 30, None) == -1
    assert lib.qn_gemv_t_ws(p, 0, p, 10, 4, 9, p, p, 1 << 30, None) == -1
    assert lib.qn_update_bounded_ws(p, p, 0, 10, 4, 10, 1.0, 0.1, 7, p, p, p, p, 1 << 30, None) == -1
    assert lib.qn_diag_gram_ex(p, 0, None, 10, 4, 10, 5, p, p, None) == -1   # no such kernel
    assert lib.qn_diag_gram_ex(p, 0, None, 1 << 23, 4, 1 << 23, 2, p, p, None) == -1


def test_workspace_bytes_is_a_host_side_function_of_the_problem(lib):
    # no device here: 256 compute units are assumed
    f = lib.qn_workspace_bytes
    assert f(0, 4, 0) == 0 and f(10, 0, 0) == 0 and f(10, 65, 0) == 0 and f(10, 4, 9) == 0
    small = f(4096, 4, 0)
    big = max(f(1 << 40, m, dt) for m in (16, 32, 48, 64) for dt in (0, 1, 2))
    assert 0 < small < big <= 6 * 1024 * 1024
    assert f(124_000_000, 32, 0) % 256 == 0
    # monotone in n up to the point where the grid is full
    assert f(100, 32, 0) <= f(20_000, 32, 0) <= f(124_000_000, 32, 0) == f(1 << 40, 32, 0)


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    from paper_1709_05069_amd import _lib
    monkeypatch.setattr(_lib, "_LIB", None)
    monkeypatch.setattr(_lib, "LIB_PATH", str(tmp_path / "libqn.so"))
    with pytest.raises(RuntimeError, match="no fallback"):
        _lib.load()
