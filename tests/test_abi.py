"""The C ABI without a GPU: the library loads, exports every function that
include/qn.h declares, and its host-only entry points behave."""
import os
import re
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "qn.h")


def _declared_functions():
    src = open(os.path.join(ROOT, "include", "qn.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    names = re.findall(r"\b(qn_[a-z0-9_]+)\s*\(", src)
    return sorted(set(names))


@pytest.fixture(scope="module")
def lib():
    from paper_1709_05069_amd import _lib
    if not os.path.exists(_lib.LIB_PATH):
        from paper_1709_05069_amd import build
        build.build()
    return _lib.load()


def test_header_declares_the_four_entry_points_of_the_step():
    names = _declared_functions()
    for required in ("qn_update", "qn_gram", "qn_eig", "qn_apply"):
        assert required in names


def test_header_is_valid_c99(tmp_path):
    # the boundary is a C ABI: the header must compile as plain C, not only as C++
    src = tmp_path / "use_qn.c"
    src.write_text('#include "qn.h"\nint main(void) { return QN_MAX_M > 0 ? 0 : 1; }\n')
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
    seen = {lib.qn_status_string(c) for c in (0, -1, -2, -3, -4)}
    assert len(seen) == 5
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


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    from paper_1709_05069_amd import _lib
    monkeypatch.setattr(_lib, "_LIB", None)
    monkeypatch.setattr(_lib, "LIB_PATH", str(tmp_path / "libqn.so"))
    with pytest.raises(RuntimeError, match="no fallback"):
        _lib.load()
