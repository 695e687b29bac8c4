"""Do the pins bite?  Each case plants one plausible mistake in a copy of the
oracle's C source (on the CPU, in a temporary directory), builds it, and runs
the whole pin suite of test_oracle_pins.py against the mutant: at least one pin
must fail.  The real oracle is restored afterwards."""
import os
import subprocess

import pytest

import oracle
import test_oracle_pins as pins

SRC = os.path.join(os.path.dirname(oracle.__file__), "qn_oracle.c")

MUTANTS = [
    ("mean divisor", "mean[i] = s / (double)m;", "mean[i] = s / (double)(m + 1);"),
    ("centring sign", "(int64_t)k * ld + i) - mean[i];", "(int64_t)k * ld + i) + mean[i];"),
    ("gram drops a row",
     "for (int64_t i = 0; i < n; ++i)\n                s += G[(int64_t)a * n + i] * G[(int64_t)b * n + i];",
     "for (int64_t i = 0; i < n - 1; ++i)\n                s += G[(int64_t)a * n + i] * G[(int64_t)b * n + i];"),
    ("rotation sign", "const double sn = t * cs;", "const double sn = -t * cs;"),
    ("ascending sort", "if (mu[l] > mu[best])", "if (mu[l] < mu[best])"),
    ("sigma is the eigenvalue", "sigma[k] = mu[k] > 0.0 ? sqrt(mu[k]) : 0.0;",
     "sigma[k] = mu[k] > 0.0 ? mu[k] : 0.0;"),
    ("strict cutoff", "sigma[j] >= lambda * sigma[0]", "sigma[j] > lambda * sigma[0]"),
    ("eq.4 without 1/sigma", "mapped[i] += alpha / sigma[k] * y[i];", "mapped[i] += alpha * y[i];"),
    ("eq.4 with 1/sigma^2", "mapped[i] += alpha / sigma[k] * y[i];",
     "mapped[i] += alpha / (sigma[k] * sigma[k]) * y[i];"),
    ("z_perp sign", "zperp[i] -= alpha * u[i];", "zperp[i] += alpha * u[i];"),
    ("y_k built from G", "ty += Theta[(int64_t)l * n + i] * vk[l];", "ty += G[(int64_t)l * n + i] * vk[l];"),
    ("u_k not normalised", "u[i] /= nrm;", "u[i] /= nrm2;"),
    ("eq.2 sign of tau", "theta_new[i] = theta_bar[i] - tau * step[i];",
     "theta_new[i] = theta_bar[i] + tau * step[i];"),
    ("streaming w wrong", "w_acc[a] += d[a] * gbar;", "w_acc[a] += d[a];"),
    ("streaming Gram uncentred", "d[k] -= gbar;", "d[k] -= 0.0;"),
    ("alpha without 1/sigma", "a /= sg[k];", "a /= 1.0;"),
    ("closed form Theta + G", "corr += c[k] * (th - gr);", "corr += c[k] * (th + gr);"),
    ("closed form correction sign", "theta_new[i] = tbar - tau * (gbar + corr);",
     "theta_new[i] = tbar - tau * (gbar - corr);"),
    ("bf16 shift", "<< 16;", "<< 15;"),
    ("f16 exponent bias", "v = ldexp((double)(frac | 0x400), e - 25);",
     "v = ldexp((double)(frac | 0x400), e - 24);"),
    ("f16 subnormals dropped", "v = ldexp((double)frac, -24);", "v = 0.0;"),
    ("transposed eigenvector storage", "c[r] += Vl[k * m + r] * a / sg[k];",
     "c[r] += Vl[r * m + k] * a / sg[k];"),
    ("cap from the eigenvalue", "return cap_tau(tau, s2 > 0.0, sqrt(s2), sigma_max);",
     "return cap_tau(tau, s2 > 0.0, s2, sigma_max);"),
    ("cap is a floor", "return fmin(tau, 1.0 / smax);", "return fmax(tau, 1.0 / smax);"),
    ("secant quotient inverted", "const double q = sqrt(g2) / sqrt(y2);",
     "const double q = sqrt(y2) / sqrt(g2);"),
    ("secant norm from G", "yv += Theta[(int64_t)r * n + i] * V[k * m + r];",
     "yv += G[(int64_t)r * n + i] * V[k * m + r];"),
    ("secant from Gram without the root", "sigma[k] / sqrt(y2 > 0.0 ? y2 : 0.0);",
     "sigma[k] / (y2 > 0.0 ? y2 : 0.0);"),
    ("secant from Gram transposed V", "row += Ct[q * m + r] * V[k * m + q];",
     "row += Ct[q * m + r] * V[q * m + k];"),
]


def _pin_calls():
    calls = []
    for name in sorted(dir(pins)):
        fn = getattr(pins, name)
        if not name.startswith("test_") or not callable(fn):
            continue
        marks = [mk for mk in getattr(fn, "pytestmark", []) if mk.name == "parametrize"]
        if not marks:
            calls.append((name, fn, ()))
            continue
        argnames, argvalues = marks[0].args[0], marks[0].args[1]
        nargs = len([a for a in argnames.split(",") if a.strip()])
        for v in argvalues:
            calls.append((name, fn, tuple(v) if nargs > 1 else (v,)))
    return calls


def _failing_pins():
    failed = []
    for name, fn, args in _pin_calls():
        try:
            fn(*args)
        except Exception:                 # an assertion, or the oracle giving up
            failed.append(name)
    return failed


def test_the_real_oracle_passes_when_run_this_way():
    assert len(_pin_calls()) >= 40
    assert _failing_pins() == []


@pytest.mark.parametrize("label,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(label, old, new, tmp_path, monkeypatch):
    text = open(SRC).read()
    assert text.count(old) == 1, f"mutation site for '{label}' not unique"
    mutant_c = tmp_path / "qn_oracle.c"
    mutant_c.write_text(text.replace(old, new))
    (tmp_path / "qn_oracle.h").write_text(open(SRC[:-2] + ".h").read())
    so = tmp_path / "libmutant.so"
    subprocess.check_call(["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-o", str(so),
                           str(mutant_c), "-lm"])
    monkeypatch.setattr(oracle, "_LIB", oracle.load_library(str(so)))
    failed = _failing_pins()
    assert failed, f"no pin notices: {label}"
