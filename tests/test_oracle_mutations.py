"""The pins must notice plausible mistakes.  Each case below plants one mistake in a copy of the
oracle's C source (a wrong sign, a dropped factor, a wrong constant or index, a different reading
of the self term), builds it, routes the oracle front end through it and checks that at least one
pin of tests/test_oracle_pins.py fails.  Everything here runs on the CPU."""
import inspect
import os
import subprocess
import tempfile

import pytest

import oracle
import test_oracle_pins as pins

SRC = os.path.join(os.path.dirname(oracle.__file__), "sdkde_oracle.c")

MUTATIONS = [
    ("score numerator sign", "num[k] += -(p[k] - xj[k]) * w;", "num[k] += (p[k] - xj[k]) * w;"),
    ("score misses a factor h", "num[k] / (h * h * den)", "num[k] / (h * den)"),
    ("score numerator coordinate reversed", "num[k] += -(p[k] - xj[k]) * w;", "num[k] += -(p[k] - xj[d - 1 - k]) * w;"),
    ("kernel exponent h^2 instead of 2h^2", "a[j] = -r2 / (2.0 * h * h);", "a[j] = -r2 / (h * h);"),
    ("distance uses first coordinate only", "for (int32_t k = 0; k < d; ++k) {\n            double diff", "for (int32_t k = 0; k < 1; ++k) {\n            double diff"),
    ("sample row stride", "const double *xj = X + j * (int64_t)d;\n        double r2", "const double *xj = X + j;\n        double r2"),
    ("leave-one-out score", "double w = exp(a[j] - amax);\n                    den += w;", "double w = (a[j] == 0.0) ? 0.0 : exp(a[j] - amax);\n                    den += w;"),
    ("debias h^2 instead of h^2/2", "X[t] + 0.5 * h * h * S[t]", "X[t] + h * h * S[t]"),
    ("debias sign", "X[t] + 0.5 * h * h * S[t]", "X[t] - 0.5 * h * h * S[t]"),
    ("density misses (2 pi)^(d/2)", " - 0.5 * (double)d * log(two_pi);", ";"),
    ("density h instead of h^d", "(double)d * log(h)", "log(h)"),
    ("density misses 1/n", "-log((double)n) - ", "- "),
    ("log-sum-exp forgets the shift", "double lp = amax + log(sum) + lognorm;", "double lp = log(sum) + lognorm;"),
    ("laplace factor d instead of d/2", "double factor = 1.0 + 0.5 * (double)d + a[j];", "double factor = 1.0 + (double)d + a[j];"),
    ("laplace factor sign of r^2 term", "double factor = 1.0 + 0.5 * (double)d + a[j];", "double factor = 1.0 + 0.5 * (double)d - a[j];"),
]


def _pin_functions():
    out = []
    for name, fn in inspect.getmembers(pins, inspect.isfunction):
        if name.startswith("test_") and name not in ("test_oracle_rejects_bad_arguments",
                                                     "test_silverman_rule_reduces_to_1d_textbook_constant",
                                                     "test_generators_are_seeded_and_shaped"):
            out.append(fn)
    return out


def _run_pins():
    """Runs every pin; returns the names of those that fail."""
    failed = []
    cloud = pins.make_cloud()
    for fn in _pin_functions():
        params = inspect.signature(fn).parameters
        marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
        cases = [()]
        if marks:
            vals = marks[0].args[1]
            cases = [v if isinstance(v, tuple) else (v,) for v in vals]
        for case in cases:
            args = list(case) + ([cloud] if "cloud" in params else [])
            try:
                fn(*args)
            except Exception:       # an assertion, a ValueError from a NaN, ...
                failed.append(fn.__name__)
                break
    return failed


def test_pins_pass_on_the_real_oracle():
    oracle.use_library(None)
    assert _run_pins() == []


@pytest.mark.parametrize("what,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught(what, old, new):
    text = open(SRC).read()
    assert text.count(old) >= 1, f"mutation target for '{what}' not found in the oracle source"
    with tempfile.TemporaryDirectory() as tmp:
        src = os.path.join(tmp, "mutant.c")
        lib = os.path.join(tmp, "libmutant.so")
        open(src, "w").write(text.replace(old, new, 1))
        subprocess.check_call(["gcc", "-O1", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-w", "-o", lib, src, "-lm"])
        try:
            oracle.use_library(lib)
            failed = _run_pins()
        finally:
            oracle.use_library(None)
    assert failed, f"no pin noticed: {what}"
