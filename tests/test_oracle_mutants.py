"""Are the pins strong enough?  Plant one plausible mistake at a time in a copy
of the oracle's C source (a flipped sign, a dropped term, a wrong operand or
index, a swapped order, fused multiply-add), build it, and check that at least
one pin test fails for every such mutant.  CPU only; the mistakes are planted in
the oracle, never in the GPU path."""
import ctypes
import inspect
import itertools
import os
import sys

import pytest

from conftest import load_golden
from oracle import build as oracle_build
from oracle import odsgd_oracle as oracle

import test_oracle_dcasgd_pins as dc_pins
import test_oracle_pins as sgd_pins

SRC = open(oracle_build.SRC).read()

# (name, text to find, replacement, how many times it must occur, extra cflags)
MUTANTS = [
    ("sum_sign", "s = s + g[m][i];", "s = s - g[m][i];", 1),
    ("sum_drops_last_worker", "for (int m = 1; m < M; ++m)\n            s = s + g[m][i];",
     "for (int m = 1; m < M - 1; ++m)\n            s = s + g[m][i];", 1),
    ("sum_descending_order", "for (int m = 1; m < M; ++m)\n            s = s + g[m][i];",
     "for (int m = M - 1; m >= 1; --m)\n            s = s + g[m][i];", 1),
    ("scale_dropped", "real gb = s * scale;", "real gb = s;", 1),
    ("default_scale_not_mean", "return (real)1 / (real)M;", "return (real)1;", 1),
    ("global_decay_wrong_operand", "real r = weight_decay * w0;\n        real d = gb + r;",
     "real r = weight_decay * v0;\n        real d = gb + r;", 1),
    ("global_decay_sign", "real d = gb + r;", "real d = gb - r;", 1),
    ("momentum_wrong_operand", "real a = momentum * v0;", "real a = momentum * w0;", 1),
    ("velocity_sign", "real v1 = a - b;", "real v1 = a + b;", 1),
    ("weight_step_sign", "real w1 = w0 + v1;", "real w1 = w0 - v1;", 1),
    ("lr_dropped", "real b = lr * d;", "real b = d;", 1),
    ("stores_swapped", "v[i] = v1;\n        w[i] = w1;", "v[i] = w1;\n        w[i] = v1;", 1),
    ("local_decay_dropped", "real dm = g[m][i] + r;\n            real pm", "real dm = g[m][i];\n            real pm", 1),
    ("local_decay_sign", "real dm = g[m][i] + r;\n            real pm", "real dm = g[m][i] - r;\n            real pm", 1),
    ("local_step_sign", "real pm = local_lr * dm;\n            u[m][i] = w0 - pm;",
     "real pm = local_lr * dm;\n            u[m][i] = w0 + pm;", 1),
    ("local_uses_global_lr", "(n, M, w, g, u, -1, local_lr, weight_decay);", "(n, M, w, g, u, -1, lr, weight_decay);", 1),
    ("local_worker_filter_inverted", "if (worker >= 0 && m != worker)", "if (worker >= 0 && m == worker)", 4),
    ("local_reads_new_weights",
     "ODSGD_NAME(odsgd_oracle_local)(n, M, w, g, u, -1, local_lr, weight_decay);\n"
     "    ODSGD_NAME(odsgd_oracle_global)(n, M, w, v, g, lr, momentum, weight_decay,\n"
     "                                    grad_scale);",
     "ODSGD_NAME(odsgd_oracle_global)(n, M, w, v, g, lr, momentum, weight_decay,\n"
     "                                    grad_scale);\n"
     "    ODSGD_NAME(odsgd_oracle_local)(n, M, w, g, u, -1, local_lr, weight_decay);", 1),
    ("warmup_hands_out_momentum", "u[m][i] = w[i];", "u[m][i] = v[i];", 1),
    ("dc_delay_sign", "real dlt = w0 - u[m][i];", "real dlt = u[m][i] - w0;", 2),
    ("dc_gradient_not_squared", "real gg = gm * gm;", "real gg = gm;", 2),
    ("dcc_lambda_dropped", "real c2 = c1 * lambda;", "real c2 = c1;", 1),
    ("dc_compensation_sign", "real em = dm + c2;", "real em = dm - c2;", 2),
    ("dca_mean_square_weights", "real s2 = one_minus_decay * gg;", "real s2 = ms_decay * gg;", 1),
    ("dca_mean_square_decay_dropped", "real s1 = ms_decay * ms[m][i];", "real s1 = ms[m][i];", 1),
    ("dca_state_not_stored", "ms[m][i] = msq;", ";", 1),
    ("dca_epsilon_dropped", "real rad = msq + epsilon;", "real rad = msq;", 1),
    ("dca_no_square_root", "real den = ODSGD_SQRT(rad);", "real den = rad;", 1),
    ("dca_multiplies_by_root", "real lam = lambda / den;", "real lam = lambda * den;", 1),
    ("dca_uses_plain_lambda", "real c2 = c1 * lam;", "real c2 = c1 * lambda;", 1),
    ("local_momentum_dropped", "real am = local_momentum * lv[m][i];", "real am = lv[m][i];", 1),
    ("local_velocity_sign", "real lv1 = am - pm;", "real lv1 = am + pm;", 1),
    ("local_velocity_not_stored", "lv[m][i] = lv1;", ";", 1),
    ("local_velocity_subtracted", "u[m][i] = w0 + lv1;", "u[m][i] = w0 - lv1;", 1),
    ("local_momentum_decay_dropped", "real dm = g[m][i] + r;\n            real am", "real dm = g[m][i];\n            real am", 1),
]
FLAG_MUTANTS = [("fused_multiply_add", ["-ffp-contract=fast", "-mfma"])]


def _cases(module, fixtures):
    """Every test function of a pin module, expanded over its parametrize marks."""
    out = []
    for name, fn in sorted(vars(module).items()):
        if not name.startswith("test_") or not callable(fn):
            continue
        axes = []
        for mark in getattr(fn, "pytestmark", []):
            if mark.name == "parametrize":
                argnames = [a.strip() for a in mark.args[0].split(",")]
                vals = [v if isinstance(v, (tuple, list)) and len(argnames) > 1 else (v,) for v in mark.args[1]]
                axes.append([dict(zip(argnames, v)) for v in vals])
        for combo in itertools.product(*axes) if axes else [()]:
            kwargs = {}
            for d in combo:
                kwargs.update(d)
            for p in inspect.signature(fn).parameters:
                if p in fixtures:
                    kwargs[p] = fixtures[p]
            out.append((name, fn, kwargs))
    return out


def _first_failing_pin(cases):
    for name, fn, kwargs in cases:
        try:
            fn(**kwargs)
        except AssertionError:
            return name
        except Exception as e:  # a mutant may also blow up inside a pin
            return "%s (%s)" % (name, type(e).__name__)
    return None


@pytest.fixture(scope="module")
def pin_cases():
    fixtures = {"golden_w2": load_golden("hand_expanded_w2.txt"),
                "golden_dcasgd": load_golden("hand_expanded_dcasgd.txt")}
    return _cases(sgd_pins, fixtures) + _cases(dc_pins, fixtures)


def _with_library(path, cases):
    saved = oracle._LIB
    oracle._LIB = ctypes.CDLL(path)
    try:
        return _first_failing_pin(cases)
    finally:
        oracle._LIB = saved


def test_unmodified_oracle_passes_every_pin(pin_cases, tmp_path):
    src = tmp_path / "oracle_copy.c"
    src.write_text(SRC)
    lib = oracle_build.build(force=True, lib=str(tmp_path / "libcopy.so"), src=str(src))
    assert _with_library(lib, pin_cases) is None


@pytest.mark.parametrize("mutant", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_text_mutant_is_caught(mutant, pin_cases, tmp_path):
    name, old, new, count = mutant
    assert SRC.count(old) == count, "mutation site of %s not found %d time(s): the oracle changed" % (name, count)
    src = tmp_path / (name + ".c")
    src.write_text(SRC.replace(old, new))
    lib = oracle_build.build(force=True, lib=str(tmp_path / ("lib" + name + ".so")), src=str(src),
                             extra_cflags=["-Wno-unused-variable", "-Wno-unused-parameter",
                                           "-Wno-unused-but-set-variable"])
    killer = _with_library(lib, pin_cases)
    assert killer is not None, "no pin notices the planted mistake '%s'" % name


@pytest.mark.parametrize("mutant", FLAG_MUTANTS, ids=[m[0] for m in FLAG_MUTANTS])
def test_flag_mutant_is_caught(mutant, pin_cases, tmp_path):
    name, flags = mutant
    src = tmp_path / (name + ".c")
    src.write_text(SRC)
    lib = oracle_build.build(force=True, lib=str(tmp_path / ("lib" + name + ".so")), src=str(src),
                             extra_cflags=flags)
    assert _with_library(lib, pin_cases) is not None, "no pin notices '%s'" % name
