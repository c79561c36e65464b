"""Do the pins bite?  Each case plants ONE plausible mistake in a copy of an oracle source (a dropped term, a wrong
sign or index, a transposed operand, an off-by-one), builds the copy on the CPU, binds it in place of the oracle's
library and runs the pin tests of that source: at least one of them must fail.  The shipped sources themselves are
never touched, and nothing here runs on a GPU."""
import ctypes
import importlib
import inspect
import os
import subprocess

import pytest

import oracle

HERE = os.path.dirname(os.path.abspath(__file__))
ORACLE_DIR = os.path.dirname(os.path.abspath(oracle.__file__))
SOURCES = ("ptqtp_oracle.c", "ptqtp_quantizer_oracle.c", "ptqtp_block_oracle.c")

# (source file, pin module, what is planted, text to find, replacement)
MUTATIONS = [
    ("ptqtp_oracle.c", "test_oracle_pins", "scales of the two planes swapped",
     "acc += al1 * s1 + al2 * s2;", "acc += al2 * s1 + al1 * s2;"),
    ("ptqtp_oracle.c", "test_oracle_pins", "second plane dropped",
     "acc += al1 * s1 + al2 * s2;", "acc += al1 * s1;"),
    ("ptqtp_oracle.c", "test_oracle_pins", "second plane subtracted",
     "acc += al1 * s1 + al2 * s2;", "acc += al1 * s1 - al2 * s2;"),
    ("ptqtp_oracle.c", "test_oracle_pins", "scale of the mirrored group",
     "double al1 = ptqtp_oracle_half_to_double(a1[n * NG + g]);", "double al1 = ptqtp_oracle_half_to_double(a1[n * NG + (NG - 1 - g)]);"),
    ("ptqtp_oracle.c", "test_oracle_pins", "scales indexed [group][row]",
     "double al2 = ptqtp_oracle_half_to_double(a2[n * NG + g]);", "double al2 = ptqtp_oracle_half_to_double(a2[g * N + n]);"),
    ("ptqtp_oracle.c", "test_oracle_pins", "output written transposed",
     "y[m * N + n] = acc;", "y[n * M + m] = acc;"),
    ("ptqtp_oracle.c", "test_oracle_pins", "group starts one column late",
     "for (int64_t k = g * G; k < (g + 1) * G; ++k) {", "for (int64_t k = g * G + 1; k < (g + 1) * G; ++k) {"),
    ("ptqtp_oracle.c", "test_oracle_pins", "scale applied once per row, with the last group's value",
     "acc += al1 * s1 + al2 * s2;", "acc = (g == NG - 1) ? al1 * (acc + s1) + al2 * s2 : acc + s1;"),
    ("ptqtp_oracle.c", "test_oracle_pins", "bound without the absolute value of the scales",
     "bnd += fabs(al1) * b1 + fabs(al2) * b2;", "bnd += al1 * b1 + al2 * b2;"),
    ("ptqtp_oracle.c", "test_oracle_pins", "binary16 exponent bias off by one",
     "else               v = ldexp((double)(1024 + frac), e - 25);", "else               v = ldexp((double)(1024 + frac), e - 24);"),
    ("ptqtp_oracle.c", "test_oracle_pins", "binary16 subnormals flushed to zero",
     "if (e == 0)        v = ldexp((double)frac, -24);", "if (e == 0)        v = 0.0;"),
    ("ptqtp_oracle.c", "test_oracle_pins", "2-bit fields packed from the top of the byte",
     "byte |= code << (2 * j);", "byte |= code << (2 * (3 - j));"),
    ("ptqtp_oracle.c", "test_oracle_pins", "codes 01 and 11 read the wrong way round",
     "T[n * K + 4 * b + j] = (int8_t)(code == 3u ? -1 : (int)code);", "T[n * K + 4 * b + j] = (int8_t)(code == 1u ? -1 : (code == 3u ? 1 : 0));"),
    ("ptqtp_oracle.c", "test_oracle_pins", "unused code 10 accepted",
     "if (code == 2u) return ORACLE_ERR_CODE;", "if (code == 2u) code = 0u;"),
    ("ptqtp_oracle.c", "test_oracle_pins", "memory model with one scale per (row, group)",
     "return 2 * n * d * 2 + groups * 2 * n * 16;", "return 2 * n * d * 2 + groups * n * 16;"),
    ("ptqtp_quantizer_oracle.c", "test_quantizer_oracle_pins", "off-diagonal of the inverse with the wrong sign",
     "double i11 = A22 * rdet, i12 = -A12 * rdet, i22 = A11 * rdet;", "double i11 = A22 * rdet, i12 = A12 * rdet, i22 = A11 * rdet;"),
    ("ptqtp_quantizer_oracle.c", "test_quantizer_oracle_pins", "diagonal of the inverse not swapped",
     "double i11 = A22 * rdet, i12 = -A12 * rdet, i22 = A11 * rdet;", "double i11 = A11 * rdet, i12 = -A12 * rdet, i22 = A22 * rdet;"),
    ("ptqtp_quantizer_oracle.c", "test_quantizer_oracle_pins", "ridge term left out",
     "double A11 = (double)s11 + lam, A22 = (double)s22 + lam;", "double A11 = (double)s11, A22 = (double)s22;"),
    ("ptqtp_quantizer_oracle.c", "test_quantizer_oracle_pins", "last minimum instead of the first",
     "if (e < best) { best = e; bc1 = c1; bc2 = c2; }", "if (e <= best) { best = e; bc1 = c1; bc2 = c2; }"),
    ("ptqtp_quantizer_oracle.c", "test_quantizer_oracle_pins", "candidate order with the second plane outermost",
     "const double v = (double)c1 * a1 + (double)c2 * a2;", "const double v = (double)c2 * a1 + (double)c1 * a2;"),
    ("ptqtp_quantizer_oracle.c", "test_quantizer_oracle_pins", "zero initialised to -1",
     "const int8_t s = (int8_t)(w < 0.0 ? -1 : 1);", "const int8_t s = (int8_t)(w <= 0.0 ? -1 : 1);"),
    ("ptqtp_quantizer_oracle.c", "test_quantizer_oracle_pins", "stopping rule on the squared norm",
     "if (sqrt(sum) < eps) break;", "if (sum < eps) break;"),
    ("ptqtp_quantizer_oracle.c", "test_quantizer_oracle_pins", "right-hand side of the second plane from the first",
     "B2 += t2[j] * wf;", "B2 += t1[j] * wf;"),
    ("ptqtp_quantizer_oracle.c", "test_quantizer_oracle_pins", "condition-number threshold 1e12 instead of 1e6",
     "if (!(kappa < 1.0e6)) {", "if (!(kappa < 1.0e12)) {"),
    ("ptqtp_quantizer_oracle.c", "test_quantizer_oracle_pins", "regularisation grows with kappa instead of its square root",
     "const double grow = sqrt(kappa / 1.0e6);", "const double grow = kappa / 1.0e6;"),
    ("ptqtp_quantizer_oracle.c", "test_quantizer_oracle_pins", "regularisation capped at 2 instead of 1",
     "if (!(nl <= 1.0)) nl = 1.0;", "if (!(nl <= 2.0)) nl = 2.0;"),
    ("ptqtp_quantizer_oracle.c", "test_quantizer_oracle_pins", "regularisation not capped",
     "if (!(nl <= 1.0)) nl = 1.0;", "if (nl != nl) nl = 1.0;"),
    ("ptqtp_quantizer_oracle.c", "test_quantizer_oracle_pins", "binary16 rounding towards zero",
     "if (rem > 0.5 || (rem == 0.5 && fmod(r, 2.0) == 1.0)) r += 1.0;", "if (rem > 1.5) r += 1.0;"),
    ("ptqtp_block_oracle.c", "test_block_oracle_pins", "silu with the sign of the exponent flipped",
     "return z / (1.0 + exp(-z));", "return z / (1.0 + exp(z));"),
    ("ptqtp_block_oracle.c", "test_block_oracle_pins", "sigmoid alone instead of z * sigmoid",
     "return z / (1.0 + exp(-z));", "return 1.0 / (1.0 + exp(-z));"),
    ("ptqtp_block_oracle.c", "test_block_oracle_pins", "gate and up halves swapped",
     "ptqtp_oracle_silu(y[m * 2 * I + i]) * y[m * 2 * I + I + i]",
     "ptqtp_oracle_silu(y[m * 2 * I + I + i]) * y[m * 2 * I + i]"),
    ("ptqtp_block_oracle.c", "test_block_oracle_pins", "gate and up interleaved instead of stacked",
     "ptqtp_oracle_silu(y[m * 2 * I + i]) * y[m * 2 * I + I + i]",
     "ptqtp_oracle_silu(y[m * 2 * I + 2 * i]) * y[m * 2 * I + 2 * i + 1]"),
    ("ptqtp_block_oracle.c", "test_block_oracle_pins", "residual subtracted",
     "out[i] = y[i] + half_bits_to_double(r[i]);", "out[i] = y[i] - half_bits_to_double(r[i]);"),
    ("ptqtp_block_oracle.c", "test_block_oracle_pins", "residual widened with the exponent off by one",
     "else              v = ldexp((double)(1024 + frac), e - 25);", "else              v = ldexp((double)(1024 + frac), e - 24);"),
    ("ptqtp_block_oracle.c", "test_block_oracle_pins", "binary16 rounding with an 11-bit fraction",
     "double quantum = ldexp(1.0, lead - 10);", "double quantum = ldexp(1.0, lead - 11);"),
    ("ptqtp_block_oracle.c", "test_block_oracle_pins", "binary16 rounding: ties away from zero",
     "double q = nearbyint(a / quantum) * quantum;", "double q = round(a / quantum) * quantum;"),
    ("ptqtp_block_oracle.c", "test_block_oracle_pins", "binary16 rounding: no overflow to infinity",
     "if (q >= 65520.0) q = INFINITY;", ""),
    ("ptqtp_block_oracle.c", "test_block_oracle_pins", "binary16 rounding: no subnormal range",
     "if (lead < -14) lead = -14;", ""),
    ("ptqtp_block_oracle.c", "test_block_oracle_pins", "binary16 rounding: sign lost",
     "return v < 0 ? -q : q;", "return q;"),
]


def _build_mutant(tmp_path, source, find, replace):
    text = open(os.path.join(ORACLE_DIR, source)).read()
    assert text.count(find) == 1, f"the text to mutate must occur exactly once in {source}: {find!r}"
    files = []
    for name in SOURCES:
        dst = tmp_path / name
        body = open(os.path.join(ORACLE_DIR, name)).read()
        dst.write_text(body.replace(find, replace) if name == source else body)
        files.append(str(dst))
    lib = tmp_path / "libmutant.so"
    subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off", "-o", str(lib), *files, "-lm"])
    return str(lib)


def _run_pins(module_name):
    """Run every fixture-free pin test of a module (parametrised ones over their argument lists); the names that fail."""
    mod = importlib.import_module(module_name)
    failed = []
    for name, fn in sorted(vars(mod).items()):
        if not name.startswith("test_") or not callable(fn):
            continue
        marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
        params = inspect.signature(fn).parameters
        if len(marks) > 1 or (not marks and params):
            continue                                  # needs fixtures or stacked parametrisation: not driven from here
        cases = [()]
        if marks:
            names = [a.strip() for a in marks[0].args[0].split(",")]
            cases = [c if isinstance(c, (tuple, list)) and len(names) > 1 else (c,) for c in marks[0].args[1]]
        for case in cases:
            try:
                fn(*case)
            except (Exception, pytest.fail.Exception):   # an assertion, an unmet pytest.raises, or an error the mistake provokes
                failed.append(name)
                break
    return failed


def test_pins_pass_on_the_shipped_oracle():
    for module in ("test_oracle_pins", "test_quantizer_oracle_pins", "test_block_oracle_pins"):
        assert _run_pins(module) == []


@pytest.mark.parametrize("source,module,what,find,replace", MUTATIONS, ids=[m[2] for m in MUTATIONS])
def test_planted_mistake_is_caught(tmp_path, monkeypatch, source, module, what, find, replace):
    mutant = oracle._bind(ctypes.CDLL(_build_mutant(tmp_path, source, find, replace)))
    oracle._load()                                    # make sure the real library is what gets restored
    monkeypatch.setattr(oracle, "_lib", mutant)
    failed = _run_pins(module)
    assert failed, f"no pin notices: {what}"
