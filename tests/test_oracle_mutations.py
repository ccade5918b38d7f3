"""Do the pins bite?  Each case plants one plausible mistake in a COPY of the oracle's C source (a
dropped term, a wrong sign, a wrong index, a misplaced decay), builds it on the CPU and runs the pin
tests against it: at least one pin must fail.  The shipped oracle is never modified."""
import ctypes
import os
import subprocess

import pytest

from oracle import oracle
from tests import test_oracle_bwd_pins as bwd_pins
from tests import test_oracle_pins as fwd_pins

SRC = os.path.join(os.path.dirname(oracle.__file__), "gla_oracle.c")

# (name, text to find, replacement, which occurrence)
MUTATIONS = [
    ("fwd_decay_also_on_new_term", "Si[j] = a * Si[j] + kt[i] * vt[j]", "Si[j] = a * (Si[j] + kt[i] * vt[j])", 0),
    ("fwd_decay_sign", "const double a = exp(gt[i]);", "const double a = exp(-gt[i]);", 0),
    ("fwd_scale_dropped", "const double qi = scale * qt[i];", "const double qi = qt[i];", 0),
    ("fwd_decay_on_columns", "const double a = exp(gt[i]);", "const double a = exp(gt[(i + 1) % dk]);", 0),
    ("local_gcum_exclusive", "acc += g[ok + (size_t)t * sk + i];\n                        G_cum[ok + (size_t)t * sk + i] = acc;",
     "G_cum[ok + (size_t)t * sk + i] = acc;\n                        acc += g[ok + (size_t)t * sk + i];", 0),
    ("scan_decay_on_local_too", "cur[(size_t)i * dv + j] = a * cur[(size_t)i * dv + j] + loc[(size_t)i * dv + j];",
     "cur[(size_t)i * dv + j] = a * (cur[(size_t)i * dv + j] + loc[(size_t)i * dv + j]);", 0),
    ("scan_decay_sign", "const double a = exp(gt[i]);", "const double a = exp(-gt[i]);", 1),
    ("apply_decay_dropped", "const double w = scale * qt[i] * exp(Gt[i]);", "const double w = scale * qt[i];", 0),
    ("apply_scale_dropped", "const double w = scale * qt[i] * exp(Gt[i]);", "const double w = qt[i] * exp(Gt[i]);", 0),
    ("bwd_dg_alpha_dropped", "dg[ok + t * sk + i] = a * accg;", "dg[ok + t * sk + i] = accg;", 0),
    ("bwd_dg_wrong_state", "accg += d * Sp[i * dv + j];", "accg += d * St[i * dv + j];", 0),
    ("bwd_carry_decay_dropped", "E[i * dv + j] = a * dS[i * dv + j];", "E[i * dv + j] = dS[i * dv + j];", 0),
    ("bwd_dq_scale_dropped", "dq[ok + t * sk + i] = scale * accq;", "dq[ok + t * sk + i] = accq;", 0),
    ("bwd_dq_state_before_token", "accq += dOt[j] * St[i * dv + j];", "accq += dOt[j] * Sp[i * dv + j];", 0),
    ("bwd_dS_scale_dropped", "const double d = E[i * dv + j] + scale * qt[i] * dOt[j];",
     "const double d = E[i * dv + j] + qt[i] * dOt[j];", 0),
    ("bwd_dk_uses_carry_only", "acck += d * vt[j];", "acck += E[i * dv + j] * vt[j];", 0),
    ("bwd_dv_transposed", "dv_out[ov + t * sv + j] += kt[i] * d;", "dv_out[ov + t * sv + j] += kt[i] * dS[(j % dk) * dv + (i % dv)];", 0),
]


def pins():
    """Every pin as a zero-argument callable."""
    calls = []
    for mod in (fwd_pins, bwd_pins):
        for name in sorted(dir(mod)):
            fn = getattr(mod, name)
            if not name.startswith("test_") or not callable(fn):
                continue
            marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
            if not marks:
                calls.append((name, fn))
                continue
            combos = [{}]
            for m in marks:
                keys = [k.strip() for k in m.args[0].split(",")]
                new = []
                for val in m.args[1]:
                    vals = val if len(keys) > 1 else (val,)
                    for c in combos:
                        new.append({**c, **dict(zip(keys, vals))})
                combos = new
            for c in combos:
                calls.append(("%s%s" % (name, c), (lambda f=fn, kw=c: f(**kw))))
    return calls


@pytest.mark.parametrize("mutation", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught(mutation, tmp_path, monkeypatch):
    name, old, new, nth = mutation
    text = open(SRC).read()
    pos = -1
    for _ in range(nth + 1):
        pos = text.index(old, pos + 1)
    mutated = text[:pos] + new + text[pos + len(old):]
    src, lib = tmp_path / "mut.c", tmp_path / "libmut.so"
    src.write_text(mutated)
    subprocess.check_call(["gcc", "-O1", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", str(lib), str(src), "-lm"])
    monkeypatch.setattr(oracle, "_lib", oracle._bind(ctypes.CDLL(str(lib))))
    caught = []
    for pin_name, fn in pins():
        try:
            fn()
        except AssertionError:
            caught.append(pin_name)
    assert caught, "no pin noticed the planted mistake '%s'" % name


def test_unmutated_oracle_passes_the_same_harness():
    for pin_name, fn in pins():
        fn()
