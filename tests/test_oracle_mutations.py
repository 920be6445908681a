"""Do the pins have teeth?  Each case plants one plausible mistake in a temporary copy of the C oracle (never in
the tree), rebuilds it, and requires that at least one pin of the corresponding pin module fails.  CPU only."""
import ctypes
import importlib
import os
import subprocess
import sys

import pytest

from oracle import oracle as O

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(os.path.dirname(HERE), "oracle", "meft_oracle.c")

# (name, text in the source, replacement, pin module that has to notice)
MUTANTS = [
    ("router_bias_dropped", "+ (bias ? (double)bias[b] : 0.0);", ";", "test_oracle_pins"),
    ("ties_to_the_higher_index", "by_score_desc_id_asc", None, "test_oracle_pins"),     # handled below
    ("relu_dropped_in_forward", "const double a = cand[i].s > 0.0 ? cand[i].s : 0.0;",
     "const double a = cand[i].s;", "test_oracle_pins"),
    ("keys_used_for_values", "const float* vj = V + (size_t)j * d;\n        for (int32_t c = 0; c < d; ++c) ot[c] += a * (double)vj[c];",
     "const float* vj = K + (size_t)j * d;\n        for (int32_t c = 0; c < d; ++c) ot[c] += a * (double)vj[c];",
     "test_oracle_pins"),
    ("relu_derivative_dropped", "ds[p] = score[p] > 0.0 ? g : 0.0;", "ds[p] = g;", "test_oracle_pins"),
    ("relu_derivative_at_zero_is_one", "ds[p] = score[p] > 0.0 ? g : 0.0;", "ds[p] = score[p] >= 0.0 ? g : 0.0;",
     "test_oracle_pins"),
    ("dh_uses_values", "const float* kj = K + (size_t)j * d;\n        for (int32_t c = 0; c < d; ++c) dht[c] += ds[p] * (double)kj[c];",
     "const float* kj = V + (size_t)j * d;\n        for (int32_t c = 0; c < d; ++c) dht[c] += ds[p] * (double)kj[c];",
     "test_oracle_pins"),
    ("adam_no_bias_correction", "w[o + c] -= lr * (mn / c1) / (sqrt(vn / c2) + eps);",
     "w[o + c] -= lr * mn / (sqrt(vn) + eps);", "test_oracle_adam"),
    ("adam_eps_inside_the_root", "w[o + c] -= lr * (mn / c1) / (sqrt(vn / c2) + eps);",
     "w[o + c] -= lr * (mn / c1) / sqrt(vn / c2 + eps);", "test_oracle_adam"),
    ("adam_second_moment_not_squared", "const double vn = b2 * v[o + c] + (1.0 - b2) * gr * gr;",
     "const double vn = b2 * v[o + c] + (1.0 - b2) * fabs(gr);", "test_oracle_adam"),
    ("union_relu_dropped", "if (sc > 0.0)\n        for (int32_t c = 0; c < d; ++c) ot[c] += sc * (double)V[j * d + c];",
     "for (int32_t c = 0; c < d; ++c) ot[c] += sc * (double)V[j * d + c];", "test_oracle_union"),
    ("union_dk_uses_activation", "dk[c] += g * (double)h[(size_t)t * d + c];",
     "dk[c] += sc * (double)h[(size_t)t * d + c];", "test_oracle_union"),
]


def _mutate(text, name, old, new):
    if name == "ties_to_the_higher_index":
        # flip the tie-break of the comparator: equal scores now order the higher id first
        old = "return (x->id > y->id) - (x->id < y->id);\n}\n\nstatic int by_id_asc"
        new = "return (x->id < y->id) - (x->id > y->id);\n}\n\nstatic int by_id_asc"
    assert text.count(old) >= 1, f"{name}: pattern not found"
    return text.replace(old, new, 1)


def _pins(module_name):
    mod = importlib.import_module("tests." + module_name)
    fns = [getattr(mod, n) for n in dir(mod) if n.startswith("test_")]
    return mod, fns


def _run_pins(module_name):
    """Runs every pin of the module that needs no fixture or parameter; returns the names of those that fail."""
    import inspect
    mod, fns = _pins(module_name)
    failed = []
    for fn in fns:
        params = inspect.signature(fn).parameters
        marks = getattr(fn, "pytestmark", [])
        kwargs = {}
        if any(p.default is inspect._empty for p in params.values()):
            # parametrized or fixture-driven pins: take the first parameter set of a parametrize mark, else skip
            pm = [m for m in marks if m.name == "parametrize"]
            if len(pm) == 1 and len(params) == 1:
                kwargs = {pm[0].args[0]: pm[0].args[1][0]}
            elif "golden" in params and len(params) == 1:
                from tests.conftest import load_golden
                kwargs = {"golden": load_golden}
            else:
                continue
        try:
            fn(**kwargs)
        except BaseException:   # an assertion, or a pin that trips over nonsense results
            failed.append(fn.__name__)
    return failed


@pytest.mark.parametrize("name,old,new,module", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_a_planted_mistake_is_caught(tmp_path, name, old, new, module):
    text = _mutate(open(SRC).read(), name, old, new)
    src = tmp_path / "mutant.c"
    lib = tmp_path / "libmutant.so"
    src.write_text(text)
    subprocess.check_call(["gcc", "-O1", "-fopenmp", "-shared", "-fPIC", "-o", str(lib), str(src), "-lm"])
    mutant = ctypes.CDLL(str(lib))
    O._load()
    for fn in ("meft_oracle_route", "meft_oracle_fwd", "meft_oracle_bwd", "meft_oracle_apply", "meft_oracle_threads",
               "meft_oracle_adam_rows", "meft_oracle_union_fwd", "meft_oracle_union_bwd"):
        getattr(mutant, fn).restype = ctypes.c_int
    real = O._lib
    O._lib = mutant
    try:
        failed = _run_pins(module)
    finally:
        O._lib = real
    assert failed, f"no pin of {module} noticed the mistake '{name}'"
    # and with the real oracle back in place the same pins pass again
    assert _run_pins(module) == []
