"""The pins are only worth something if a plausible mistake in the oracle fails one of them.
Each case below plants one mistake in a COPY of an oracle source (a dropped term, a wrong sign or
index, a transposed operand, an off-by-one), runs the pin tests against the mutant and requires at
least one of them to fail.  CPU only; the real oracle is never modified."""
import importlib
import inspect
import os
import sys
import types

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

CAT_MUTATIONS = [
    ("inclusive instead of exclusive prefix product", "s[b, k] = run\n                run = run * conf[b, k]",
     "run = run * conf[b, k]\n                s[b, k] = run"),
    ("decay exponent off by one", "float(gamma) ** k", "float(gamma) ** (k + 1)"),
    ("estimated length ignores the valid length", "if k < vl[b]:\n                exp_len[b] += s[b, k] * conf[b, k]",
     "if True:\n                exp_len[b] += s[b, k] * conf[b, k]"),
    ("log-sum-exp without the max shift added back", "lse[r0:r1] = mm + np.log(", "lse[r0:r1] = np.log("),
    ("target log-prob with the wrong sign", "logq[r0:r1][ok] = Z[rows[ok], yy[ok]] - lse[r0:r1][ok]",
     "logq[r0:r1][ok] = lse[r0:r1][ok] - Z[rows[ok], yy[ok]]"),
    ("loss not multiplied by beta", "loss = (beta / n_norm) * float(", "loss = (1.0 / n_norm) * float("),
    ("normaliser counts all rows", "n_valid = int(valid.sum())", "n_valid = int(valid.size)"),
    ("weight not masked on ignored rows", "w = np.where(valid, s, 0.0)", "w = s.copy()"),
    ("one-hot subtracted twice", "dZ = g[r][:, None] * (Q - hot)", "dZ = g[r][:, None] * (Q - 2.0 * hot)"),
    ("dW from untransposed dZ rows (wrong operand)", "dW += dZ.T @ H64[r0:r1]", "dW += (dZ.T @ H64[r0:r1])[::-1]"),
    ("accepted prefix counts all hits", "while n < vl[b] and hit[b, n]:\n            n += 1\n        out[b] = n",
     "out[b] = int(hit[b, :vl[b]].sum())"),
    ("gradient scale forgets beta", "return gout * beta * w / float(n_valid)", "return gout * w / float(n_valid)"),
    ("sequence gather starts one position late", "conf[b, k] = c_seq[n + k]", "conf[b, k] = c_seq[min(n + k + 1, len(c_seq) - 1)]"),
]

KD_MUTATIONS = [
    ("reverse KL", 'out["kd"][sl] = np.sum(P * (logP - logQ), axis=1)',
     'out["kd"][sl] = np.sum(np.exp(logQ) * (logQ - logP), axis=1)'),
    ("beta applied to the KD term too", 'tok = beta * (-st["logq"]) + st["kd"]', 'tok = beta * (-st["logq"] + st["kd"])'),
    ("confidence from the draft instead of the teacher", 'np.exp(st["logp_t"])', 'np.exp(st["logq"])'),
    ("teacher term dropped from the gradient", "(beta * (Q - hot) + (Q - P))", "(beta * (Q - hot) + Q)"),
    ("gradient scale carries beta", "return O.row_scale(w, 1.0, n_valid, reduction, gout)",
     "return O.row_scale(w, 0.1, n_valid, reduction, gout)"),
]

INJECT_MUTATIONS = [
    ("gate applied to the embedding too", "return np.asarray(E, dtype=np.float64) + np.asarray(xi, dtype=np.float64)[:, None] * t",
     "return np.asarray(xi, dtype=np.float64)[:, None] * (np.asarray(E, dtype=np.float64) + t)"),
    ("projection not transposed back", "return dT, dT.T @ X", "return dT, (X.T @ dT).T[::-1]"),
]


def _mutant(module_name, old, new):
    real = importlib.import_module(module_name)
    src = inspect.getsource(real)
    assert src.count(old) >= 1, f"pattern not found in {module_name}: {old!r}"
    mod = types.ModuleType(real.__name__)
    mod.__package__ = real.__package__
    mod.__file__ = real.__file__
    exec(compile(src.replace(old, new), real.__file__, "exec"), mod.__dict__)
    return mod


def _run_pins(test_module_name, attr, mutant, extra=None):
    """Run every argument-free or parametrised pin test of a module with `attr` (the oracle alias it
    uses) pointing at the mutant; return the names of the tests that failed."""
    tm = importlib.import_module(test_module_name)
    saved = {attr: getattr(tm, attr)}
    setattr(tm, attr, mutant)
    for k, v in (extra or {}).items():
        saved[k] = getattr(tm, k)
        setattr(tm, k, v)
    failed = []
    try:
        for name, fn in inspect.getmembers(tm, inspect.isfunction):
            if not name.startswith("test_") or fn.__module__ != tm.__name__:
                continue
            marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
            if marks:
                names = [n.strip() for n in marks[0].args[0].split(",")]
                calls = [dict(zip(names, v if len(names) > 1 else (v,))) for v in marks[0].args[1]]
            elif not inspect.signature(fn).parameters:
                calls = [{}]
            else:
                continue
            for kw in calls:
                try:
                    fn(**kw)
                except pytest.skip.Exception:
                    pass
                except Exception:
                    failed.append(name)
    finally:
        for k, v in saved.items():
            setattr(tm, k, v)
    return failed


@pytest.mark.parametrize("what,old,new", CAT_MUTATIONS, ids=[m[0] for m in CAT_MUTATIONS])
def test_cat_oracle_pins_catch(what, old, new):
    failed = _run_pins("tests.test_oracle_pins", "O", _mutant("oracle.cat_oracle", old, new))
    assert failed, f"no pin noticed: {what}"


@pytest.mark.parametrize("what,old,new", KD_MUTATIONS, ids=[m[0] for m in KD_MUTATIONS])
def test_kd_oracle_pins_catch(what, old, new):
    real = importlib.import_module("oracle.cat_kd_oracle")
    src = inspect.getsource(real)
    assert old in src
    mod = types.ModuleType(real.__name__)
    mod.__package__ = "oracle"
    exec(compile(src.replace(old, new), real.__file__, "exec"), mod.__dict__)
    failed = _run_pins("tests.test_oracle_kd_pins", "KD", mod)
    assert failed, f"no pin noticed: {what}"


@pytest.mark.parametrize("what,old,new", INJECT_MUTATIONS, ids=[m[0] for m in INJECT_MUTATIONS])
def test_inject_oracle_pins_catch(what, old, new):
    failed = _run_pins("tests.test_oracle_inject_pins", "I", _mutant("oracle.inject_oracle", old, new))
    assert failed, f"no pin noticed: {what}"


def test_unmutated_oracles_pass_the_same_harness():
    for tmod, attr, omod in (("tests.test_oracle_pins", "O", "oracle.cat_oracle"),
                             ("tests.test_oracle_kd_pins", "KD", "oracle.cat_kd_oracle"),
                             ("tests.test_oracle_inject_pins", "I", "oracle.inject_oracle")):
        assert _run_pins(tmod, attr, importlib.import_module(omod)) == []
