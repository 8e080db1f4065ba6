"""The pins of the cosine-similarity oracle are only worth something if a plausible mistake in
the oracle fails one of them.  Each case plants one mistake in a copy of oracle/cosine.py (on the
CPU, in a temporary module) and runs the pin tests against the copy: at least one must fail."""
import importlib.util
import inspect
import os

import pytest

import test_oracle_cosine as pins

SRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle", "cosine.py")

MISTAKES = [
    ("operands swapped", "rows.append(g - wf)", "rows.append(wf - g)"),
    ("replica alone instead of the difference", "rows.append(g - wf)", "rows.append(wf)"),
    ("bf16 widened with the wrong shift", "<< 16", "<< 15"),
    ("products added in fp32", "d = outer_grads(g, w_bits).astype(np.float64)", "d = outer_grads(g, w_bits)"),
    ("Gram matrix divided by n", "return d @ d.T", "return d @ d.T / d.shape[1]"),
    ("norm without the square root", "norm = np.sqrt(np.diag(G))", "norm = np.diag(G)"),
    ("divided by the squared norms", "G[a, b] / den if den > 0", "G[a, b] / (den * den) if den > 0"),
    ("only one norm in the denominator", "den = norm[a] * norm[b]", "den = norm[a] * norm[a]"),
    ("zero norm reads as similarity 1", "if den > 0 else 0.0", "if den > 0 else 1.0"),
    ("mean includes the diagonal", "for b in range(a + 1, M)]", "for b in range(a, M)]"),
    ("mean over ordered pairs", "/ len(pairs)) if pairs", "/ (2 * len(pairs))) if pairs"),
    ("one replica gives mean 1", "if pairs else 0.0", "if pairs else 1.0"),
    ("union keeps only the last set", "        G = G + np.asarray(x, np.float64)\n", "        G = np.asarray(x, np.float64)\n"),
    ("union averages the Gram matrices", "        G = G + np.asarray(x, np.float64)\n",
     "        G = G + np.asarray(x, np.float64) / len(grams)\n"),
]


def _pin_calls():
    """Every pin test of test_oracle_cosine with each of its parameter sets."""
    calls = []
    for name, fn in inspect.getmembers(pins, inspect.isfunction):
        if not name.startswith("test_"):
            continue
        marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
        if not marks:
            calls.append((name, fn, {}))
            continue
        assert len(marks) == 1
        arg, values = marks[0].args
        for v in values:
            calls.append((f"{name}[{v}]", fn, {arg: v}))
    return calls


def _load_mutant(tmp_path, text, tag):
    path = tmp_path / f"cosine_mutant_{tag}.py"
    path.write_text(text)
    spec = importlib.util.spec_from_file_location(f"cosine_mutant_{tag}", path)
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_unmodified_copy_passes(tmp_path, monkeypatch):
    monkeypatch.setattr(pins, "cosine", _load_mutant(tmp_path, open(SRC).read(), "none"))
    for _, fn, kw in _pin_calls():
        fn(**kw)


@pytest.mark.parametrize("what,old,new", MISTAKES, ids=[m[0] for m in MISTAKES])
def test_planted_mistake_is_caught(tmp_path, monkeypatch, what, old, new):
    text = open(SRC).read()
    assert text.count(old) == 1, f"{what}: the text to replace must occur exactly once"
    monkeypatch.setattr(pins, "cosine", _load_mutant(tmp_path, text.replace(old, new), "m"))
    caught = []
    for name, fn, kw in _pin_calls():
        try:
            fn(**kw)
        except Exception as e:                      # an assertion, or a crash of the broken oracle
            caught.append(f"{name}: {type(e).__name__}")
    assert caught, f"no pin notices: {what}"
