"""Each planted mistake in a copy of oracle/evalparams.py must fail at least one of its pins."""
import importlib.util
import inspect
import os

import pytest

import test_oracle_evalparams as pins

SRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle", "evalparams.py")

MISTAKES = [
    ("truncation instead of rounding", "rounded = (bits + 0x7fff + ((bits >> 16) & 1)) >> 16", "rounded = bits >> 16"),
    ("ties away from zero", "rounded = (bits + 0x7fff + ((bits >> 16) & 1)) >> 16", "rounded = (bits + 0x8000) >> 16"),
    ("ties to odd", "((bits >> 16) & 1)", "(1 - ((bits >> 16) & 1))"),
    ("NaN rounds into infinity", "    out[nan] = ((bits[nan] >> 16) | 0x40).astype(np.uint16)\n", ""),
    ("first replica is the last one", "return w_bits[0].copy()", "return w_bits[-1].copy()"),
    ("outer parameters truncated", "return bf16_round(g)", "return (g.view(np.uint32) >> 16).astype(np.uint16)"),
    ("sum instead of mean", "return bf16_round(acc / np.float32(len(w_bits)))", "return bf16_round(acc)"),
    ("divides by M - 1", "np.float32(len(w_bits))", "np.float32(max(len(w_bits) - 1, 1))"),
    ("accumulates in bf16", "        acc = acc + (w.astype(np.uint32) << 16).view(np.float32)       # one fp32 addition per replica\n",
     "        acc = acc + (w.astype(np.uint32) << 16).view(np.float32)\n        acc = (bf16_round(acc).astype(np.uint32) << 16).view(np.float32)\n"),
    ("accumulates in fp64", "acc = np.zeros(w_bits[0].shape, np.float32)", "acc = np.zeros(w_bits[0].shape, np.float64)"),
    ("adds the replicas in reverse order", "for w in w_bits:", "for w in w_bits[::-1]:"),
    ("widens bf16 with the wrong shift", "(w.astype(np.uint32) << 16)", "(w.astype(np.uint32) << 15)"),
]


def _pin_calls():
    calls = []
    for name, fn in inspect.getmembers(pins, inspect.isfunction):
        if not name.startswith("test_"):
            continue
        marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
        if not marks:
            calls.append((name, fn, {}))
            continue
        arg, values = marks[0].args
        for v in values:
            calls.append((f"{name}[{v}]", fn, {arg: v}))
    return calls


def _load(tmp_path, text, tag):
    path = tmp_path / f"evalparams_{tag}.py"
    path.write_text(text)
    spec = importlib.util.spec_from_file_location(f"evalparams_{tag}", path)
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_unmodified_copy_passes(tmp_path, monkeypatch):
    monkeypatch.setattr(pins, "ep", _load(tmp_path, open(SRC).read(), "none"))
    for _, fn, kw in _pin_calls():
        fn(**kw)


@pytest.mark.parametrize("what,old,new", MISTAKES, ids=[m[0] for m in MISTAKES])
def test_planted_mistake_is_caught(tmp_path, monkeypatch, what, old, new):
    text = open(SRC).read()
    assert text.count(old) == 1, f"{what}: the text to replace must occur exactly once"
    monkeypatch.setattr(pins, "ep", _load(tmp_path, text.replace(old, new), "m"))
    caught = []
    for name, fn, kw in _pin_calls():
        try:
            fn(**kw)
        except Exception as e:
            caught.append(f"{name}: {type(e).__name__}")
    assert caught, f"no pin notices: {what}"
