"""Each planted mistake in a copy of oracle/engine.py must fail at least one pin of test_oracle_engine."""
import importlib.util
import inspect
import os

import pytest

import test_oracle_engine as pins

SRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle", "engine.py")

MISTAKES = [
    ("the message is formed from the replicas at the receive step",
     "                    dequant_reduce_nesterov(self.g[sl], self.mom[sl], codes, scales, self.fmt, self.lr, self.mu, n=n)\n",
     "                    codes, scales = quantize_outer_grad(self.g[sl].copy(), [w[sl].copy() for w in self.w], self.fmt)\n"
     "                    dequant_reduce_nesterov(self.g[sl], self.mom[sl], codes, scales, self.fmt, self.lr, self.mu, n=n)\n"),
    ("every worker merges at the smallest delay", "                if t == ts + self.tau[m]:", "                if t == ts + min(self.tau):"),
    ("the outer update waits for the largest delay", "            if t == ts + min(self.tau):", "            if t == ts + max(self.tau):"),
    ("the mean and the outer update run once per worker", "            if t == ts + min(self.tau):",
     "            if t in {ts + d for d in self.tau}:"),
    ("the merge mixes with weight 1 - alpha on the replica", "merge_overlap(self.g[sl], [self.w[m][sl]], self.alpha)",
     "merge_overlap(self.g[sl], [self.w[m][sl]], 1.0 - self.alpha)"),
    ("without overlap the replicas are not updated",
     "                    fragment_outer_step(self.g[sl], self.mom[sl], ws, ws, self.fmt, self.lr, self.mu, self.alpha)",
     "                    fragment_outer_step(self.g[sl], self.mom[sl], ws, [x.copy() for x in ws], self.fmt, self.lr, self.mu, self.alpha)"),
    ("only the first span of a fragment is synchronised", "                for off, n, _ in plan.spans[p]:\n                    sl = slice(off, off + n)\n                    ws =",
     "                for off, n, _ in plan.spans[p][:1]:\n                    sl = slice(off, off + n)\n                    ws ="),
    ("a fragment's synchronisation covers the whole model", "                    sl = slice(off, off + n)\n                    ws =",
     "                    sl = slice(0, self.g.size)\n                    ws ="),
    ("the outer learning rate is applied twice", "self.lr, self.mu, self.alpha)\n                sent += 1",
     "2 * self.lr, self.mu, self.alpha)\n                sent += 1"),
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
    text = text.replace("from . import (", "from oracle import (").replace("from .plan import RefPlan", "from oracle.plan import RefPlan")
    path = tmp_path / f"engine_{tag}.py"
    path.write_text(text)
    spec = importlib.util.spec_from_file_location(f"engine_{tag}", path)
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_unmodified_copy_passes(tmp_path, monkeypatch):
    monkeypatch.setattr(pins, "RefEngine", _load(tmp_path, open(SRC).read(), "none").RefEngine)
    for _, fn, kw in _pin_calls():
        fn(**kw)


@pytest.mark.parametrize("what,old,new", MISTAKES, ids=[m[0] for m in MISTAKES])
def test_planted_mistake_is_caught(tmp_path, monkeypatch, what, old, new):
    text = open(SRC).read()
    assert text.count(old) == 1, f"{what}: the text to replace must occur exactly once"
    monkeypatch.setattr(pins, "RefEngine", _load(tmp_path, text.replace(old, new), "m").RefEngine)
    caught = []
    for name, fn, kw in _pin_calls():
        try:
            fn(**kw)
        except Exception as e:
            caught.append(f"{name}: {type(e).__name__}")
    assert caught, f"no pin notices: {what}"
