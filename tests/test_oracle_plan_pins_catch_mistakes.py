"""Each planted mistake in a copy of oracle/plan.py must fail at least one pin of test_oracle_plan."""
import importlib.util
import inspect
import os

import pytest

import test_oracle_plan as pins

SRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle", "plan.py")

MISTAKES = [
    ("a fragment may be sent at its offset itself", "            k = 1\n            while self.offsets[p] + k * self.H <= t:",
     "            k = 0\n            while self.offsets[p] + k * self.H <= t:"),
    ("send condition with the sign of the offset flipped", "                if self.offsets[p] + k * self.H == t:\n                    out.append(p)\n                k += 1\n        return out\n\n    def receives",
     "                if k * self.H - self.offsets[p] == t:\n                    out.append(p)\n                k += 1\n        return out\n\n    def receives"),
    ("the receive comes tau steps early", "self.offsets[p] + k * self.H + self.tau == t", "self.offsets[p] + k * self.H - self.tau == t"),
    ("the receive ignores tau", "self.offsets[p] + k * self.H + self.tau == t", "self.offsets[p] + k * self.H == t"),
    ("strided pattern deals blocks in chunks", "block_fragment.append(shift + i % P)", "block_fragment.append(shift + (i * P) // n_blocks)"),
    ("sequential pattern deals blocks round robin", "                if (p * n_blocks) // P <= i < ((p + 1) * n_blocks) // P:\n                    owner = p",
     "                if i % P == p:\n                    owner = p"),
    ("default offsets rounded up", "offsets = [(p * H) // P for p in range(P)]", "offsets = [-((-p * H) // P) for p in range(P)]"),
    ("default offsets all zero", "offsets = [(p * H) // P for p in range(P)]", "offsets = [0 for p in range(P)]"),
    ("the head travels with the first fragment", "            p = block_fragment[n_blocks - 1]", "            p = block_fragment[0]"),
    ("the embedding travels with the last fragment", "            p = 0 if pre_own_fragment else block_fragment[0]",
     "            p = 0 if pre_own_fragment else block_fragment[n_blocks - 1]"),
    ("the own-fragment variant keeps the embedding with block 0", "            p = 0 if pre_own_fragment else block_fragment[0]",
     "            p = block_fragment[0]"),
    ("spans do not advance through the model", "        pos += int(numel)", "        pos += 0"),
    ("the aligned layout always inserts padding", "        while pos % align != 0:\n            pos += 1",
     "        pos += 1\n        while pos % align != 0:\n            pos += 1"),
    ("the aligned layout ignores the alignment", "        while pos % align != 0:\n            pos += 1", "        pass"),
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
        assert len(marks) == 1
        names, values = marks[0].args
        names = [n.strip() for n in names.split(",")]
        for v in values:
            v = v if isinstance(v, (tuple, list)) and len(names) > 1 else (v,)
            calls.append((f"{name}{list(v)}", fn, dict(zip(names, v))))
    return calls


def _load(tmp_path, text, tag):
    path = tmp_path / f"plan_{tag}.py"
    path.write_text(text)
    spec = importlib.util.spec_from_file_location(f"plan_{tag}", path)
    mod = importlib.util.module_from_spec(spec)
    import sys
    sys.modules[spec.name] = mod            # dataclasses look their module up by name
    spec.loader.exec_module(mod)
    return mod


def test_unmodified_copy_passes(tmp_path, monkeypatch):
    monkeypatch.setattr(pins, "fragment_plan", _load(tmp_path, open(SRC).read(), "none").fragment_plan)
    for _, fn, kw in _pin_calls():
        fn(**kw)


@pytest.mark.parametrize("what,old,new", MISTAKES, ids=[m[0] for m in MISTAKES])
def test_planted_mistake_is_caught(tmp_path, monkeypatch, what, old, new):
    text = open(SRC).read()
    assert text.count(old) == 1, f"{what}: the text to replace must occur exactly once"
    monkeypatch.setattr(pins, "fragment_plan", _load(tmp_path, text.replace(old, new), "m").fragment_plan)
    caught = []
    for name, fn, kw in _pin_calls():
        try:
            fn(**kw)
        except Exception as e:
            caught.append(f"{name}: {type(e).__name__}")
    assert caught, f"no pin notices: {what}"
