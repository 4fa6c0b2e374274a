"""Do the oracle's pins bite?  (CPU only.)

Each case plants ONE plausible mistake in a copy of the oracle's source (a dropped term, a wrong
sign, a wrong index, a swapped or transposed operand, an off-by-one), loads the copy as a module
of its own and runs every pin of tests/test_oracle_pins.py against it.  At least one pin must
fail for every planted mistake, and all must pass on the unmodified source.  The oracle on disk
is never touched and the HIP path is not involved."""
import itertools
import os
import sys
import types

import pytest

from oracle import moe_oracle as orc

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
import test_oracle_pins as pins  # noqa: E402

SOURCE = open(orc.__file__).read()

# (what is planted, text in the oracle, replacement)
MISTAKES = [
    ("bf16 decoded with the wrong shift", "<< np.uint32(16)", "<< np.uint32(15)"),
    ("router bias dropped", "z = z + np.asarray(bias, dtype=np.float32).astype(np.float64)[None, :]", "z = z + 0.0"),
    ("router bias subtracted", "z = z + np.asarray(bias", "z = z - np.asarray(bias"),
    ("softmax exponent sign", "ez = np.exp(z - z.max(axis=1, keepdims=True))", "ez = np.exp(z.max(axis=1, keepdims=True) - z)"),
    ("softmax normalised over the whole batch", "return ez / ez.sum(axis=1, keepdims=True)", "return ez / ez.sum()"),
    ("ties go to the higher index", "win = np.argmax(work, axis=1)", "win = E - 1 - np.argmax(work[:, ::-1], axis=1)"),
    ("winner masked with 0 instead of -inf", "work[rows, win] = -np.inf", "work[rows, win] = 0.0"),
    ("arg-min instead of arg-max", "win = np.argmax(work, axis=1)", "win = np.argmin(work, axis=1)"),
    ("renormalisation forgotten", "        w = w / w.sum(axis=1, keepdims=True)\n", "        w = w * 1.0\n"),
    ("raw scores renormalised", "    elif gating != GATE_SOFTMAX:\n        raise ValueError(\"unknown gating\")\n",
     "    else:\n        w = w / w.sum(axis=1, keepdims=True)\n"),
    ("sigmoid of -z", "sg = 1.0 / (1.0 + np.exp(-z[rows, idx]))", "sg = 1.0 / (1.0 + np.exp(z[rows, idx]))"),
    ("sigmoid gate not normalised", "return sg / sg.sum(axis=1, keepdims=True)", "return sg"),
    ("counting sort not stable (slots placed in reverse)", "    for j, e in enumerate(flat):\n        r = cursor[e]",
     "    for j, e in reversed(list(enumerate(flat))):\n        r = cursor[e]"),
    ("row_of and src_of exchanged", "        row_of[j] = r\n        src_of[r] = j\n", "        row_of[r] = j\n        src_of[j] = r\n"),
    ("inclusive prefix sum", "    cursor = offsets[:-1].copy()\n", "    cursor = offsets[1:].copy() - 1\n"),
    ("offsets one expert late", "offsets[e + 1] = offsets[e] + counts[e]", "offsets[e + 1] = offsets[e] + counts[max(e - 1, 0)]"),
    ("gather by slot instead of token", "[np.asarray(src_of) // k]", "[np.asarray(src_of) % np.asarray(x_bits).shape[0]]"),
    ("block schedule drops a last block of one row", "for r in range(0, int(offsets[e + 1]) - int(offsets[e]), M)]",
     "for r in range(0, int(offsets[e + 1]) - int(offsets[e]) - 1, M)]"),
    ("block schedule in absolute rows", "    return [(e, r) for e in range(len(offsets) - 1)",
     "    return [(e, r + int(offsets[e])) for e in range(len(offsets) - 1)"),
    ("SiLU sign", "return a / (1.0 + np.exp(-a))", "return a / (1.0 + np.exp(a))"),
    ("SiLU without the factor a", "return a / (1.0 + np.exp(-a))", "return 1.0 / (1.0 + np.exp(-a))"),
    ("gate and up exchanged", "h = silu(g) * u", "h = silu(u) * g"),
    ("up projection computed with the gate weights", "    wu = bf16_to_f64(wu_bits)\n", "    wu = bf16_to_f64(wg_bits)\n"),
    ("SwiGLU product replaced by a sum", "h = silu(g) * u", "h = silu(g) + u"),
    ("router matrix transposed where shapes allow", "z = bf16_to_f64(x_bits) @ bf16_to_f64(wr_bits).T",
     "wr_ = bf16_to_f64(wr_bits)\n    z = bf16_to_f64(x_bits) @ (wr_ if wr_.shape[0] == wr_.shape[1] else wr_.T)"),
    ("gate projection transposed where shapes allow", "g = xrows @ wg.T", "g = xrows @ (wg if wg.shape[0] == wg.shape[1] else wg.T)"),
    ("up projection transposed where shapes allow", "u = xrows @ wu.T", "u = xrows @ (wu if wu.shape[0] == wu.shape[1] else wu.T)"),
    ("down projection transposed where shapes allow", "v = h @ wd.T", "v = h @ (wd if wd.shape[0] == wd.shape[1] else wd.T)"),
    ("combine without the gate weights", "y += w[tok, i][:, None] * v[:, i, :]", "y += v[:, i, :]"),
    ("combine with the slots' weights reversed", "y += w[tok, i][:, None] * v[:, i, :]", "y += w[tok, k - 1 - i][:, None] * v[:, i, :]"),
    ("combine drops the last slot", "    for i in range(k):\n        y += w[tok, i]", "    for i in range(max(k - 1, 1)):\n        y += w[tok, i]"),
    ("expert results stored under the wrong slot", "        v[tt, ii] = ve\n", "        v[tt, (ii + 1) % k] = ve\n"),
]


def _load(source, name):
    mod = types.ModuleType(name)
    mod.__file__ = orc.__file__
    exec(compile(source, orc.__file__, "exec"), mod.__dict__)
    return mod


def _pin_calls():
    """Every pin as a zero-argument callable (parametrised pins once per parameter set)."""
    calls = []
    for name in sorted(vars(pins)):
        fn = getattr(pins, name)
        if not (name.startswith("test_") and callable(fn)):
            continue
        marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
        if not marks:
            calls.append((name, fn))
            continue
        axes = []
        for m in marks:
            names = [n.strip() for n in m.args[0].split(",")]
            axes.append([dict(zip(names, v if len(names) > 1 else (v,))) for v in m.args[1]])
        for combo in itertools.product(*axes):
            kw = {}
            for part in combo:
                kw.update(part)
            calls.append((f"{name}{sorted(kw.items())}", lambda fn=fn, kw=kw: fn(**kw)))
    return calls


def _failing_pins(module, monkeypatch, first_only=True):
    monkeypatch.setattr(pins, "orc", module)
    failed = []
    for name, call in _pin_calls():
        try:
            call()
        except Exception:     # an assertion, or the mistake making the oracle itself raise
            failed.append(name)
            if first_only:
                break
    return failed


def test_all_pins_pass_on_the_oracle_as_it_is(monkeypatch):
    assert len(_pin_calls()) >= 20
    assert _failing_pins(_load(SOURCE, "oracle_copy"), monkeypatch, first_only=False) == []


@pytest.mark.parametrize("what,old,new", MISTAKES, ids=[m[0] for m in MISTAKES])
def test_a_planted_mistake_fails_a_pin(monkeypatch, what, old, new):
    assert SOURCE.count(old) >= 1, f"the oracle no longer contains the text this case edits: {old!r}"
    mutated = _load(SOURCE.replace(old, new), "oracle_with_a_mistake")
    failed = _failing_pins(mutated, monkeypatch)
    assert failed, f"no pin notices: {what}"
