"""Do the oracle's pins have teeth?  Each case below plants ONE plausible mistake in a copy of the
oracle's C source (a dropped term, a wrong sign or index, a max started at zero, a swapped
comparison ...), builds the copy, points the oracle loader at it and re-runs the pins: at least one
pin has to fail for every planted mistake, and all of them pass on the unchanged source.
CPU only; nothing here touches the HIP path."""
import os
import subprocess

import pytest

import oracle
from tests import test_oracle_pins as pins

SRC = os.path.join(os.path.dirname(os.path.abspath(oracle.__file__)), "espn_oracle.c")

# (name, text in the source, replacement, which occurrence: 0 = the plain path, 1 = the compressed path)
MUTANTS = [
    ("max over document rows started at zero", "double best = -INFINITY;", "double best = 0.0;", 0),
    ("smaller-than instead of greater-than in the max", "if (dot > best) best = dot;", "if (dot < best) best = dot;", 0),
    ("sum over query rows replaced by a max", "score += best;", "if (best > score || i == 0) score = best;", 0),
    ("first vector component dropped", "for (int32_t c = 0; c < d; ++c) dot += qd[",
     "for (int32_t c = 1; c < d; ++c) dot += qd[", 0),
    ("document components read in reverse", "dd[j * d + c];", "dd[j * d + (d - 1 - c)];", 0),
    ("last row of every document dropped", "int64_t s = offsets[id], e = offsets[id + 1];",
     "int64_t s = offsets[id], e = offsets[id + 1] - (offsets[id + 1] > offsets[id]);", 0),
    ("rows of the preceding document included", "int64_t s = offsets[id], e = offsets[id + 1];",
     "int64_t s = offsets[id > 0 ? id - 1 : 0], e = offsets[id + 1];", 0),
    ("ascending instead of descending scores",
     "if (a->score > b->score) return -1;\n    if (a->score < b->score) return 1;",
     "if (a->score > b->score) return 1;\n    if (a->score < b->score) return -1;", 0),
    ("ties to the higher id", "if (a->id < b->id) return -1;\n    if (a->id > b->id) return 1;",
     "if (a->id < b->id) return 1;\n    if (a->id > b->id) return -1;", 0),
    ("binary16 exponent bias off by one", "expo - 25);", "expo - 24);", 0),
    ("binary16 subnormals flushed to zero", "v = ldexp((double)frac, -24);", "v = 0.0;", 0),
    ("sign of binary16 ignored", "return sign ? -v : v;", "return v;", 0),
    ("prior subtracted instead of added", "scores[x] + alpha * (double)prior[x];", "scores[x] - alpha * (double)prior[x];", 0),
    ("partial re-ranking: tail taken from the wrong position", "out_ids[(int64_t)b * k + j] = cand[(int64_t)b * K + j];",
     "out_ids[(int64_t)b * k + j] = cand[(int64_t)b * K + (j - R)];", 0),
    ("merge: second list dropped", "for (int32_t j = 0; j < kb; ++j) {", "for (int32_t j = 0; j < 0; ++j) {", 0),
    ("Eq. 4 inverted", "return bandwidth_bytes_per_s * budget_s / bytes_per_query;",
     "return bytes_per_query / (bandwidth_bytes_per_s * budget_s);", 0),
    ("compressed path: max started at zero", "double best = -INFINITY;", "double best = 0.0;", 1),
    ("compressed path: document scale forgotten", "dd[x] = scale * espn_oracle_e4m3_to_double(", "dd[x] = espn_oracle_e4m3_to_double(", 0),
    ("compressed path: last row dropped", "for (int64_t j = 0; j < e - s; ++j) {", "for (int64_t j = 0; j + 1 < e - s; ++j) {", 0),
    ("E4M3 exponent bias off by one", "expo - 10);", "expo - 9);", 0),
    ("E4M3 subnormals flushed to zero", "v = ldexp((double)frac, -9);", "v = 0.0;", 0),
    ("E4M3 sign ignored", "return sign ? -v : v;", "return v;", 1),
]


def replace_nth(text, old, new, n):
    pos = -1
    for _ in range(n + 1):
        pos = text.find(old, pos + 1)
        assert pos >= 0, "the oracle's source does not contain %r %d time(s)" % (old, n + 1)
    return text[:pos] + new + text[pos + len(old):]


def pin_calls():
    """Every pin of tests/test_oracle_pins.py as a zero-argument callable (parametrised ones expanded)."""
    calls = []
    for name in sorted(dir(pins)):
        fn = getattr(pins, name)
        if not (name.startswith("test_") and callable(fn)):
            continue
        marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
        if not marks:
            calls.append((name, fn))
            continue
        assert len(marks) == 1, name
        for value in marks[0].args[1]:
            calls.append(("%s[%r]" % (name, value if not isinstance(value, dict) else value.get("name")),
                          lambda fn=fn, value=value: fn(value)))
    return calls


def failing_pins():
    failed = []
    for name, call in pin_calls():
        try:
            call()
        except Exception as exc:          # an assertion, or the oracle refusing its own output
            failed.append("%s: %s" % (name, type(exc).__name__))
    return failed


def build_variant(tmp_path, text):
    src = tmp_path / "oracle_variant.c"
    lib = tmp_path / "liboracle_variant.so"
    src.write_text(text)
    subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
                           "-o", str(lib), str(src), "-lm"])
    return str(lib)


def use_library(monkeypatch, path):
    monkeypatch.setattr(oracle, "_lib", None)
    monkeypatch.setattr(oracle, "build", lambda force=False: path)


def test_every_pin_passes_on_the_unchanged_source(tmp_path, monkeypatch):
    use_library(monkeypatch, build_variant(tmp_path, open(SRC).read()))
    assert failing_pins() == []


@pytest.mark.parametrize("name,old,new,which", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_a_planted_mistake_fails_a_pin(name, old, new, which, tmp_path, monkeypatch):
    use_library(monkeypatch, build_variant(tmp_path, replace_nth(open(SRC).read(), old, new, which)))
    failed = failing_pins()
    assert failed, "no pin noticed: " + name
    print("%s -> %d pins fail, e.g. %s" % (name, len(failed), failed[0]))
