"""Checks of the oracle as a C program (CPU only; each runs the pin suite in a child process
against another build of ``oracle/lola_oracle.c``):

* a build with AddressSanitizer and UndefinedBehaviorSanitizer must pass every pin with no report
  (the oracle keeps its caches in hand-managed arrays: realloc, memmove, index bookkeeping);
* copies of the source with ONE planted mistake each (a transposed operand, a wrong sign, a dropped
  term, an off-by-one window, a reversed tie rule ...) must each fail at least one pin, which shows
  that the pins constrain every part of the oracle's arithmetic.
"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "lola_oracle.c")
PINS = os.path.join(ROOT, "tests", "test_oracle_pins.py")


def run_pins(tmp_path, src=SRC, cflags="", preload=None, stop_at_first=True):
    env = dict(os.environ, LOLA_ORACLE_SRC=src, LOLA_ORACLE_LIBDIR=str(tmp_path), LOLA_ORACLE_CFLAGS=cflags,
               OMP_NUM_THREADS="4")
    if preload:
        env["LD_PRELOAD"] = ":".join([preload] + ([os.environ["LD_PRELOAD"]] if os.environ.get("LD_PRELOAD") else []))
        # the interpreter itself is not instrumented: its own allocations are not this test's subject
        env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1"
        env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    cmd = [sys.executable, "-m", "pytest", PINS, "-q", "-p", "no:cacheprovider"] + (["-x"] if stop_at_first else [])
    return subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True)


def test_pins_pass_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(asan) or not os.path.exists(asan):
        pytest.skip("gcc has no AddressSanitizer runtime here")
    r = run_pins(tmp_path, cflags="-fsanitize=address,undefined -fno-sanitize-recover=all -fno-omit-frame-pointer -g",
                 preload=os.path.realpath(asan), stop_at_first=False)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, tail
    assert "ERROR: AddressSanitizer" not in tail and "runtime error" not in tail, tail
    assert os.path.exists(os.path.join(str(tmp_path), "liblola_oracle_f64.so"))   # the child really built its own copy


# (name, text in the oracle, its replacement[, which occurrence: 1 = first])
MUTANTS = [
    ("logit scale dropped for the cached pairs", "real w = (real)exp((double)((real)c->scale * dot));",
     "real w = (real)exp((double)dot);", 2),
    ("logit scale dropped for the window pairs", "real w = (real)exp((double)((real)c->scale * dot));",
     "real w = (real)exp((double)dot);", 3),
    ("query heads of a group mapped to the wrong kv head (generation)", "int hq = h * g + r;", "int hq = r * c->Hkv + h;", 1),
    ("query heads of a group mapped to the wrong kv head (prefill)", "int hq = h * g + r;", "int hq = r * c->Hkv + h;", 2),
    ("projection matrix read transposed", "W[(size_t)i * m + j]", "W[(size_t)j * d + i]"),
    ("negative half of phi uses the positive exponent", "real en = (real)exp((double)(zmin - z));",
     "real en = (real)exp((double)(z - zmax));"),
    ("tie rule reversed", "t->sp.idx[o] < t->sp.idx[e]", "t->sp.idx[o] > t->sp.idx[e]"),
    ("smallest scores kept", "(score[o] > score[e])", "(score[o] < score[e])"),
    ("window one pair too long", "if (t->win.n > c->eta) {", "if (t->win.n > c->eta + 1) {"),
    ("denominator without the s term", "den += p * t->s[f];", "den += 0 * t->s[f];"),
    ("s folded on half of the features", "t->s[f] += p;", "t->s[f] += (f < D/2) ? p : 0;"),
    ("causal mask excludes the token itself", "attend(c, t, Wq + (size_t)hq * d * m, qr, ck, cv, i + 1, out + off);",
     "attend(c, t, Wq + (size_t)hq * d * m, qr, ck, cv, i, out + off);"),
    ("recall without its normaliser", "pred = num / den;", "pred = num;"),
    ("one pair too few leaves the window in a chunk", "int n_ev = t->win.n - c->eta;", "int n_ev = t->win.n - c->eta - 1;"),
    ("error with the wrong sign", "real e = pred - v[j];", "real e = pred + v[j];"),
]


@pytest.mark.parametrize("mut", MUTANTS, ids=[m[0].replace(" ", "_") for m in MUTANTS])
def test_a_planted_mistake_fails_a_pin(tmp_path, mut):
    name, old, new = mut[:3]
    nth = mut[3] if len(mut) > 3 else 1
    src = open(SRC).read()
    assert src.count(old) >= nth, f"the oracle no longer contains the text this mutant replaces: {old!r}"
    parts = src.split(old)
    mutated = old.join(parts[:nth]) + new + old.join(parts[nth:])
    mutant = os.path.join(str(tmp_path), "lola_oracle_mutant.c")
    with open(mutant, "w") as f:
        f.write(mutated)
    r = run_pins(tmp_path, src=mutant)
    assert r.returncode != 0, f"no pin noticed: {name}"
    assert " failed" in r.stdout, r.stdout[-1500:] + r.stderr[-1500:]   # a pin failed (not a build or import error)
