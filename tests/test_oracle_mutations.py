"""Do the pins have teeth?  One plausible mistake at a time is planted in a COPY of the C oracle (a wrong nibble order, a
transposed lane map, a flipped sign, a shifted group, a wrong tie rule, a wrong rounding) and the pin tests are run against
that copy in a child process: every planted mistake must make at least one pin fail, and the untouched copy must pass.
Everything happens on the CPU, in a temporary directory; the oracle in the tree is never modified."""
import concurrent.futures
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "oracle_w4.c")

# (what the mistake is, text in the source, what replaces it, how many places hold that text)
MUTATIONS = [
    ("packed layout: nibble slot = e instead of the interleaved order", "int p = 4 * (e & 1) + (e >> 1);", "int p = e;", 1),
    ("packed layout: k-step and lane-group indices exchanged", "int t = kk / 32, h = (kk % 32) / 8, e = kk % 8;",
     "int t = (kk % 32) / 8, h = kk / 32, e = kk % 8;", 1),
    ("packed layout: lane = 4*c + h instead of 16*h + c", "int lane = 16 * h + c;", "int lane = 4 * c + h;", 2),
    ("scale/zero word: zero-point read from the low half", "(uint16_t)(w >> 16);", "(uint16_t)(w & 0xFFFFu);", 2),
    ("sampled matmul: one term dropped", "        acc += orc_fp16_to_double(X[(size_t)m * K + k]) * w;\n",
     "        acc += orc_fp16_to_double(X[(size_t)m * K + k]) * w; if (k == 5) acc -= w;\n", 2),
    ("matmul: q + z instead of q - z", "acc[j] += x * (((double)qr[j] - zp[j]) * sc[j]);",
     "acc[j] += x * (((double)qr[j] + zp[j]) * sc[j]);", 1),
    ("matmul: group constants refreshed one row late", "if (k % g == 0) {", "if (k % g == 1 || k == 0) {", 1),
    ("quantiser: zero-point ties away from zero", "float zf = clampf(rintf(-mn / sf), 0.0f, qmax);",
     "float zf = clampf(floorf(-mn / sf + 0.5f), 0.0f, qmax);", 1),
    ("quantiser: code ties away from zero", "float qf = clampf(rintf(w / sf) + zf, 0.0f, qmax);",
     "float qf = clampf(roundf(w / sf) + zf, 0.0f, qmax);", 1),
    ("fp64 -> fp16: ties up instead of to even", "double r = nearbyint(ldexp(a, 10 - p));",
     "double r = floor(ldexp(a, 10 - p) + 0.5);", 1),
    ("fp16 -> fp64: subnormal scale off by one bit", "v = ldexp((double)frac, -24); ", "v = ldexp((double)frac, -25); ", 1),
    ("interchange words: nibbles in reverse order", "& 0xF) << (4 * t);", "& 0xF) << (4 * (7 - t));", 2),
]


def _run_pins(src_path):
    env = dict(os.environ, ORACLE_W4_SRC=src_path)
    return subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                           "-p", "no:cacheprovider"], cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)


def test_every_planted_mistake_fails_a_pin(tmp_path):
    text = open(SRC).read()
    jobs = {}
    clean = tmp_path / "clean"
    clean.mkdir()
    shutil.copy(SRC, clean / "oracle_w4.c")
    jobs["(untouched copy)"] = str(clean / "oracle_w4.c")
    for i, (what, old, new, count) in enumerate(MUTATIONS):
        assert text.count(old) == count, f"mutation {i} ({what}): expected {count} place(s), found {text.count(old)}"
        d = tmp_path / f"m{i}"
        d.mkdir()
        (d / "oracle_w4.c").write_text(text.replace(old, new))
        jobs[what] = str(d / "oracle_w4.c")
    with concurrent.futures.ThreadPoolExecutor(max_workers=4) as pool:
        results = dict(zip(jobs, pool.map(_run_pins, jobs.values())))
    ok = results.pop("(untouched copy)")
    assert ok.returncode == 0, "the untouched copy must pass its pins:\n" + ok.stdout[-2000:]
    survivors = [what for what, r in results.items() if r.returncode == 0]
    assert not survivors, f"planted mistakes no pin caught: {survivors}"
    for what, r in results.items():
        assert "failed" in r.stdout or "error" in r.stdout.lower(), (what, r.stdout[-500:])
