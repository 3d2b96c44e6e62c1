#!/usr/bin/env python3
"""Writes tests/golden/bruteforce_rank4_extent8.txt: the tally of oracle/bruteforce over the universe BASELINE config 1
names (every layout with at most 4 modes and extents at most 8: all mode orders, one stride zeroed, one boundary
padded, every regrouping) for the unary operations, all ordered pairs of the rank <= 3 / extent <= 3 subset and 2500
seeded random pairs drawn from the whole universe for the binary ones (pairs of layouts of up to 4096 elements each are
checked coordinate by coordinate; most take a fraction of a second, a few take minutes: 2500 of them cost about an hour
of one core pair, 20 000 did not finish in 14 core hours).  Calls only oracle/ code.

The run takes about three hours on 8 cores, so it is cut into parts (the unary phase, 32 slices of the pair phase, the random
pairs) whose tallies add up; each part's output is kept under PARTS (default: a directory beside this file's output in the
system's temporary directory, or $BRUTEFORCE_PARTS), and a part that is already there is not run again: an interrupted
run picks up where it stopped.  `RUN_SLOW_UNIVERSE=1 pytest -m slow` runs everything again and compares."""
import os
import subprocess
import sys
import tempfile
import time

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
RANDOM_PAIRS = os.environ.get("BRUTEFORCE_RANDOM", "2500")   # the committed tally was written with the default
BASE = ["--rank", "4", "--extent", "8", "--pair-rank", "3", "--pair-extent", "3", "--random", RANDOM_PAIRS, "--product-budget", "4096"]
SLICES = 32
OUT = os.path.join(ROOT, "tests", "golden", "bruteforce_rank4_extent8.txt")


def build():
    src = [os.path.join(ROOT, "oracle", f) for f in ("bruteforce.cpp", "layout_oracle.cpp")]
    exe = os.path.join(ROOT, "oracle", "bruteforce")
    subprocess.check_call(["g++", "-std=c++17", "-O2", "-fopenmp", "-o", exe] + src)
    return exe


def parts():
    yield "unary", ["--phases", "unary"]
    for k in range(SLICES):
        yield "pairs_%02d_of_%d" % (k, SLICES), ["--phases", "pairs", "--pair-slice", "%d/%d" % (k, SLICES)]
    yield "random", ["--phases", "random"]


def tally_of(text):
    t = {}
    for ln in text.splitlines():
        f = ln.split()
        if len(f) >= 7 and f[1] == "cases":
            t[f[0]] = (int(f[2]), int(f[4]), int(f[6]))
    return t


def run(parts_dir=None, fresh=False):
    exe = build()
    parts_dir = parts_dir or os.environ.get("BRUTEFORCE_PARTS") or os.path.join(tempfile.gettempdir(), "bruteforce_rank4_extent8_parts")
    os.makedirs(parts_dir, exist_ok=True)
    total, seconds, rc, headers, failures = {}, 0.0, 0, [], []
    for name, extra in parts():
        path = os.path.join(parts_dir, name + ".txt")
        if fresh or not os.path.exists(path):
            t0 = time.time()
            r = subprocess.run([exe] + BASE + extra, capture_output=True, text=True)
            text = "# part %s: exit status %d, %.0f s\n%s" % (name, r.returncode, time.time() - t0, r.stdout)
            with open(path + ".tmp", "w") as f:
                f.write(text)
            os.replace(path + ".tmp", path)
            print("part", name, "done in %.0f s" % (time.time() - t0), flush=True)
        text = open(path).read()
        first = text.splitlines()[0]
        rc |= int(first.split("exit status ")[1].split(",")[0])
        seconds += float(first.split(", ")[1].split(" s")[0])
        if name == "unary":
            headers = [ln for ln in text.splitlines() if ln.startswith("unary universe")]
        if name == "random":   # the part that names the number of random pairs it really ran
            headers += [ln for ln in text.splitlines() if ln.startswith("pair universe")]
        failures += [ln for ln in text.splitlines() if "first failure" in ln]
        for k, v in tally_of(text).items():
            s = total.get(k, (0, 0, 0))
            total[k] = tuple(a + b for a, b in zip(s, v))
    lines = ["# command: oracle/bruteforce %s, run as %d parts (--phases unary | --phases pairs --pair-slice k/%d | --phases random) whose tallies are added"
             % (" ".join(BASE), SLICES + 2, SLICES),
             "# exit status %d, %.0f s of part run time in all" % (rc, seconds)] + headers
    for k in sorted(total):
        lines.append("%-40s cases %10d  checked-ok %10d  failed %d" % (k, total[k][0], total[k][1], total[k][2]))
    lines += failures
    lines.append("FAILED" if rc or any(v[2] for v in total.values()) else "ALL POST-CONDITIONS HOLD")
    return rc, "\n".join(lines) + "\n"


if __name__ == "__main__":
    rc, text = run()
    with open(OUT, "w") as f:
        f.write(text)
    sys.stdout.write(text)
    sys.exit(rc)
