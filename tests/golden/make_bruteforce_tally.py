#!/usr/bin/env python3
"""Writes tests/golden/bruteforce_rank4_extent8.txt: the tally of oracle/bruteforce over the universe BASELINE config 1
names (every layout with at most 4 modes and extents at most 8: all mode orders, one stride zeroed, one boundary
padded, every regrouping) for the unary operations, all ordered pairs of the rank <= 3 / extent <= 3 subset and 10^6
seeded random pairs drawn from the whole universe for the binary ones.  Calls only oracle/ code.  About an hour on
8 cores; `pytest -m slow` (RUN_SLOW_UNIVERSE=1) runs it again and compares."""
import os
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
ARGS = ["--rank", "4", "--extent", "8", "--pair-rank", "3", "--pair-extent", "3", "--random", "1000000", "--product-budget", "4096"]
OUT = os.path.join(ROOT, "tests", "golden", "bruteforce_rank4_extent8.txt")


def build():
    src = [os.path.join(ROOT, "oracle", f) for f in ("bruteforce.cpp", "layout_oracle.cpp")]
    exe = os.path.join(ROOT, "oracle", "bruteforce")
    subprocess.check_call(["g++", "-std=c++17", "-O2", "-fopenmp", "-o", exe] + src)
    return exe


def run():
    exe = build()
    t0 = time.time()
    r = subprocess.run([exe] + ARGS, capture_output=True, text=True)
    text = "# command: oracle/bruteforce %s\n# exit status %d, %.0f s, OMP threads %s\n%s" % (
        " ".join(ARGS), r.returncode, time.time() - t0, os.environ.get("OMP_NUM_THREADS", "all"), r.stdout)
    return r.returncode, text


if __name__ == "__main__":
    rc, text = run()
    with open(OUT, "w") as f:
        f.write(text)
    sys.stdout.write(text)
    sys.exit(rc)
