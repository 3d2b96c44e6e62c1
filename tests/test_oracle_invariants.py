"""Post-conditions of the algebra, by brute force over small layouts (oracle/bruteforce.cpp),
plus a few invariants checked from Python with numpy on the same oracle."""
import itertools
import os
import subprocess

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def bruteforce_binary():
    src = [os.path.join(ROOT, "oracle", f) for f in ("bruteforce.cpp", "layout_oracle.cpp")]
    out = os.path.join(ROOT, "oracle", "bruteforce")
    hdr = os.path.join(ROOT, "oracle", "layout_oracle.hpp")
    if not os.path.exists(out) or os.path.getmtime(out) < max(os.path.getmtime(p) for p in src + [hdr]):
        subprocess.check_call(["g++", "-std=c++17", "-O2", "-fopenmp", "-o", out] + src)
    return out


def test_bruteforce_universe(bruteforce_binary):
    """Every layout of rank <= 3 with extents <= 4 (all mode orders, one stride zeroed, one boundary
    padded, every regrouping) and every stride in 0..6; all ordered pairs of the rank <= 2 subset and
    20000 seeded random pairs.  The rank-4 / extent-8 universe of the first workload is the slow test below."""
    r = subprocess.run([bruteforce_binary], capture_output=True, text=True, timeout=900)
    assert r.returncode == 0, r.stdout[-3000:]
    assert "ALL POST-CONDITIONS HOLD" in r.stdout
    # the sweep must actually have exercised successful results of every operation
    for line in r.stdout.splitlines():
        f = line.split()
        if len(f) >= 6 and f[1] == "cases" and f[0] not in ("composition_refused", "logical_product_sampled"):
            assert int(f[4]) > 1000, line


def _tally_lines(text):
    return sorted(ln.split() for ln in text.splitlines() if " cases " in ln)


def test_rank4_extent8_universe_tally_is_committed():
    """BASELINE config 1's universe (every layout with at most 4 modes and extents at most 8): the tally that
    tests/golden/make_bruteforce_tally.py wrote is in the repository, covers every operation and reports no failure."""
    path = os.path.join(ROOT, "tests", "golden", "bruteforce_rank4_extent8.txt")
    text = open(path).read()
    assert "--rank 4 --extent 8" in text.splitlines()[0]
    assert "ALL POST-CONDITIONS HOLD" in text and "exit status 0" in text
    names = set()
    for f in _tally_lines(text):
        names.add(f[0])
        assert f[-1] == "0" and f[-2] == "failed", f
        if f[0] in ("coalesce", "coalesce_bymode", "right_inverse", "complement"):
            assert int(f[2]) > 4000000, f            # the whole unary universe, every regrouping
        if f[0] in ("composition", "logical_divide"):
            assert int(f[2]) > 300000000 and int(f[4]) > 100000000, f
    assert {"coalesce", "complement", "right_inverse", "left_inverse", "composition", "logical_divide", "zipped_divide",
            "logical_product", "blocked_raked_product", "max_common_vector"} <= names


@pytest.mark.slow
@pytest.mark.skipif(os.environ.get("RUN_SLOW_UNIVERSE") != "1", reason="about three hours on 8 cores: set RUN_SLOW_UNIVERSE=1")
def test_rank4_extent8_universe_rerun():
    """Runs the universe again and compares its tally with the committed one."""
    import importlib.util
    spec = importlib.util.spec_from_file_location("make_tally", os.path.join(ROOT, "tests", "golden", "make_bruteforce_tally.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    import tempfile
    rc, text = mod.run(parts_dir=tempfile.mkdtemp(), fresh=True)
    assert rc == 0, text[-3000:]
    assert _tally_lines(text) == _tally_lines(open(mod.OUT).read())


def _flat_layouts(max_rank, max_extent):
    for r in range(1, max_rank + 1):
        for shape in itertools.product(range(1, max_extent + 1), repeat=r):
            for perm in itertools.permutations(range(r)):
                d, run = [0] * r, 1
                for m in perm:
                    d[m] = run
                    run *= shape[m]
                yield shape, tuple(d)


def _text(shape, stride):
    if len(shape) == 1:
        return "%d:%d" % (shape[0], stride[0])
    return "(%s):(%s)" % (",".join(map(str, shape)), ",".join(map(str, stride)))


def test_compact_layouts_are_bijections_with_two_sided_inverse(oracle):
    # Sec. 3.4.1: a bijection on Z_|L| has a full inverse: L(L^-1(k)) = k = L^-1(L(k))
    for shape, stride in _flat_layouts(3, 5):
        L = oracle.Layout(_text(shape, stride))
        inv = oracle.right_inverse(L)
        n = L.size
        assert inv.size == n
        f, g = L.offsets(), inv.offsets()
        assert (f[g] == np.arange(n)).all() and (g[f] == np.arange(n)).all()
        # and its complement is the single mode that steps over the whole image (Table complements, row 1-3)
        assert str(oracle.complement(L)) == "1:%d" % n


def test_column_major_compact_is_identity(oracle):
    # closed form: strides = exclusive prefix products of the extents => L(i) = i (identity layouts, Sec. 3.3.1)
    for shape in itertools.product(range(1, 6), repeat=3):
        stride = (1, shape[0], shape[0] * shape[1])
        L = oracle.Layout(_text(shape, stride))
        assert (L.offsets() == np.arange(L.size)).all()
        assert str(oracle.coalesce(L)) in ("%d:1" % L.size, "1:0")


def test_layout_function_against_numpy_strides(oracle):
    # a flat layout is numpy's (shape, strides) with Fortran-order enumeration of coordinates
    rng = np.random.default_rng(7)
    for _ in range(200):
        r = int(rng.integers(1, 5))
        shape = tuple(int(x) for x in rng.integers(1, 7, size=r))
        stride = tuple(int(x) for x in rng.integers(0, 40, size=r))
        L = oracle.Layout(_text(shape, stride))
        base = np.arange(L.cosize, dtype=np.int64)
        view = np.lib.stride_tricks.as_strided(base, shape=shape, strides=tuple(8 * d for d in stride))
        assert (L.offsets() == view.flatten(order="F")).all()


def test_composition_identity_laws(oracle):
    # Sec. 3.3.1: I_D o B = B and A o I_S = A (as functions; printed form for flat inputs)
    for shape, stride in _flat_layouts(3, 4):
        A = oracle.Layout(_text(shape, stride))
        n = A.size
        ident = "%d:1" % max(A.cosize, 1)
        assert (oracle.composition(ident, A).offsets() == A.offsets()).all()
        right = oracle.Layout(_text(shape, tuple(int(np.prod(shape[:k])) for k in range(len(shape)))))
        assert (oracle.composition(A, right).offsets() == A.offsets()).all()
        assert n == right.size


def test_associativity_when_images_nest(oracle):
    # Sec. 3.3.1: image(C) inside Z(B) and image(B) inside Z(A) => A o (B o C) = (A o B) o C
    rng = np.random.default_rng(11)
    done = 0
    compact = [(_text(s, d)) for s, d in _flat_layouts(3, 4)]
    while done < 300:
        A, B, C = (oracle.Layout(compact[int(rng.integers(len(compact)))]) for _ in range(3))
        if B.size == 1 or C.size == 1:
            continue
        if C.cosize > B.size or B.cosize > A.size:
            continue
        try:
            bc = oracle.composition(B, C)
            ab = oracle.composition(A, B)
            lhs = oracle.composition(A, bc)
            rhs = oracle.composition(ab, C)
        except oracle.OracleError:
            continue
        assert (lhs.offsets() == rhs.offsets()).all(), (A, B, C)
        done += 1


def test_zipped_divide_of_partition_workload(oracle):
    # third workload: (S,D,H,B) col-major over (D,S,H,B), tiler <128,64>; the rest mode keeps untouched modes whole
    z = oracle.zipped_divide("(4096,128,32,64):(128,1,524288,16777216)", "(128,64):(1,1)")
    assert str(z) == "((128,64),(32,2,32,64)):((128,1),(16384,64,524288,16777216))"
