"""Layouts with integer-semimodule strides (Sec. 2.3.2): coordinate layouts (strides a*e_i) and XOR
layouts (strides f_d).  The oracle is pinned to what the paper prints (tests/golden/semimodule_layouts.txt)
and to the definition by brute force; the library is compared with the oracle."""
import numpy as np
import pytest

import paper_2603_02298_amd as lc
from conftest import golden_lines


def _parse_fixture():
    lines = golden_lines("semimodule_layouts.txt")
    mats, comps, rinvs = [], [], []
    i = 0
    while i < len(lines):
        ln = lines[i]
        if ln.startswith("matrix "):
            text = ln[len("matrix "):].split("|")[0].strip()
            rows = [lines[i + 1 + r].split() for r in range(4)]
            mats.append((text, rows))
            i += 5
        elif ln.startswith("composition "):
            a, b, r, _ = [x.strip() for x in ln[len("composition "):].split("|")]
            comps.append((a, b, r))
            i += 1
        elif ln.startswith("right_inverse "):
            a, r, _ = [x.strip() for x in ln[len("right_inverse "):].split("|")]
            rinvs.append((a, r))
            i += 1
        else:
            raise AssertionError(ln)
    return mats, comps, rinvs


def _value(text):
    return tuple(int(x) for x in text.split(",")) if "," in text else int(text)


@pytest.mark.parametrize("side", ["oracle", "library"])
def test_printed_layouts(oracle, side):
    S = oracle.SLayout if side == "oracle" else lc.SLayout
    compose = oracle.slayout_composition if side == "oracle" else lc.lc_slayout_composition
    rinv = oracle.slayout_right_inverse if side == "oracle" else lc.lc_slayout_right_inverse
    mats, comps, rinvs = _parse_fixture()
    assert len(mats) == 3 and len(comps) == 2 and len(rinvs) == 2
    for text, rows in mats:
        L = S(text)
        assert str(L) == text
        ncol = len(rows[0])
        for m in range(4):
            for n in range(ncol):
                assert L(m + 4 * n) == _value(rows[m][n]), (text, m, n)     # the matrices are 4 x N, column-major coordinates
    for a, b, r in comps:
        assert str(compose(a, b)) == r, (a, b)
    for a, r in rinvs:
        assert str(rinv(a)) == r, a


def test_definition_by_brute_force(oracle):
    # Eq. innerprod in the semimodule, retyped here: digits of the integral coordinate (colexicographic,
    # Sec. 2.2.2) times the strides, added per axis (e_i) or by XOR (f_d)
    rng = np.random.default_rng(232)
    for trial in range(300):
        n = int(rng.integers(1, 5))
        ext = [int(rng.integers(1, 6)) for _ in range(n)]
        kind = ["e", "f", "i"][trial % 3]
        if kind == "e":
            strides = [(int(rng.integers(0, 7)), int(rng.integers(0, 3))) for _ in range(n)]
            text = ",".join(("%de%d" % s) if s[0] else "0" for s in strides)
        elif kind == "f":
            strides = [(int(rng.integers(0, 40)), 0) for _ in range(n)]
            text = ",".join("f%d" % s[0] for s in strides)
        else:
            strides = [(int(rng.integers(0, 40)), 0) for _ in range(n)]
            text = ",".join(str(s[0]) for s in strides)
        layout = ("(%s):(%s)" % (",".join(map(str, ext)), text)) if n > 1 else "%d:%s" % (ext[0], text)
        Lo, Ll = oracle.SLayout(layout), lc.SLayout(layout)
        size = int(np.prod(ext))
        rank = 1 + max([s[1] for s in strides if s[0]] + [0]) if kind == "e" else 1
        for i in range(size + 3):
            digits, q = [], i
            for k, e in enumerate(ext):
                digits.append(q if k == n - 1 else q % e)
                q //= e
            if kind == "e" and any(s[0] for s in strides):
                want = [0] * rank
                for dgt, s in zip(digits, strides):
                    if s[0]:
                        want[s[1]] += dgt * s[0]
                want = tuple(want)
            elif kind == "f":
                want = 0
                for dgt, s in zip(digits, strides):
                    want ^= dgt * s[0]
            else:
                want = sum(dgt * s[0] for dgt, s in zip(digits, strides))
            assert Lo(i) == want, (layout, i)
            assert Ll(i) == want, (layout, i)


def _random_int_layout(rng):
    n = int(rng.integers(1, 4))
    ext = [int(rng.choice([1, 2, 3, 4, 6, 8])) for _ in range(n)]
    st = [int(rng.choice([0, 1, 2, 3, 4, 6, 8, 12, 16])) for _ in range(n)]
    return "(%s):(%s)" % (",".join(map(str, ext)), ",".join(map(str, st))) if n > 1 else "%d:%d" % (ext[0], st[0])


def test_composition_with_coordinate_strides(oracle):
    # Z^(*,..,*) is a module, so R(c) = A(B(c)) must hold for every admissible B; library == oracle in print
    rng = np.random.default_rng(233)
    done = 0
    for _ in range(1500):
        n = int(rng.integers(1, 4))
        ext = [int(rng.choice([2, 3, 4, 6, 8])) for _ in range(n)]
        axes = [int(rng.integers(0, 3)) for _ in range(n)]
        coef = [int(rng.integers(1, 5)) for _ in range(n)]
        A = "(%s):(%s)" % (",".join(map(str, ext)), ",".join("%de%d" % (c, a) for c, a in zip(coef, axes))) if n > 1 else "%d:%de%d" % (ext[0], coef[0], axes[0])
        B = _random_int_layout(rng)
        try:
            Ro = oracle.slayout_composition(A, B)
        except oracle.OracleError as e:
            with pytest.raises(lc.LayoutCopyError) as le:
                lc.lc_slayout_composition(A, B)
            assert le.value.status_name == e.status_name, (A, B)
            continue
        Rl = lc.lc_slayout_composition(A, B)
        assert str(Rl) == str(Ro), (A, B)
        Ao, Bo = oracle.SLayout(A), oracle.Layout(B)
        if Bo.cosize > int(np.prod(ext)):
            continue                      # B reaches past A's domain: only the shapes were compared
        rank = max(len(Ao(0)), 1)
        for c in range(Bo.size):
            got, want = Ro(c), Ao(Bo(c))
            got = got if isinstance(got, tuple) else (got,)
            got = got + (0,) * (rank - len(got))
            assert got == want, (A, B, c)
        done += 1
    assert done > 300, done


def test_right_inverse_of_coordinate_layouts(oracle):
    rng = np.random.default_rng(234)
    checked = 0
    for _ in range(400):
        n = int(rng.integers(1, 5))
        ext = [int(rng.choice([1, 2, 3, 4, 5])) for _ in range(n)]
        axes = [int(rng.integers(0, 2)) for _ in range(n)]
        coef = [int(rng.choice([0, 1, 1, 2, 3, 4, 6])) for _ in range(n)]
        A = "(%s):(%s)" % (",".join(map(str, ext)), ",".join(("%de%d" % (c, a)) if c else "0" for c, a in zip(coef, axes))) if n > 1 else \
            "%d:%s" % (ext[0], ("%de%d" % (coef[0], axes[0])) if coef[0] else "0")
        Ao = oracle.SLayout(A)
        if Ao.kind != "coord":
            continue
        Ro, Rl = oracle.slayout_right_inverse(A), lc.lc_slayout_right_inverse(A)
        assert str(Ro) == str(Rl), A
        rank = len(Ao(0))
        # A(R(c)) = c for every coordinate c of R's domain: R has one top-level mode per axis, so the
        # integral coordinate i of R splits colexicographically into the per-axis coordinates
        import re
        shape = str(Ro).split(":")[0]
        if rank == 1:
            sizes = [int(np.prod([int(x) for x in re.findall(r"\d+", shape)]))]
        else:
            depth, parts, cur = 0, [], ""
            for ch in shape[1:-1]:
                if ch == "," and depth == 0:
                    parts.append(cur)
                    cur = ""
                    continue
                depth += ch == "("
                depth -= ch == ")"
                cur += ch
            parts.append(cur)
            sizes = [int(np.prod([int(x) for x in re.findall(r"\d+", part)])) for part in parts]
        assert len(sizes) == rank, (A, str(Ro))
        R = oracle.Layout(str(Ro))
        assert R.size == int(np.prod(sizes))
        for i in range(R.size):
            crd, q = [], i
            for sz in sizes:
                crd.append(q % sz)
                q //= sz
            assert Ao(R(i)) == tuple(crd), (A, str(Ro), i)
        # and the box is as large as it can be along every axis: one more step is not in the image, or not invertible there
        checked += 1
    assert checked > 200, checked


def test_coalesce_keeps_the_function(oracle):
    rng = np.random.default_rng(235)
    for trial in range(400):
        n = int(rng.integers(1, 5))
        ext = [int(rng.choice([1, 2, 2, 3, 4])) for _ in range(n)]
        if trial % 2:
            st = ["f%d" % int(rng.choice([0, 1, 2, 4, 5, 8, 16])) for _ in range(n)]
        else:
            ax = int(rng.integers(0, 2))
            st, run = [], 1
            for e in ext:
                r = rng.random()
                st.append("%de%d" % (run, ax) if r < 0.6 else ("%de%d" % (int(rng.integers(1, 9)), int(rng.integers(0, 2))) if r < 0.9 else "0"))
                run *= e
        A = "(%s):(%s)" % (",".join(map(str, ext)), ",".join(st)) if n > 1 else "%d:%s" % (ext[0], st[0])
        Ao = oracle.SLayout(A)
        Co, Cl = oracle.slayout_coalesce(A), lc.lc_slayout_coalesce(A)
        assert str(Co) == str(Cl), A
        for i in range(Ao.size):
            a, c = Ao(i), Co(i)
            a = a if isinstance(a, tuple) else (a,)
            c = c if isinstance(c, tuple) else (c,)
            m = max(len(a), len(c))
            assert a + (0,) * (m - len(a)) == c + (0,) * (m - len(c)), (A, i)


def test_lds_slot_layouts_are_derived_xor_layouts(oracle):
    # The transposing kernels park vector g of a tile at LDS slot g ^ ((g >> s) & m) [^ a second such term].  In the
    # paper's terms that is a layout over the bits of g with XOR strides (Sec. 2.3.2): bit b carries f_(2^b), and a bit
    # that a term folds down by s carries f_(2^b + 2^(b-s)).  The planner derives the folds from the park layout's bits and
    # prints the layout; here the semimodule libraries (ours and the oracle's) evaluate that text against the slot formula,
    # and the property the derivation is for is checked directly: the 8 lanes of a 16-byte write pass hit 8 different
    # 16-byte bank groups of the 128 bytes the banks span, for every pass and every vector of a tile.
    import re
    from paper_2603_02298_amd import workloads as W
    cases = [W.workload(n, sc) for n, sc in (("c1", 1), ("c2", 1), ("c2", 16), ("c3", 1), ("c5", 1), ("c5", 256))]
    layouts = [(w.src_layout, w.dst_layout, w.dtype) for w in cases]
    layouts += [("(64,2,64):(1,64,128)", "(64,2,64):(128,64,1)", "f32"),          # a park layout whose low lane bits come from two modes
                ("(16,4,64,8):(1,16,64,4096)", "(16,4,64,8):(2048,512,1,64)", "bf16")]
    derived = 0
    for s_, d_, dt in layouts:
        desc = lc.Plan(s_, d_, dt).describe()
        text = re.search(r"lds_layout=(\S+)", desc).group(1)
        sh = int(re.search(r"swizzle_shift=(-?\d+)", desc).group(1))
        derived += "swizzle=derived" in desc
        n_vec = 1 << text.split(":")[0].count("2")
        strides = [int(x[1:]) for x in text.split(":")[1].strip("()").split(",")]
        for S in (oracle.SLayout, lc.SLayout):
            L = S(text)
            for g in list(range(0, min(n_vec, 2048))) + [n_vec - 1]:
                want = 0
                for b, d in enumerate(strides):
                    if (g >> b) & 1:
                        want ^= d
                assert L(g) == want, (text, g)
        if sh >= 0:   # the first term is the printed shift: every bit it folds is shift above its target
            assert all(d == (1 << b) or d & ((1 << b) - 1) for b, d in enumerate(strides)), text
    assert derived >= 6, derived


def test_lds_bank_model_against_the_counter(oracle):
    # the planner's bank model against SQ_LDS_BANK_CONFLICT read on an MI355X for address patterns made for the purpose
    # (extra cycles per wavefront instruction; the summary of that run is under profiles/)
    import ctypes
    L = lc.lib()
    L.lc_debug_lds_conflicts.argtypes = [ctypes.POINTER(ctypes.c_uint32), ctypes.c_int, ctypes.c_int]

    def model(fn, width, write):
        a = (ctypes.c_uint32 * 64)(*[fn(l) for l in range(64)])
        return L.lc_debug_lds_conflicts(a, width, 1 if write else 0)
    measured = [   # (width, write?, pattern, extra cycles per instruction)
        (16, True, lambda l: l * 16, 0), (16, True, lambda l: l * 32, 8), (16, True, lambda l: l * 64, 24), (16, True, lambda l: (l * 128) % 65536, 56),
        (16, True, lambda l: (l % 8) * 16 + (l // 8) * 256, 0), (16, True, lambda l: (l % 4) * 16 + (l // 4) * 256, 8),
        (16, True, lambda l: (l % 4) * 16 + (l // 4) * 128, 8), (16, True, lambda l: (l % 8) * 16 + (l // 8) * 128, 0),
        (16, True, lambda l: (l // 2) * 16 + (l % 2) * 256, 8), (16, True, lambda l: (l % 8) * 16 + (l // 8) * 2048, 0),
        (16, False, lambda l: l * 16, 0), (16, False, lambda l: l * 32, 4), (16, False, lambda l: l * 64, 12), (16, False, lambda l: (l * 128) % 65536, 28),
        (16, False, lambda l: (l % 16) * 16 + (l // 16) * 256, 0), (16, False, lambda l: (l % 8) * 16 + (l // 8) * 256, 4),
        (16, False, lambda l: (l % 8) * 16 + (l // 8) * 128, 0), (16, False, lambda l: (l % 16) * 16 + (l // 16) * 128, 4),
        (16, False, lambda l: (l % 16) * 16 + (l // 16) * 2048, 0), (16, False, lambda l: (l % 8) * 16 + (l // 8) * 2048, 4),
        (16, False, lambda l: (l % 4) * 16 + (l // 4) * 2048, 12),
        (8, True, lambda l: l * 8, 0), (8, True, lambda l: l * 16, 4), (8, True, lambda l: (l % 16) * 8 + (l // 16) * 128, 0),
        (8, True, lambda l: (l % 8) * 8 + (l // 8) * 128, 4), (8, True, lambda l: (l % 16) * 8 + (l // 16) * 2048, 0),
        (8, False, lambda l: l * 8, 0), (8, False, lambda l: l * 16, 2), (8, False, lambda l: (l % 16) * 8 + (l // 16) * 128, 0),
        (8, False, lambda l: (l % 16) * 8 + (l // 16) * 256, 2), (8, False, lambda l: (l % 32) * 8 + (l // 32) * 2048, 0),
        (4, True, lambda l: l * 4, 0), (4, True, lambda l: l * 8, 2), (4, True, lambda l: (l % 16) * 4 + (l // 16) * 128, 2),
        (4, True, lambda l: (l % 32) * 4 + (l // 32) * 128, 0),
        (4, False, lambda l: l * 4, 0), (4, False, lambda l: l * 8, 2), (4, False, lambda l: (l % 16) * 4 + (l // 16) * 128, 2),
        (4, False, lambda l: (l % 32) * 4 + (l // 32) * 128, 0), (4, False, lambda l: (l * 64) % 65536, 30)]
    for width, write, fn, want in measured:
        assert model(fn, width, write) == want, (width, write, [fn(l) for l in range(8)], want)
    # the parking writes of a 32 x 32 fp32 tile (4 x 4 micro-tiles): folding bit 4 and up (what the old, 16-lanes-per-pass
    # model chose) leaves a 2-way conflict, 8 extra cycles per write, 32768 per launch of the 1024^2 transpose as the
    # counter showed; folding from bit 5 is free
    park = lambda fold: (lambda l: (lambda g: (g ^ ((g >> fold) & 15)) * 16)((l % 8) * 32 + (l // 8)))
    assert model(park(4), 16, True) == 8 and model(park(5), 16, True) == 0


def test_errors():
    for bad, status in [("(4,8):(e0)", "NOT_CONGRUENT"), ("(4,8):(e0,f1)", "INVALID_ARG"), ("(4,8):(e0,x)", "PARSE"),
                        ("(4,0):(e0,e1)", "BAD_EXTENT"), ("4:e99", "PARSE")]:
        with pytest.raises(lc.LayoutCopyError) as e:
            lc.SLayout(bad)
        assert e.value.status_name == status, bad
    with pytest.raises(lc.LayoutCopyError):
        lc.lc_slayout_right_inverse("(8,8):(f1,f9)")
    with pytest.raises(lc.LayoutCopyError) as e:
        lc.lc_slayout_composition("(8,8):(e0,e1)", "(4,3):(3,1)")     # stride 3 does not divide into the modes of (8,8)
    assert e.value.status_name in ("STRIDE_DIVISIBILITY", "SHAPE_DIVISIBILITY")


# ---------------------------------------------------------------------------------------------
# Right-inverse of layouts with XOR strides (Table rinv, last row: "possible to define"; the reading taken here:
# R = (2,...,2):(f_x0, f_x1, ...), x_b the smallest integral coordinate whose offset is 2^b, A(R(k)) = k on all of R).
# The printed FORM is this build's choice (parity unpinned); the defining property, the size and the special cases are pinned.
# ---------------------------------------------------------------------------------------------
def _brute_xor_right_inverse_size(A):
    """Largest j with a function r on [0, 2^j) that is a XOR layout over the bits of k and inverts A: found independently
    of either implementation by trying, for growing j, whether the smallest preimages of 2^0 .. 2^(j-1) combine."""
    img = [A(i) for i in range(A.size)]
    first = {}
    for i, v in enumerate(img):
        first.setdefault(v, i)
    xs = []
    while (1 << len(xs)) in first:
        xs.append(first[1 << len(xs)])
    for j in range(len(xs), -1, -1):
        ok = True
        for k in range(1 << j):
            c = 0
            for b in range(j):
                if (k >> b) & 1:
                    c ^= xs[b]
            if c >= A.size or img[c] != k:
                ok = False
                break
        if ok:
            return j, xs[:j]
    return 0, []


def test_xor_right_inverse_oracle_pins(oracle):
    # the swizzle of Table TVLayoutExamples' Swizzled row is its own inverse (XOR-ing bit 3.. into bit 0.. twice is the identity)
    r = oracle.slayout_xor_right_inverse("(8,8):(f1,f9)")
    assert str(r) == "(2,2,2,2,2,2):(f1,f2,f4,f9,f18,f36)"
    assert all(oracle.SLayout("(8,8):(f1,f9)")(r(k)) == k for k in range(64)) and all(r(k) == oracle.SLayout("(8,8):(f1,f9)")(k) for k in range(64))
    # Table rinv's own XOR example, (4,(4,3)):(f1,(f5,f16)): offsets 0..31 are inverted; 32 is reached (coordinate 32) but
    # 16 xor 32 = 48 is no coordinate of a 48-element layout
    A = oracle.SLayout("(4,(4,3)):(f1,(f5,f16))")
    r = oracle.slayout_xor_right_inverse(A)
    assert r.size == 32 and all(A(r(k)) == k for k in range(32))
    # strides that are plain powers of two: XOR is addition, the inverse is the ordinary right-inverse of the integer layout
    for text, ints in (("(4,4):(f1,f4)", "(4,4):(1,4)"), ("(8,2,4):(f8,f1,f2)", "(8,2,4):(8,1,2)"), ("(4,2):(f2,f1)", "(4,2):(2,1)")):
        r, ri = oracle.slayout_xor_right_inverse(text), oracle.right_inverse(ints)
        assert r.size == ri.size and all(r(k) == ri(k) for k in range(r.size)), (text, str(r), str(ri))
    # nothing to invert: 1 is not in the image; a carry inside a mode (3 * f3 = f9, not f3 xor f6) ends the inverse early
    assert str(oracle.slayout_xor_right_inverse("(4,4):(f3,f12)")) == "1:0"
    A = oracle.SLayout("(4,4):(f1,f3)")
    r = oracle.slayout_xor_right_inverse(A)
    assert r.size == 8 and all(A(r(k)) == k for k in range(8))
    # brute force: random XOR layouts, additive or not; the size is the largest that works, the modes are the smallest preimages
    rng = np.random.default_rng(5)
    for _ in range(300):
        rank = int(rng.integers(1, 4))
        ext = [int(rng.choice([2, 3, 4, 8])) for _ in range(rank)]
        strides = [int(rng.integers(0, 40)) for _ in range(rank)]
        text = "(%s):(%s)" % (",".join(map(str, ext)), ",".join("f%d" % d if d else "0" for d in strides))
        if all(d == 0 for d in strides):
            continue
        A = oracle.SLayout(text)
        j, xs = _brute_xor_right_inverse_size(A)
        r = oracle.slayout_xor_right_inverse(A)
        assert r.size == (1 << j), (text, str(r), j)
        assert all(A(r(k)) == k for k in range(r.size)), text
        if j:
            assert str(r) == ("(%s):(%s)" % (",".join(["2"] * j), ",".join("f%d" % x for x in xs)) if j > 1 else "2:f%d" % xs[0]), (text, str(r), xs)


def test_xor_right_inverse_library_against_oracle(oracle):
    # the library eliminates over F2 (layouts that are additive over XOR of coordinates); the oracle applies the definition
    cases = ["(8,8):(f1,f9)", "(4,4):(f1,f5)", "(4,4):(f1,f4)", "(8,2,4):(f8,f1,f2)", "(4,2):(f2,f1)", "(4,4):(f3,f12)",
             "(2,2,2,2,2,2,2,2,2,2,2):(f1,f2,f4,f8,f16,f32,f65,f130,f260,f512,f1024)",     # the LDS slot layout of workload 2's tiles
             "(2,2,2,2):(f1,f1,f2,f4)",                                                  # not injective: the smallest preimage is taken
             "(4,4,4):(f1,f1,f4)", "(2,4,2):(f6,f1,f4)", "(16,4):(f3,f48)"]
    rng = np.random.default_rng(6)
    for _ in range(200):
        rank = int(rng.integers(1, 5))
        ext = [int(rng.choice([2, 4, 8])) for _ in range(rank)]
        text = "(%s):(%s)" % (",".join(map(str, ext)), ",".join("f%d" % int(rng.integers(1, 64)) for _ in range(rank)))
        cases.append(text)
    for _ in range(200):   # strides of one or two bits far enough apart that a mode's multiples meet no carry: always additive
        rank = int(rng.integers(1, 5))
        ext = [int(rng.choice([2, 4, 8])) for _ in range(rank)]
        ds = []
        for e in ext:
            lo = int(rng.integers(0, 6))
            d = 1 << lo
            if rng.integers(0, 2):
                d |= 1 << (lo + e.bit_length() - 1 + int(rng.integers(0, 3)))
            ds.append(d)
        cases.append("(%s):(%s)" % (",".join(map(str, ext)), ",".join("f%d" % d for d in ds)))
    checked = 0
    for text in cases:
        want = oracle.slayout_xor_right_inverse(text)
        try:
            got = lc.lc_slayout_xor_right_inverse(text)
        except lc.LayoutCopyError as e:
            # refused: some stride's multiples carry inside its mode (the oracle's inverse then stops where additivity does)
            assert e.status_name == "INVALID_ARG", text
            A = oracle.SLayout(text)
            ext = [int(x) for x in text.split(":")[0].strip("()").split(",")]
            ds = [int(x[1:]) for x in text.split(":")[1].strip("()").split(",")]
            assert any(any(c * d != _xor_multiples(c, d) for c in range(e_)) for e_, d in zip(ext, ds)), text
            continue
        assert str(got) == str(want), (text, str(got), str(want))
        A = lc.SLayout(text)
        assert all(A(got(k)) == k for k in range(got.size)), text
        checked += 1
    assert checked > 200
    for bad in ("(3,4):(f1,f4)", "(4,4):(f1,f3)", "(4,4):(1,4)", "(4,4):(e0,e1)"):
        with pytest.raises(lc.LayoutCopyError):
            lc.lc_slayout_xor_right_inverse(bad)


def _xor_multiples(c, d):
    r, u = 0, 0
    while c >> u:
        if (c >> u) & 1:
            r ^= d << u
        u += 1
    return r


# ---------------------------------------------------------------------------------------------
# Composition with XOR strides.  The construction of Sec. 3.3 (each mode of the result walks one leaf of A and takes that
# leaf's stride scaled by its step) is functional composition only while the modes that walk one leaf add up without a
# carry; the oracle compares its result with A(B(c)) and refuses otherwise.  Pinned here to hand-checked cases and to a
# closed form of "a carry can happen" that is derived independently: mode j of the result contributes c_j * m_j with
# m_j = step_j * d_k, and two modes in one leaf can carry iff the OR of their possible contributions share a bit.
# ---------------------------------------------------------------------------------------------
XOR_COMPOSITION_SIDES = ["oracle", "library"]


def _xor_sides(oracle, side):
    return (oracle.slayout_composition, oracle.OracleError) if side == "oracle" else (lc.lc_slayout_composition, lc.LayoutCopyError)


@pytest.mark.parametrize("side", XOR_COMPOSITION_SIDES)
def test_xor_composition_hand_cases(oracle, side):
    compose, error = _xor_sides(oracle, side)
    # A = 4:f5, B = (2,2):(1,2): contributions {0,5} and {0,10} share no bit: R = (2,2):(f5,f10), R(1,1) = 15 = A(3)
    R = compose("4:f5", "(2,2):(1,2)")
    assert str(R) == "(2,2):(f5,f10)" and R(3) == 15 and oracle.SLayout("4:f5")(3) == 15
    # A = 8:f3, B = (2,2):(1,2): {0,3} and {0,6} meet in bit 1: A(B(1,1)) = A(3) = 9 but f3 xor f6 = 5: no layout result
    with pytest.raises(error) as e:
        compose("8:f3", "(2,2):(1,2)")
    assert e.value.status_name == "NOT_SEGREGATED"
    # a single mode of B per leaf never carries, whatever the stride
    assert str(compose("(8,8):(f3,f24)", "(4,4):(2,8)")) == "(4,4):(f6,f24)"


def _random_xor_layout(rng):
    n = int(rng.integers(1, 4))
    ext = [int(rng.choice([2, 4, 8, 3, 6])) for _ in range(n)]
    st = [int(rng.choice([1, 2, 3, 4, 5, 8, 9, 16, 17, 24])) for _ in range(n)]
    return "(%s):(%s)" % (",".join(map(str, ext)), ",".join("f%d" % d for d in st)) if n > 1 else "%d:f%d" % (ext[0], st[0])


@pytest.mark.parametrize("side", XOR_COMPOSITION_SIDES)
def test_xor_composition_is_exact_or_refused(oracle, side):
    compose, error = _xor_sides(oracle, side)
    rng = np.random.default_rng(235)
    composed = refused = 0
    for _ in range(3000):
        A, B = _random_xor_layout(rng), _random_int_layout(rng)
        Ao, Bo = oracle.SLayout(A), oracle.Layout(B)
        # the closed form, from the integer composition of the proxy layouts alone: P has A's shape and place values
        # with a gap of 2 after each leaf, so a mode of P o B with stride t walks leaf k = the last leaf whose place <= t
        ext = [int(x) for x in A.split(":")[0].strip("()").split(",")]
        ds = [int(x[1:]) for x in A.split(":")[1].strip("()").split(",")]
        place, run = [], 1
        for e_ in ext:
            place.append(run)
            run *= 2 * e_
        P = "(%s):(%s)" % (",".join(map(str, ext)), ",".join(map(str, place))) if len(ext) > 1 else "%d:%d" % (ext[0], place[0])
        try:
            PB = oracle.composition(P, B)
        except oracle.OracleError as err:
            with pytest.raises(error) as e2:
                compose(A, B)
            assert e2.value.status_name == err.status_name, (A, B)
            continue
        import re
        shp, strd = [[int(x) for x in re.findall(r"\d+", part)] for part in str(PB).split(":")]
        masks = {}
        carry = False
        for s_, t in zip(shp, strd):
            if s_ == 1 or t == 0:
                continue
            k = max(i for i in range(len(place)) if place[i] <= t)
            if t % place[k]:
                carry = None          # not a walk inside one leaf: refused for another reason
                break
            m = (t // place[k]) * ds[k]
            mask = 0
            for c in range(s_):
                mask |= c * m
            for other in masks.setdefault(k, []):
                carry = carry or bool(other & mask)
            masks[k].append(mask)
        if carry is None:
            continue
        if carry:
            with pytest.raises(error) as e2:
                compose(A, B)
            assert e2.value.status_name == "NOT_SEGREGATED", (A, B)
            refused += 1
            continue
        R = compose(A, B)
        assert str(R) == str(oracle.slayout_composition(A, B)), (A, B)
        for c in range(Bo.size):
            assert R(c) == Ao(Bo(c)), (A, B, c)
        composed += 1
    assert composed > 300 and refused > 100, (composed, refused)
