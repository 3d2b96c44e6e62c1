"""The oracle against what the paper prints: coordinate lists, offset matrices, worked
algebra results, slices.  Values live in tests/golden/ with their citations."""
import numpy as np
import pytest

from conftest import golden_lines


def _blocks(lines):
    i = 0
    while i < len(lines):
        assert lines[i].startswith("layout ")
        text, cite = [x.strip() for x in lines[i][len("layout "):].split("|")]
        _, r, c = lines[i + 1].split()
        r, c = int(r), int(c)
        mat = np.array([[int(x) for x in lines[i + 2 + k].split()] for k in range(r)], dtype=np.int64)
        assert mat.shape == (r, c)
        yield text, cite, mat
        i += 2 + r


def test_coordinate_lists(oracle):
    # Fig. coordlists: idx2crd for every compatible coordinate set, and crd2idx as its inverse
    for ln in golden_lines("coordinate_lists.txt"):
        shape, i, crd = [x.strip() for x in ln.split("|")]
        assert oracle.idx2crd(shape, int(i)) == crd, ln
    L = oracle.Layout("((2,3),2):((1,2),6)")
    for i in range(12):
        assert L.crd2idx(L.natural(i)) == i
        assert L.crd2idx(oracle.idx2crd("(6,2)", i)) == i


def test_idx2crd_beyond_size_is_out_of_bounds(oracle):
    # Sec. 2.2.2, out-of-bounds coordinates: only the last entry grows
    assert oracle.idx2crd("(2,3)", 6) == "(0,3)"
    assert oracle.idx2crd("(2,3)", 11) == "(1,5)"
    assert oracle.idx2crd("((2,3),2)", 12) == "((0,0),2)"


def test_congruence_and_compatibility_examples(oracle):
    # Sec. 2.1 and Sec. 2.2.1 worked examples
    assert oracle.congruent("(4,8)", "(5,7)") and oracle.congruent("(4,(2,4))", "(7,(3,2))")
    assert not oracle.congruent("(4,8)", "(4,(2,4))") and not oracle.congruent("(4,(2,4))", "(0,((0,0)))")
    assert oracle.weakly_congruent("30", "(1,2)") and oracle.weakly_congruent("(1,2)", "(5,(0,7))")
    assert oracle.weakly_congruent("(1,2,3)", "((0,0),0,0)")
    assert not oracle.weakly_congruent("(1,2)", "(1,2,3)") and not oracle.weakly_congruent("(5,(0,7))", "((0,0),0)")
    assert oracle.shape_compatible("30", "(2,15)") and oracle.shape_compatible("(2,15)", "(2,(3,5))")
    assert oracle.shape_compatible("30", "(6,5)") and oracle.shape_compatible("(6,5)", "((3,2),5)")
    assert not oracle.shape_compatible("(2,(3,5))", "((3,2),5)") and not oracle.shape_compatible("((3,2),5)", "(2,(3,5))")


def test_worked_evaluation(oracle):
    # Sec. 2.4.1: L(22) = L(2,5) = L((0,1),(1,1)) = 26
    L = oracle.Layout("((2,2),(4,2)):((1,8),(2,16))")
    assert L(22) == 26 and L((2, 5)) == 26 and L(((0, 1), (1, 1))) == 26
    assert L.natural(22) == "((0,1),(1,1))"
    assert (L.rank, L.depth, L.size, L.cosize) == (2, 2, 32, 32)


def test_offset_matrices(oracle):
    # Fig. layouts, Fig. slicing, Fig. blockedproduct, Fig. rakedproduct: L(m,n) for every cell
    n = 0
    for text, cite, mat in _blocks(golden_lines("layout_offset_matrices.txt")):
        L = oracle.Layout(text)
        R, C = mat.shape
        got = L.offsets().reshape(C, R).T          # integral coordinate i = m + R*n (colexicographic)
        assert (got == mat).all(), cite
        for m in range(R):
            for c in range(C):
                assert L((m, c)) == mat[m, c], (cite, m, c)
        n += 1
    assert n == 9


def test_identity_layouts(oracle):
    # Sec. 3.3.1: three layouts I_24 with L(i) = i
    for text in ["24:1", "(4,6):(1,4)", "(3,(4,2)):(1,(3,12))"]:
        assert (oracle.Layout(text).offsets() == np.arange(24)).all()


def test_folding_examples(oracle):
    # Fig. folding (Sec. 1.3): the 4x2 fold coalesces to a flat layout, the 2x4 fold has none
    flat = oracle.Layout("(2,2,2):(2,1,4)")
    a = oracle.Layout("((2,2),2):((2,4),1)")
    b = oracle.Layout("(2,(2,2)):(2,(1,4))")
    assert (b.offsets() == flat.offsets()).all()          # (i,(j,k)) enumerates like (i,j,k)
    for i in range(2):
        for j in range(2):
            for k in range(2):
                assert a(((i, k), j)) == flat((i, j, k)) == 2 * i + j + 4 * k
    assert str(oracle.coalesce_bymode(a)) == "(4,2):(2,1)"
    assert str(oracle.coalesce_bymode(b)) == "(2,(2,2)):(2,(1,4))"


def _run(oracle, op, args):
    if op == "complement":
        return str(oracle.complement(args[0]))
    if op == "complement_under":
        return str(oracle.complement(args[0], int(args[1])))
    if op == "max_common_vector":
        k = oracle.max_common_vector(args[0], args[1])
        assert k == oracle.max_common_vector_def(args[0], args[1])
        return str(k)
    return str(getattr(oracle, op)(*args))


def test_algebra_examples(oracle):
    n = 0
    for ln in golden_lines("algebra_examples.txt"):
        parts = [x.strip() for x in ln.split("|")]
        op, args, expect, cite = parts[0], parts[1:-2], parts[-2], parts[-1]
        if expect.startswith("FAIL:"):
            with pytest.raises(oracle.OracleError) as e:
                _run(oracle, op, args)
            if expect != "FAIL:ANY":
                assert e.value.status_name == expect[5:], ln
        else:
            got = _run(oracle, op, args)
            if op == "complement_under":
                # Sec. 3.5.2 prints these complements without the final extent-1 mode
                got_l = oracle.Layout(got)
                assert str(oracle.coalesce(got_l)) == expect or got == expect, ln
            else:
                assert got == expect, ln
        n += 1
    assert n == 65


def test_associativity_counterexample(oracle):
    # Sec. 3.3.1: both groupings evaluate, to different layouts, because image(2:5) is not inside Z(4:1)
    inner = oracle.composition("4:1", "2:5")
    assert str(oracle.composition("(5,3):(1,7)", inner)) == "2:7"
    left = oracle.composition("(5,3):(1,7)", "4:1")
    assert str(oracle.composition(left, "2:5")) == "2:5"


def test_logical_products_from_complement_and_composition(oracle):
    # Sec. 3.5.1: A (x) B = (A, A* o B) for the two printed products
    for a, b, expect in [("(3,4):(4,1)", "(2,5):(1,2)", "(2,5):(12,24)"), ("(4,8):(20,2)", "(3,2):(2,1)", "(3,2):(80,1)")]:
        assert str(oracle.composition(oracle.complement(a), b)) == expect


def test_slice_operation(oracle):
    # Fig. slicing: offset and remaining layout exactly as printed
    A = "((3,2),((2,3),2)):((4,1),((2,15),100))"
    for ln in golden_lines("slices.txt"):
        crd, off, rest = [x.strip() for x in ln.split("|")]
        got_off, got_rest = oracle.slice_layout(A, crd)
        assert (got_off, str(got_rest)) == (int(off), rest), ln
    assert oracle.slice_layout(A, "(2,5)")[0] == oracle.Layout(A)((2, 5)) and str(oracle.slice_layout(A, "(2,5)")[1]) == "1:0"
    assert str(oracle.slice_layout(A, "_")[1]) == A and str(oracle.slice_layout(A, "(_,_)")[1]) == A
    # tile-then-slice (end of Sec. 3.5.2): one tile of a zipped_divide
    z = oracle.zipped_divide("(8,16):(20,1)", "(4,8):(1,2)")
    off, tile = oracle.slice_layout(z, "(_,(1,1))")
    assert (off, str(tile)) == (81, "(4,8):(20,2)")


def test_slice_property_on_random_layouts(oracle):
    # Sec. 2.5.1: for every coordinate c* of the remaining layout, L(c' + c*) = offset + rest(c*)
    import re
    rng = np.random.default_rng(251)
    checked = 0
    for _ in range(400):
        n = int(rng.integers(1, 5))
        ext = [int(rng.integers(1, 6)) for _ in range(n)]
        strd = [int(rng.integers(0, 40)) for _ in range(n)]
        # random nesting of the n leaves
        def nest(items):
            if len(items) == 1:
                return items[0]
            if len(items) == 2 or rng.random() < 0.5:
                return "(" + ",".join(items) + ")"
            k = int(rng.integers(1, len(items)))
            return "(" + nest(items[:k]) + "," + nest(items[k:]) + ")"
        tags = ["#%d#" % i for i in range(n)]
        skeleton = nest(tags)
        def fill(vals):
            return re.sub(r"#(\d+)#", lambda m: str(vals[int(m.group(1))]), skeleton)
        L = oracle.Layout(fill(ext) + ":" + fill(strd))
        holes = [bool(rng.random() < 0.5) for _ in range(n)]
        fixed = [int(rng.integers(0, e)) for e in ext]
        off, rest = oracle.slice_layout(L, fill(["_" if h else v for h, v in zip(holes, fixed)]))
        hole_ext = [e for e, h in zip(ext, holes) if h]
        assert rest.size == int(np.prod(hole_ext)) if hole_ext else rest.size == 1
        for j in range(rest.size):
            vals, q = list(fixed), j
            for i in range(n):
                if holes[i]:
                    vals[i] = q % ext[i]
                    q //= ext[i]
            full = fill(vals)
            assert L(full if n > 1 or full.startswith("(") else int(full)) == off + rest(j), (str(L), holes, fixed, j)
            checked += 1
    assert checked > 3000


def test_slices(oracle):
    # Fig. slicing: fixing part of a natural coordinate leaves an offset and the sublayout of the free modes
    A = oracle.Layout("((3,2),((2,3),2)):((4,1),((2,15),100))")

    def fill(c, free_vals):
        if c == "_":
            return free_vals.pop(0)
        if isinstance(c, tuple):
            return tuple(fill(x, free_vals) for x in c)
        return c

    def parse(t):
        return eval(t.replace("_", "'_'"))

    def free_shape(c, shape, out):
        if c == "_":
            out.append(shape)
        elif isinstance(c, tuple):
            for x, s in zip(c, shape):
                free_shape(x, s, out)

    shape = ((3, 2), ((2, 3), 2))
    for ln in golden_lines("slices.txt"):
        crd_t, off, rest_t = [x.strip() for x in ln.split("|")]
        crd = parse(crd_t)
        rest = oracle.Layout(rest_t)
        free = []
        free_shape(crd, shape, free)
        def prod(s):
            return s if isinstance(s, int) else int(np.prod([prod(x) for x in s]))
        sizes = [prod(s) for s in free]
        # every choice of the free coordinates: A(c' + c*) = offset + rest(c*)
        for j in range(rest.size):
            vals, q = [], j
            for s in sizes:
                vals.append(q % s)
                q //= s
            assert A(fill(crd, list(vals))) == int(off) + rest(j), (ln, j)
