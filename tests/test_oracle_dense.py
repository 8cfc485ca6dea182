"""Pins for the dense CPU oracle (oracle/rsr_oracle.c): the product by its definition.

Every expected value here comes from the paper's printed example, from a closed
form, from an invariant of the product, from numpy's own integer / float64
matrix product (a library routine used as a second opinion), or from a
set-membership brute force on tiny matrices - never from the oracle itself and
never from the HIP path.
"""
import itertools

import numpy as np
import pytest

from oracle import dense


def rng(seed):
    return np.random.default_rng(seed)


# ---- the paper's worked example -------------------------------------------------
def test_paper_matrix_times_printed_vector(golden):
    B = np.array(golden["matrix_B"]["rows"], dtype=np.int8)
    d = golden["derived_product"]
    v = np.array(d["v"])
    want = np.array(d["v_dot_B"])
    assert np.array_equal(dense.matvec_i8(B, v.astype(np.int8)), want)
    assert np.array_equal(dense.matvec_f32(B, v.astype(np.float32)), want.astype(np.float64))


def test_orientation_vector_multiplies_from_the_left():
    # rows != cols: a transposed operand or swapped shape cannot pass this
    A = np.array([[1, 0, -1], [0, 1, 1]], dtype=np.int8)  # 2 x 3
    v = np.array([2, 7], dtype=np.int8)
    assert np.array_equal(dense.matvec_i8(A, v), [2, 7, 5])
    assert np.array_equal(dense.matvec_f32(A, v.astype(np.float32)), [2.0, 7.0, 5.0])
    with pytest.raises(ValueError):
        dense.matvec_i8(A, np.array([1, 2, 3], dtype=np.int8))


# ---- closed forms ----------------------------------------------------------------
@pytest.mark.parametrize("rows,cols", [(1, 1), (5, 3), (64, 17), (300, 129)])
def test_all_ones_gives_sum_of_v_everywhere(rows, cols):
    v8 = rng(rows * 31 + cols).integers(-127, 128, size=rows, dtype=np.int8)
    out = dense.matvec_i8(np.ones((rows, cols), np.int8), v8)
    assert np.array_equal(out, np.full(cols, int(v8.astype(np.int64).sum())))
    vf = rng(rows + cols).standard_normal(rows).astype(np.float32)
    outf = dense.matvec_f32(np.ones((rows, cols), np.int8), vf)
    exact = float(np.sum(vf.astype(np.float64)))
    assert np.allclose(outf, exact, rtol=0, atol=1e-12 * np.abs(vf).sum())


def test_all_zeros_identity_and_single_entry():
    n = 37
    v = rng(1).integers(-127, 128, size=n, dtype=np.int8)
    assert np.array_equal(dense.matvec_i8(np.zeros((n, 11), np.int8), v), np.zeros(11, np.int64))
    assert np.array_equal(dense.matvec_i8(np.eye(n, dtype=np.int8), v), v.astype(np.int64))
    assert np.array_equal(dense.matvec_i8(-np.eye(n, dtype=np.int8), v), -v.astype(np.int64))
    for r, c, s in [(0, 0, 1), (36, 10, -1), (5, 3, 1)]:
        A = np.zeros((n, 11), np.int8)
        A[r, c] = s
        want = np.zeros(11, np.int64)
        want[c] = s * int(v[r])
        assert np.array_equal(dense.matvec_i8(A, v), want)
        assert np.array_equal(dense.matvec_f32(A, v.astype(np.float32)), want.astype(np.float64))


def test_int8_extremes_do_not_wrap():
    n = 4096
    v = np.full(n, -128, dtype=np.int8)
    A = -np.ones((n, 2), np.int8)
    assert np.array_equal(dense.matvec_i8(A, v), [128 * n, 128 * n])
    v = np.full(n, 127, dtype=np.int8)
    assert np.array_equal(dense.matvec_i8(A, v), [-127 * n, -127 * n])


# ---- invariants ------------------------------------------------------------------
def test_linearity_of_the_ternary_split_and_negation():
    g = rng(7)
    A = g.integers(-1, 2, size=(150, 70)).astype(np.int8)
    Bp, Bm = (A == 1).astype(np.int8), (A == -1).astype(np.int8)
    v8 = g.integers(-127, 128, size=(3, 150), dtype=np.int8)
    assert np.array_equal(dense.matvec_i8(A, v8), dense.matvec_i8(Bp, v8) - dense.matvec_i8(Bm, v8))
    assert np.array_equal(dense.matvec_i8(-A, v8), -dense.matvec_i8(A, v8))
    vf = g.standard_normal((2, 150)).astype(np.float32)
    tol = 1e-12 * np.abs(vf).sum(axis=1, keepdims=True)
    assert np.all(np.abs(dense.matvec_f32(A, vf) - (dense.matvec_f32(Bp, vf) - dense.matvec_f32(Bm, vf))) <= tol)
    assert np.array_equal(dense.matvec_f32(-A, vf), -dense.matvec_f32(A, vf))


def test_row_permutation_invariance_and_column_locality():
    g = rng(11)
    A = g.integers(-1, 2, size=(90, 40)).astype(np.int8)
    v = g.integers(-127, 128, size=90, dtype=np.int8)
    perm = g.permutation(90)
    assert np.array_equal(dense.matvec_i8(A[perm], v[perm]), dense.matvec_i8(A, v))
    # out[c] depends on column c alone: shuffle the columns, the outputs shuffle alike
    cperm = g.permutation(40)
    assert np.array_equal(dense.matvec_i8(A[:, cperm], v), dense.matvec_i8(A, v)[cperm])
    # and changing one column changes one output
    A2 = A.copy()
    A2[:, 13] = -A2[:, 13]
    d = dense.matvec_i8(A2, v) - dense.matvec_i8(A, v)
    assert np.count_nonzero(np.delete(d, 13)) == 0


def test_homogeneity_in_v_for_integers():
    g = rng(13)
    A = g.integers(-1, 2, size=(60, 25)).astype(np.int8)
    v = g.integers(-40, 41, size=60, dtype=np.int8)
    assert np.array_equal(dense.matvec_i8(A, (3 * v).astype(np.int8)), 3 * dense.matvec_i8(A, v))


def test_batch_equals_stacked_single_calls():
    g = rng(17)
    A = g.integers(-1, 2, size=(77, 33)).astype(np.int8)
    v8 = g.integers(-127, 128, size=(5, 77), dtype=np.int8)
    vf = g.standard_normal((5, 77)).astype(np.float32)
    assert np.array_equal(dense.matvec_i8(A, v8), np.stack([dense.matvec_i8(A, v8[b]) for b in range(5)]))
    assert np.array_equal(dense.matvec_f32(A, vf), np.stack([dense.matvec_f32(A, vf[b]) for b in range(5)]))


# ---- library routine as a second opinion -------------------------------------------
@pytest.mark.parametrize("rows,cols,kind", [(257, 130, "binary"), (1000, 513, "ternary"), (64, 64, "ternary")])
def test_against_numpy_products(rows, cols, kind):
    g = rng(rows + 3 * cols)
    A = (g.integers(0, 2, size=(rows, cols)) if kind == "binary" else g.integers(-1, 2, size=(rows, cols))).astype(np.int8)
    v8 = g.integers(-127, 128, size=(2, rows), dtype=np.int8)
    assert np.array_equal(dense.matvec_i8(A, v8), v8.astype(np.int64) @ A.astype(np.int64))
    vf = g.standard_normal((2, rows)).astype(np.float32)
    ref = vf.astype(np.float64) @ A.astype(np.float64)
    tol = 1e-12 * np.abs(vf).sum(axis=1, keepdims=True)
    assert np.all(np.abs(dense.matvec_f32(A, vf) - ref) <= tol)


# ---- brute force on tiny inputs ------------------------------------------------------
def _by_membership(A, v):
    """Sum of v over the rows where the column holds +1, minus the sum where it holds -1."""
    rows, cols = len(A), len(A[0])
    out = []
    for c in range(cols):
        plus = {r for r in range(rows) if A[r][c] == 1}
        minus = {r for r in range(rows) if A[r][c] == -1}
        out.append(sum(int(v[r]) for r in plus) - sum(int(v[r]) for r in minus))
    return out


def test_every_binary_matrix_up_to_3x3():
    v_full = np.array([3, -5, 11], dtype=np.int8)
    for rows in (1, 2, 3):
        for cols in (1, 2, 3):
            v = v_full[:rows]
            for bits in itertools.product((0, 1), repeat=rows * cols):
                A = np.array(bits, dtype=np.int8).reshape(rows, cols)
                want = _by_membership(A.tolist(), v)
                assert dense.matvec_i8(A, v).tolist() == want
                assert dense.matvec_f32(A, v.astype(np.float32)).tolist() == [float(x) for x in want]


def test_sample_of_tiny_ternary_matrices():
    g = rng(23)
    for _ in range(300):
        rows, cols = int(g.integers(1, 5)), int(g.integers(1, 5))
        A = g.integers(-1, 2, size=(rows, cols)).astype(np.int8)
        v = g.integers(-127, 128, size=rows, dtype=np.int8)
        assert dense.matvec_i8(A, v).tolist() == _by_membership(A.tolist(), v)


# ---- harness variants compute the same thing -------------------------------------------
def test_striped_and_threaded_variants_match_single_pass():
    g = rng(29)
    A = g.integers(-1, 2, size=(200, 101)).astype(np.int8)
    v8 = g.integers(-127, 128, size=(2, 200), dtype=np.int8)
    vf = g.standard_normal((2, 200)).astype(np.float32)
    full8, fullf = dense.matvec_i8(A, v8), dense.matvec_f32(A, vf)
    for t in (2, 3, 8, 500):
        assert np.array_equal(dense.matvec_i8(A, v8, threads=t), full8)
        assert np.array_equal(dense.matvec_f32(A, vf, threads=t), fullf)
    part = dense.matvec_f32(A, vf, cols=(40, 60))
    assert np.array_equal(part[:, 40:60], fullf[:, 40:60]) and np.isnan(part[:, :40]).all() and np.isnan(part[:, 60:]).all()
    part8 = dense.matvec_i8(A, v8, cols=(0, 7))
    assert np.array_equal(part8[:, :7], full8[:, :7])


def test_rejects_entries_outside_the_ternary_set():
    A = np.zeros((4, 4), np.int8)
    A[2, 1] = 2
    with pytest.raises(ValueError):
        dense.matvec_i8(A, np.ones(4, np.int8))


# ---- entries with q bits (appendix "Generalization") -------------------------------------
@pytest.mark.parametrize("q", [2, 3, 4, 8])
def test_qbit_entries_against_numpy_and_against_the_weighted_bit_planes(q):
    g = rng(600 + q)
    lo, hi = -(1 << (q - 1)), (1 << (q - 1)) - 1
    A = g.integers(lo, hi + 1, size=(300, 77)).astype(np.int8)
    A[0, 0], A[1, 0] = lo, hi
    v8 = g.integers(-127, 128, size=(2, 300), dtype=np.int8)
    v8[0, :2] = (-128, 127)
    got = dense.matvec_i8(A, v8, qbits=q)
    assert np.array_equal(got, v8.astype(np.int64) @ A.astype(np.int64))   # library routine, second opinion
    # the decomposition the appendix describes, written out with two's complement bit planes:
    # A = sum_{i<q-1} 2^i B_i - 2^(q-1) B_{q-1}, every B_i binary and multiplied on its own
    planes = [((A.astype(np.uint8) >> i) & 1).astype(np.int8) for i in range(q)]
    assert np.array_equal(sum((-(1 << i) if i == q - 1 else (1 << i)) * P.astype(np.int64) for i, P in enumerate(planes)), A)
    combined = sum((-(1 << i) if i == q - 1 else (1 << i)) * dense.matvec_i8(P, v8) for i, P in enumerate(planes))
    assert np.array_equal(got, combined)
    vf = g.standard_normal((2, 300)).astype(np.float32)
    ref = vf.astype(np.float64) @ A.astype(np.float64)
    assert np.all(np.abs(dense.matvec_f32(A, vf, qbits=q) - ref) <= 1e-12 * (1 << q) * np.abs(vf).sum(axis=1, keepdims=True))


def test_qbit_rejects_entries_outside_the_range():
    A = np.zeros((4, 4), np.int8)
    A[3, 3] = 2
    with pytest.raises(ValueError):
        dense.matvec_i8(A, np.ones(4, np.int8), qbits=2)
    assert dense.matvec_i8(A, np.ones(4, np.int8), qbits=3)[3] == 2
