"""Pins for oracle/steps.py: the paper's intermediate objects against what the paper prints and proves.

Printed values come from tests/golden/paper_examples.json (each entry cites its passage).
Identities: Proposition 3.5 (segment lengths are the value histogram), Lemma 4.2
(v.B_i = SS(v).Bin_[k]), and "the RSR++ fold equals the plain product u.Bin_[k]".
The whole of Algorithm 2 is then pinned to the dense oracle, which has pins of its own.
"""
import numpy as np
import pytest

from oracle import dense, steps


def rng(seed):
    return np.random.default_rng(seed)


# ---- printed examples -------------------------------------------------------------------
def test_row_value_first_column_is_most_significant(golden):
    ex = golden["row_value_example"]
    assert steps.row_values(np.array([ex["row"]]))[0] == ex["value"]


def test_printed_column_blocks(golden):
    B = np.array(golden["matrix_B"]["rows"])
    blocks = steps.column_blocks(B, golden["blocks_of_B"]["k"])
    assert len(blocks) == 3
    assert np.array_equal(blocks[0], golden["blocks_of_B"]["B1"])
    assert np.array_equal(blocks[2], golden["blocks_of_B"]["B3"])
    # Definition 3.1 for the middle block (the printed B_2 disagrees with the printed B)
    assert np.array_equal(blocks[1], B[:, 2:4])


def test_ragged_last_block_is_narrower():
    B = np.arange(5 * 7).reshape(5, 7) % 2
    blocks = steps.column_blocks(B, 3)
    assert [b.shape[1] for b in blocks] == [3, 3, 1]
    assert np.array_equal(np.concatenate(blocks, axis=1), B)


def test_example_3_3_permutation_and_segmentation(golden):
    ex = golden["example_3_3"]
    Bi = np.array(ex["block"])
    sigma = steps.binary_row_order(Bi)
    assert (sigma + 1).tolist() == ex["sigma_1based"]
    assert np.array_equal(Bi[sigma], ex["sorted_block"])
    assert (steps.segmentation_list(Bi) + 1).tolist() == ex["segmentation_1based"]
    assert (steps.full_segmentation(Bi) + 1).tolist() == ex["full_segmentation_1based"]


def test_printed_bin_matrices(golden):
    for k in (1, 2, 3):
        assert np.array_equal(steps.bin_matrix(k), golden["bin_matrices"][str(k)])


def test_bin_matrix_is_binary_row_ordered_with_one_row_per_value():
    for k in range(1, 9):
        M = steps.bin_matrix(k)
        assert M.shape == (1 << k, k)
        assert steps.row_values(M).tolist() == list(range(1 << k))


def test_printed_segmented_sum(golden):
    ex = golden["segmented_sum_example"]
    L = np.array(ex["full_segmentation_1based"]) - 1
    assert steps.segmented_sum_permuted(ex["v_pi"], L).tolist() == ex["SS"]
    # Eq. SS2 reaches the same sums from the vector whose permutation is the printed one
    d = golden["derived_product"]
    sigma = np.array(golden["example_3_3"]["sigma_1based"]) - 1
    v = np.array(d["unpermuted_v"])
    assert v[sigma].tolist() == ex["v_pi"]
    assert steps.segmented_sum(v, sigma, L).tolist() == ex["SS"]
    # and with the printed vector taken as v itself, the hand-worked sums of block 1
    assert steps.segmented_sum(np.array(d["v"]), sigma, L).tolist() == d["block1_u_under_SS2"]
    assert steps.fold_rsrpp(np.array(d["block1_u_under_SS2"]), 2).tolist() == d["v_dot_B"][:2]


def test_whole_method_on_the_printed_matrix(golden):
    B = np.array(golden["matrix_B"]["rows"])
    d = golden["derived_product"]
    for k in (1, 2, 3, 4, 5, 6):
        for step2 in ("fold", "product"):
            assert steps.rsr_binary(np.array(d["v"]), B, k, step2).tolist() == d["v_dot_B"]


# ---- Proposition 2.1 ------------------------------------------------------------------------
def test_ternary_split():
    A = rng(3).integers(-1, 2, size=(20, 9))
    B1, B2 = steps.ternary_split(A)
    assert set(np.unique(B1)) <= {0, 1} and set(np.unique(B2)) <= {0, 1}
    assert np.array_equal(B1 - B2, A)
    assert not np.any(B1 & B2)
    with pytest.raises(ValueError):
        steps.ternary_split(np.array([[2]]))


# ---- Definition 3.2 / 3.4, Proposition 3.5 -----------------------------------------------------
@pytest.mark.parametrize("rows,width,seed", [(1, 1, 0), (50, 3, 1), (200, 5, 2), (64, 8, 3), (9, 4, 4)])
def test_order_and_segmentation_invariants(rows, width, seed):
    Bi = rng(seed).integers(0, 2, size=(rows, width))
    vals = steps.row_values(Bi)
    sigma = steps.binary_row_order(Bi)
    L = steps.full_segmentation(Bi)
    assert sorted(sigma.tolist()) == list(range(rows))  # a permutation
    sv = vals[sigma]
    assert np.all(np.diff(sv) >= 0)  # ascending values
    for p in range(rows - 1):  # equal rows keep ascending row order
        if sv[p] == sv[p + 1]:
            assert sigma[p] < sigma[p + 1]
    assert len(L) == 1 << width and L[0] == 0 and np.all(np.diff(L) >= 0)
    # Proposition 3.5: consecutive differences are the number of rows of each value
    hist = np.bincount(vals, minlength=1 << width)
    lengths = np.diff(np.append(L, rows))
    assert np.array_equal(lengths, hist)
    for j in range(1 << width):  # every row of group j has value j
        hi = L[j + 1] if j + 1 < len(L) else rows
        assert np.all(sv[L[j] : hi] == j)


# ---- Lemma 4.2 ------------------------------------------------------------------------------------
@pytest.mark.parametrize("rows,width,seed", [(6, 2, 0), (40, 3, 1), (300, 6, 2), (17, 5, 3)])
def test_lemma_4_2_block_identity(rows, width, seed):
    g = rng(100 + seed)
    Bi = g.integers(0, 2, size=(rows, width))
    v = g.integers(-127, 128, size=rows)
    u = steps.segmented_sum(v, steps.binary_row_order(Bi), steps.full_segmentation(Bi))
    assert np.array_equal(u @ steps.bin_matrix(width), v @ Bi)


# ---- Algorithm 3 (RSR++ fold) ------------------------------------------------------------------------
@pytest.mark.parametrize("k", list(range(1, 14)))
def test_fold_equals_plain_product(k):
    g = rng(200 + k)
    u = g.integers(-(10**6), 10**6, size=1 << k)
    assert np.array_equal(steps.fold_rsrpp(u, k), u @ steps.bin_matrix(k))
    assert np.array_equal(steps.block_product_rsr(u, k), u @ steps.bin_matrix(k))
    uf = g.standard_normal(1 << k)
    assert np.allclose(steps.fold_rsrpp(uf, k), uf @ steps.bin_matrix(k), rtol=0, atol=1e-9 * np.abs(uf).sum())


def test_fold_of_a_unit_vector_reads_off_the_bits():
    k = 5
    for j in range(1 << k):
        u = np.zeros(1 << k, dtype=np.int64)
        u[j] = 1
        bits = [(j >> (k - 1 - c)) & 1 for c in range(k)]
        assert steps.fold_rsrpp(u, k).tolist() == bits


def test_the_other_reading_of_odd_indices_is_wrong():
    # counting the entries from 1 and taking the odd ones would sum the values with lowest bit 0
    u = np.array([7, 0, 0, 0])  # all weight on value 00: the product with Bin_[2] is [0, 0]
    assert steps.fold_rsrpp(u, 2).tolist() == [0, 0]
    one_based_odd_first_level = u[0::2].sum()
    assert one_based_odd_first_level == 7  # not 0: that reading contradicts u . Bin_[2]


# ---- Algorithm 2 as a whole against the dense oracle ------------------------------------------------------
@pytest.mark.parametrize(
    "rows,cols,k,kind,seed",
    [(30, 30, 3, "binary", 0), (64, 50, 4, "ternary", 1), (100, 23, 5, "ternary", 2), (17, 40, 7, "binary", 3), (256, 8, 8, "ternary", 4)],
)
def test_method_equals_definition(rows, cols, k, kind, seed):
    g = rng(300 + seed)
    A = (g.integers(0, 2, size=(rows, cols)) if kind == "binary" else g.integers(-1, 2, size=(rows, cols))).astype(np.int8)
    v = g.integers(-127, 128, size=rows, dtype=np.int8)
    want = dense.matvec_i8(A, v)
    for step2 in ("fold", "product"):
        got = steps.rsr_ternary(v.astype(np.int64), A, k, step2)
        assert np.array_equal(got, want)
    vf = g.standard_normal(rows).astype(np.float32)
    gotf = steps.rsr_ternary(vf.astype(np.float64), A, k)
    assert np.all(np.abs(gotf - dense.matvec_f32(A, vf)) <= 1e-12 * np.abs(vf).sum())


def test_matrix_equal_to_bin_k_isolates_the_fold():
    # A = Bin_[k]: sigma is the identity, every group has one row, u = v, so v.A is the fold of v
    k = 6
    A = steps.bin_matrix(k).astype(np.int8)
    v = rng(5).integers(-127, 128, size=1 << k, dtype=np.int8)
    assert steps.binary_row_order(A).tolist() == list(range(1 << k))
    assert steps.full_segmentation(A).tolist() == list(range(1 << k))
    assert np.array_equal(steps.fold_rsrpp(v.astype(np.int64), k), dense.matvec_i8(A, v))


# ---- Algorithm 1 as a whole ----------------------------------------------------------------
def test_preprocess_reproduces_the_tables_of_the_printed_matrix(golden):
    """Algorithm 1 on the printed 6x6 B with k = 2: block 1 is Example 3.3 as printed; blocks 2 and 3
    are worked by hand from the printed B (the fixture says how)."""
    B = np.array(golden["matrix_B"]["rows"])
    d = golden["derived_tables_of_B"]
    sigmas, Ls = steps.preprocess(B, d["k"])
    assert len(sigmas) == len(Ls) == 3
    assert [(s + 1).tolist() for s in sigmas] == d["sigma_1based"]
    assert [(L + 1).tolist() for L in Ls] == d["full_segmentation_1based"]
    assert (sigmas[0] + 1).tolist() == golden["example_3_3"]["sigma_1based"]
    assert (Ls[0] + 1).tolist() == golden["example_3_3"]["full_segmentation_1based"]


@pytest.mark.parametrize("rows,cols,k", [(1, 1, 1), (9, 7, 3), (40, 10, 4), (33, 17, 5), (64, 6, 6)])
def test_preprocess_invariants(rows, cols, k):
    """What Algorithm 1 must deliver whatever the matrix: one (sigma, L) per k-column block (the last
    block narrower, Definition 3.1); sigma a permutation along which the row values never decrease and
    equal rows keep their order (Definition 3.2); L with 2^width entries whose differences are the
    histogram of the row values (Proposition 3.5), computed here by counting, not by sorting."""
    B = rng(rows * 100 + cols).integers(0, 2, size=(rows, cols))
    sigmas, Ls = steps.preprocess(B, k)
    nblocks = -(-cols // k)
    assert len(sigmas) == len(Ls) == nblocks
    for i in range(nblocks):
        width = min(k, cols - i * k)
        vals = [int("".join(str(int(x)) for x in B[r, i * k : i * k + width]), 2) for r in range(rows)]
        sigma, L = sigmas[i], Ls[i]
        assert sorted(sigma.tolist()) == list(range(rows))
        along = [vals[r] for r in sigma]
        assert all(a <= b for a, b in zip(along, along[1:]))
        assert all(r0 < r1 for r0, r1, a, b in zip(sigma, sigma[1:], along, along[1:]) if a == b)
        assert len(L) == 1 << width
        ends = L.tolist()[1:] + [rows]
        assert [e - s for s, e in zip(L.tolist(), ends)] == [vals.count(j) for j in range(1 << width)]
