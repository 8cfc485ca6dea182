"""The paper's intermediate objects, written out in its own notation.

TEST INFRASTRUCTURE ONLY.  Plain numpy / Python loops, meant for small inputs.
Each function follows one definition, equation or algorithm of the paper; the
tests pin them to the examples the paper prints and to the identities it proves,
and then use them to check the index tables exported by the HIP library.

Indexing: the paper counts rows, sorted positions and list entries from 1.  The
functions here count from 0 and the docstrings say how to convert; "value j"
always means the integer j in [0, 2^k) and is the same in both conventions.

Readings taken where the paper is loose (each is checked by a test):

* Row value (Definition 3.2): the first column of a block is the most
  significant bit, as in the printed example [1,0,1,1] -> 1011_2.
* Order inside a group of equal rows: Definition 3.2 only constrains rows with
  different values; this module keeps equal rows in ascending row order (a stable
  sort), which reproduces the permutation printed in Example 3.3.
* Full segmentation (Section 3.3): L[j] is the number of rows whose value is
  below j.  For a value that occurs this is its first sorted position; for one
  that does not it is the start of the next value that does (Section 3.3 gives
  an absent value the boundary of its successor), and past the last occurring
  value it is the row count, which makes the length rule of Proposition 3.5
  hold for every j.
* RSR++ fold (Algorithm 3, Section 4.3): the printed listing indexes the pair
  sums with the outer loop variable and never copies them back; the text of
  Section 4.3 says what is meant.  "Odd indices" are odd when the 2^i entries are
  counted from 0, i.e. the entries whose value has its lowest bit set: counted
  from 1 as the paper does elsewhere, the first entry belongs to value 0, so the
  entries with lowest bit 1 are the even-numbered ones.  The reading is fixed by
  the requirement that the fold equals u . Bin_[k].
* A last block narrower than k (Definition 3.1, min(i*k, n)) has k' < k columns
  and 2^k' values.
"""
from __future__ import annotations

from typing import List, Sequence, Tuple

import numpy as np


# --------------------------------------------------------------------------- #
# Section 2.3, Proposition 2.1
# --------------------------------------------------------------------------- #
def ternary_split(A: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """A = B1 - B2 with B1 = [A == 1] and B2 = [A == -1] (Proposition 2.1)."""
    A = np.asarray(A)
    if not np.isin(A, (-1, 0, 1)).all():
        raise ValueError("entries must be in {-1,0,1}")
    return (A == 1).astype(np.int8), (A == -1).astype(np.int8)


# --------------------------------------------------------------------------- #
# Section 3.1, Definition 3.1
# --------------------------------------------------------------------------- #
def column_blocks(B: np.ndarray, k: int) -> List[np.ndarray]:
    """The k-column blocks of B: block i (from 0) holds columns i*k .. min((i+1)*k, cols)-1."""
    B = np.asarray(B)
    if k < 1:
        raise ValueError("k must be >= 1")
    cols = B.shape[1]
    nblocks = -(-cols // k)
    return [B[:, i * k : min((i + 1) * k, cols)] for i in range(nblocks)]


# --------------------------------------------------------------------------- #
# Section 3.2, Definition 3.2
# --------------------------------------------------------------------------- #
def row_values(Bi: np.ndarray) -> np.ndarray:
    """Binary value of every row of a block: columns concatenated, first column most significant."""
    Bi = np.asarray(Bi)
    if not np.isin(Bi, (0, 1)).all():
        raise ValueError("block must be binary")
    width = Bi.shape[1]
    vals = np.zeros(Bi.shape[0], dtype=np.int64)
    for c in range(width):
        vals = vals * 2 + Bi[:, c].astype(np.int64)
    return vals


def binary_row_order(Bi: np.ndarray) -> np.ndarray:
    """sigma for a block, counted from 0: sigma[p] is the row placed at sorted position p.

    Rows are sorted by ascending value; equal rows keep ascending row order.
    (The paper's sigma counts from 1: add 1 to every entry.)
    """
    return np.argsort(row_values(Bi), kind="stable").astype(np.int64)


def bin_matrix(k: int) -> np.ndarray:
    """Bin_[k]: the 2^k x k matrix whose row j is the k-bit binary form of j, first column most significant."""
    if k < 0:
        raise ValueError("k must be >= 0")
    M = np.zeros((1 << k, k), dtype=np.int64)
    for j in range(1 << k):
        for c in range(k):
            M[j, c] = (j >> (k - 1 - c)) & 1
    return M


# --------------------------------------------------------------------------- #
# Section 3.3, Definition 3.4 and the "Full Segmentation"
# --------------------------------------------------------------------------- #
def segmentation_list(Bi: np.ndarray) -> np.ndarray:
    """Start positions (from 0) of the groups of equal rows in the sorted block, occurring values only."""
    vals = np.sort(row_values(Bi), kind="stable")
    starts = [p for p in range(len(vals)) if p == 0 or vals[p] != vals[p - 1]]
    return np.asarray(starts, dtype=np.int64)


def full_segmentation(Bi: np.ndarray) -> np.ndarray:
    """L for a block: exactly 2^width entries, L[j] = number of rows with value < j (positions from 0).

    (The paper's list counts positions from 1: add 1 to every entry.)
    """
    Bi = np.asarray(Bi)
    width = Bi.shape[1]
    vals = row_values(Bi)
    L = np.zeros(1 << width, dtype=np.int64)
    for j in range(1 << width):
        L[j] = int(np.count_nonzero(vals < j))
    return L


# --------------------------------------------------------------------------- #
# Section 3.4, Algorithm 1
# --------------------------------------------------------------------------- #
def preprocess(B: np.ndarray, k: int) -> Tuple[List[np.ndarray], List[np.ndarray]]:
    """Algorithm 1: for every k-column block, its row permutation and its full segmentation."""
    sigmas, Ls = [], []
    for Bi in column_blocks(B, k):
        sigmas.append(binary_row_order(Bi))
        Ls.append(full_segmentation(Bi))
    return sigmas, Ls


# --------------------------------------------------------------------------- #
# Section 4.1, Definition 4.1 (Eq. SS1) and Eq. SS2
# --------------------------------------------------------------------------- #
def segmented_sum_permuted(v_pi: Sequence, L: Sequence[int]) -> np.ndarray:
    """Eq. SS1: sums of the already permuted vector over [L[j], L[j+1]); the last group runs to the end."""
    v_pi = np.asarray(v_pi)
    n = len(v_pi)
    m = len(L)
    u = np.zeros(m, dtype=np.result_type(v_pi.dtype, np.int64) if v_pi.dtype.kind in "iu" else np.float64)
    for j in range(m):
        hi = L[j + 1] if j + 1 < m else n
        for p in range(L[j], hi):
            u[j] += v_pi[p]
    return u


def segmented_sum(v: Sequence, sigma: Sequence[int], L: Sequence[int]) -> np.ndarray:
    """Eq. SS2: the same sums taken in place, u[j] = sum_{p in [L[j], L[j+1])} v[sigma[p]]."""
    v = np.asarray(v)
    n = len(v)
    m = len(L)
    u = np.zeros(m, dtype=np.result_type(v.dtype, np.int64) if v.dtype.kind in "iu" else np.float64)
    for j in range(m):
        hi = L[j + 1] if j + 1 < m else n
        for p in range(L[j], hi):
            u[j] += v[sigma[p]]
    return u


# --------------------------------------------------------------------------- #
# Section 4.2, Algorithm 2 (step 2) and Section 4.3, Algorithm 3
# --------------------------------------------------------------------------- #
def block_product_rsr(u: Sequence, k: int) -> np.ndarray:
    """Algorithm 2, step 2: the plain product u . Bin_[k] (k outputs, O(k 2^k))."""
    u = np.asarray(u)
    if len(u) != 1 << k:
        raise ValueError("u must have 2^k entries")
    return u @ bin_matrix(k).astype(u.dtype if u.dtype.kind == "f" else np.int64)


def fold_rsrpp(u: Sequence, k: int) -> np.ndarray:
    """Algorithm 3: u . Bin_[k] in O(2^k) by repeated halving.

    x <- u.  For i = k down to 1: r_i <- sum of the entries of x whose index, counted from 0,
    is odd; then x <- the sums of consecutive pairs of x (half as long).  r_1 .. r_k are the
    outputs for the block's columns 1 .. k.
    """
    x = np.asarray(u)
    if len(x) != 1 << k:
        raise ValueError("u must have 2^k entries")
    x = x.astype(np.float64 if x.dtype.kind == "f" else np.int64)
    r = np.zeros(k, dtype=x.dtype)
    for i in range(k, 0, -1):
        acc = x.dtype.type(0)
        for j in range(1, len(x), 2):
            acc += x[j]
        r[i - 1] = acc
        nxt = np.zeros(len(x) // 2, dtype=x.dtype)
        for j in range(len(nxt)):
            nxt[j] = x[2 * j] + x[2 * j + 1]
        x = nxt
    return r


# --------------------------------------------------------------------------- #
# Algorithm 2 as a whole, and the ternary case through Proposition 2.1
# --------------------------------------------------------------------------- #
def rsr_binary(v: Sequence, B: np.ndarray, k: int, step2: str = "fold") -> np.ndarray:
    """v . B for binary B by Algorithm 2, with step 2 either the plain product or the RSR++ fold."""
    v = np.asarray(v)
    sigmas, Ls = preprocess(B, k)  # Algorithm 1, once per matrix
    pieces = []
    for sigma, L in zip(sigmas, Ls):
        width = len(L).bit_length() - 1  # L has 2^width entries
        u = segmented_sum(v, sigma, L)
        pieces.append(fold_rsrpp(u, width) if step2 == "fold" else block_product_rsr(u, width))
    return np.concatenate(pieces)


def rsr_ternary(v: Sequence, A: np.ndarray, k: int, step2: str = "fold") -> np.ndarray:
    """v . A for ternary A: v . B1 - v . B2 (Proposition 2.1), each by Algorithm 2."""
    B1, B2 = ternary_split(A)
    return rsr_binary(v, B1, k, step2) - rsr_binary(v, B2, k, step2)
