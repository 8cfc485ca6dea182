"""Host logic of the HIP library, without a GPU: the C ABI loads and exports what include/rsr.h
declares; the index builder (Algorithm 1 + packing) reproduces the paper's tables; the packed
streams satisfy the layout the kernels assume; and a numpy walk over the packed streams that
mirrors the kernel's traversal reproduces the dense oracle's product.

No product is computed by the library here (that needs the GPU); the numpy walk is test code.
"""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2411_06360_amd as R
from oracle import dense, steps

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

# layout constants of csrc/rsr_format.h
WINDOW, DUMMY, OVF_BASE, MAX_OVF, WIN_SLOTS, TILE, MAX_DIAG = 512, 8, 520, 64, 584, 512, 40


def rng(seed):
    return np.random.default_rng(seed)


class HostIndex:
    def __init__(self, A, k):
        self.x = R.rsr_host_pack(A, k)
        self.info = R.rsr_host_info(self.x)

    def __enter__(self):
        return self

    def __exit__(self, *a):
        R.rsr_host_free(self.x)


# ---- the boundary ------------------------------------------------------------------------------
def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "rsr.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(rsr_[a-z0-9_]+)\s*\(", header))
    assert {"rsr_preprocess", "rsr_matvec", "rsr_matvec_i8", "rsr_destroy", "rsr_last_error", "rsr_info",
            "rsr_export_block", "rsr_host_pack"} <= names
    lib = R.load()
    for n in sorted(names):
        assert hasattr(lib, n), f"{n} declared in rsr.h but not exported"


def test_info_struct_matches_the_header():
    header = open(os.path.join(ROOT, "include", "rsr.h")).read()
    body = re.search(r"typedef struct rsr_info_t \{(.*?)\} rsr_info_t;", header, re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = []
    for decl in body.split(";"):
        decl = decl.strip()
        if not decl:
            continue
        ctype, names = decl.split(None, 1)
        fields += [(n.strip(), ctype) for n in names.split(",")]
    got = [(n, "int64_t" if t is ctypes.c_int64 else "int32_t") for n, t in R.RsrInfo._fields_]
    assert got == fields


def test_argument_errors_are_reported_not_raised_as_crashes():
    good = np.zeros((4, 4), np.int8)
    for A, k in [(good, 0), (good, 17), (np.zeros((0, 4), np.int8), 2), (np.zeros((4, 0), np.int8), 2)]:
        with pytest.raises(R.RsrError):
            R.rsr_host_pack(A, k)
    bad = good.copy()
    bad[2, 3] = 2
    with pytest.raises(R.RsrError) as e:
        R.rsr_host_pack(bad, 2)
    assert "row 2" in str(e.value) and "column 3" in str(e.value)
    with pytest.raises(R.RsrError):
        R.rsr_host_pack(np.zeros((65535, 1), np.int8), 1)
    lib = R.load()
    assert not lib.rsr_host_pack(None, 4, 4, 2) and "null" in R.rsr_last_error()
    assert not lib.rsr_preprocess(None, 4, 4, 2)
    assert lib.rsr_matvec(None, None, None, 1, None) < 0 and "handle" in R.rsr_last_error()
    assert lib.rsr_matvec_i8(None, None, None, 1, None) < 0
    assert lib.rsr_info(None, None) < 0
    lib.rsr_destroy(None)
    lib.rsr_host_free(None)
    with HostIndex(good, 2) as h:
        with pytest.raises(R.RsrError):
            R.rsr_host_export_block(h.x, 1, 0)  # a binary matrix has one part
        assert lib.rsr_host_export_block(h.x, 0, 99, None, None) < 0


# ---- the paper's tables ---------------------------------------------------------------------------
def test_paper_example_tables(golden):
    B = np.array(golden["matrix_B"]["rows"], dtype=np.int8)
    with HostIndex(B, 2) as h:
        assert (h.info.rows, h.info.cols, h.info.k, h.info.parts, h.info.nblocks) == (6, 6, 2, 1, 3)
        sigma, L = R.rsr_host_export_block(h.x, 0, 0)
        ex = golden["example_3_3"]
        assert (sigma + 1).tolist() == ex["sigma_1based"]
        assert (L[:-1] + 1).tolist() == ex["full_segmentation_1based"]
        assert L[-1] == 6


CASES = [
    # rows, cols, k, kind, seed
    (6, 6, 2, "binary", 0),
    (50, 37, 3, "ternary", 1),
    (300, 64, 8, "binary", 2),
    (257, 100, 10, "ternary", 3),   # k > log2(rows) region: mostly empty values, two windows
    (1024, 48, 12, "binary", 4),    # eight windows
    (700, 26, 13, "ternary", 5),    # ragged last block of width 13 -> exactly 2 blocks
    (100, 33, 16, "ternary", 6),    # widest k, ragged last block of width 1
    (40, 7, 1, "ternary", 7),
    (2000, 20, 5, "binary", 8),     # long segments (about 62 rows): overflow pieces
]


def make(rows, cols, kind, seed):
    g = rng(1000 + seed)
    if kind == "binary":
        return g.integers(0, 2, size=(rows, cols)).astype(np.int8)
    return g.integers(-1, 2, size=(rows, cols)).astype(np.int8)


@pytest.mark.parametrize("rows,cols,k,kind,seed", CASES)
def test_exported_tables_equal_the_papers_definitions(rows, cols, k, kind, seed):
    A = make(rows, cols, kind, seed)
    parts = steps.ternary_split(A) if kind == "ternary" else (A,)
    with HostIndex(A, k) as h:
        assert h.info.parts == len(parts) and h.info.nblocks == -(-cols // k)
        for p, B in enumerate(parts):
            for b, Bi in enumerate(steps.column_blocks(B, k)):
                sigma, L = R.rsr_host_export_block(h.x, p, b)
                assert np.array_equal(sigma, steps.binary_row_order(Bi)), (p, b)
                assert np.array_equal(L[:-1], steps.full_segmentation(Bi)), (p, b)
                assert L[-1] == rows


def test_ternary_without_minus_ones_is_binary_and_negative_only_is_ternary():
    A = make(30, 10, "binary", 9)
    with HostIndex(A, 4) as h:
        assert h.info.parts == 1
    with HostIndex(-A, 4) as h:
        assert h.info.parts == 2
        sigma, L = R.rsr_host_export_block(h.x, 0, 0)  # B(1) is all zeros: identity order, all rows value 0
        assert sigma.tolist() == list(range(30)) and L.tolist() == [0] + [30] * 16


# ---- the packed streams: what the kernels rely on ----------------------------------------------------
def check_streams(h, S):
    info = h.info
    rows, k, kw = info.rows, info.k, info.lo_bits
    units, entries, slots, blk = S["units"], S["entries"], S["slots"], S["blk_unit"]
    assert kw == min(k, 9)
    assert len(entries) % 8 == 0 and len(slots) % 8 == 0
    assert len(blk) == info.nblocks + 1 and blk[0] == 0 and blk[-1] == len(units)
    assert np.all(np.diff(blk.astype(np.int64)) >= 1)  # every block has a unit: its outputs get written
    assert info.index_bytes == 2 * len(entries) and info.segment_bytes == 2 * len(slots)
    assert info.work_units == len(units)
    stored = 0
    for b in range(info.nblocks):
        seen = [set(), set()]
        for ui in range(blk[b], blk[b + 1]):
            U = units[ui]
            assert U["block"] == b and U["part"] < info.parts
            assert U["units_in_block"] == blk[b + 1] - blk[b]
            assert U["npieces"] <= TILE and U["nt"] <= MAX_DIAG and U["nov"] <= MAX_OVF
            assert U["window"] < (1 << (k - kw))
            cnt8 = U["cnt8"].astype(int)
            nt, ntm = int(U["nt"]), int(U["nt_main"])
            assert ntm <= nt and np.all(cnt8[nt:] == 0)
            per_diag = np.where(np.arange(40) < ntm, 8 * cnt8, cnt8)[:nt]  # stored entries per diagonal
            assert np.all(np.diff(cnt8[:ntm]) <= 0) and np.all(np.diff(cnt8[ntm:nt]) <= 0)  # only ever shrink
            assert np.all(cnt8[ntm:nt] <= 64) and np.all(cnt8[ntm:nt] >= 1)  # a tail diagonal: one entry per lane
            assert np.all(cnt8[:ntm] * 8 > 64)  # ... and it starts as soon as 64 lanes suffice
            assert int(U["main_granules"]) == int(cnt8[:ntm].sum())
            nsl = -(-int(U["npieces"]) // 8)
            if ntm:
                assert cnt8[0] == nsl
            off = int(U["entry_off"]) * 8
            n_e = int(per_diag.sum())
            n_e8 = -(-n_e // 8) * 8
            assert off + n_e8 <= len(entries)
            assert np.all(entries[off + n_e : off + n_e8] == rows)  # the tail region is padded with nulls
            e = entries[off : off + n_e].astype(int)
            assert np.all(e <= rows)  # row index or the null index
            real = e[e < rows]
            assert len(set(real.tolist())) == len(real) and not (set(real.tolist()) & seen[U["part"]])
            seen[U["part"]] |= set(real.tolist())
            stored += len(real)
            so = int(U["slot_off"]) * 8
            ids = slots[so : so + 8 * nsl].astype(int)
            used = ids[: int(U["npieces"])]
            assert np.all(ids[int(U["npieces"]) :] == WINDOW)  # padding ranks -> dummy slot
            assert len(set(used.tolist())) == len(used)  # plain stores: one writer per slot
            regular = used[used < WINDOW]
            ovf = used[used >= WINDOW]
            assert np.all(regular < (1 << kw))
            assert sorted(ovf.tolist()) == list(range(OVF_BASE, OVF_BASE + int(U["nov"])))
            npar = 8 * (-(-int(U["nov"]) // 8))
            assert so + 8 * nsl + npar <= len(slots)
            parents = slots[so + 8 * nsl : so + 8 * nsl + int(U["nov"])].astype(int)
            assert set(parents.tolist()) <= set(regular.tolist())  # a cut segment keeps its first piece in place
            # padding is null and sits only at the end of a wide diagonal; tail diagonals have none
            p = off
            lens = np.zeros(max(8 * nsl, 64), dtype=int)
            for t in range(nt):
                d = entries[p : p + per_diag[t]].astype(int)
                valid = d < rows
                nvalid = int(valid.sum())
                assert np.all(valid[:nvalid]) and np.all(d[nvalid:] == rows)
                if t >= ntm:
                    assert nvalid == per_diag[t]
                lens[:nvalid] += 1
                p += per_diag[t]
            assert np.all(np.diff(lens[: int(U["npieces"])]) <= 0)  # ranks are ordered by descending length
            assert np.all(lens[: int(U["npieces"])] >= 1) or int(U["npieces"]) == 0
    assert stored == info.stored_rows


@pytest.mark.parametrize("rows,cols,k,kind,seed", CASES)
def test_stream_invariants(rows, cols, k, kind, seed):
    A = make(rows, cols, kind, seed)
    with HostIndex(A, k) as h:
        check_streams(h, R.rsr_host_streams(h.x))


def walk(h, S, v):
    """numpy mirror of the kernel's traversal of the packed streams (int64 arithmetic)."""
    info = h.info
    rows, cols, k, kw = info.rows, info.cols, info.k, info.lo_bits
    units, entries, slots, blk = S["units"], S["entries"], S["slots"], S["blk_unit"]
    vl = np.concatenate([np.asarray(v, dtype=np.int64), [0]])
    out = np.zeros(cols, dtype=np.int64)
    value_bits = np.array([[(j >> b) & 1 for b in range(9)] for j in range(WINDOW)], dtype=np.int64)
    for b in range(info.nblocks):
        comb = np.zeros((2, 16), dtype=np.int64)
        for ui in range(blk[b], blk[b + 1]):
            U = units[ui]
            nsl8 = 8 * (-(-int(U["npieces"]) // 8))
            acc = np.zeros(TILE, dtype=np.int64)
            p = int(U["entry_off"]) * 8
            for t in range(int(U["nt_main"])):  # wide diagonals: 8 ranks per lane
                n = 8 * int(U["cnt8"][t])
                acc[:n] += vl[entries[p : p + n].astype(int)]
                p += n
            assert p == (int(U["entry_off"]) + int(U["main_granules"])) * 8
            tacc = np.zeros(64, dtype=np.int64)
            for t in range(int(U["nt_main"]), int(U["nt"])):  # tail diagonals: lane l serves rank l
                n = int(U["cnt8"][t])
                tacc[:n] += vl[entries[p : p + n].astype(int)]
                p += n
            so = int(U["slot_off"]) * 8
            win = np.zeros(WIN_SLOTS, dtype=np.int64)
            win[slots[so : so + nsl8].astype(int)] = acc[:nsl8]
            ntail = int(U["cnt8"][int(U["nt_main"])]) if int(U["nt_main"]) < int(U["nt"]) else 0
            tslots = slots[so : so + ntail].astype(int)
            assert len(set(tslots.tolist())) == ntail
            win[tslots] += tacc[:ntail]
            r = win[:WINDOW] @ value_bits
            tot = win[:WINDOW].sum()
            for o in range(int(U["nov"])):
                par = int(slots[so + nsl8 + o])
                val = win[OVF_BASE + o]
                r = r + val * value_bits[par]
                tot += val
            for bit in range(k):
                t_ = r[bit] if bit < kw else (tot if (int(U["window"]) >> (bit - kw)) & 1 else 0)
                comb[int(U["part"]), bit] += t_
        width = info.last_block_width if b == info.nblocks - 1 else k
        for c in range(width):
            out[b * k + c] = comb[0, k - 1 - c] - comb[1, k - 1 - c]
    return out


@pytest.mark.parametrize("rows,cols,k,kind,seed", CASES)
def test_walk_over_packed_streams_gives_the_product(rows, cols, k, kind, seed):
    A = make(rows, cols, kind, seed)
    v = rng(2000 + seed).integers(-127, 128, size=rows, dtype=np.int8)
    with HostIndex(A, k) as h:
        got = walk(h, R.rsr_host_streams(h.x), v)
    assert np.array_equal(got, dense.matvec_i8(A, v))


@pytest.mark.parametrize("name", ["ones", "zeros", "identity", "equal_rows", "bin_k", "two_patterns"])
def test_degenerate_matrices(name):
    g = rng(77)
    rows, cols, k = 3000, 24, 6
    if name == "ones":
        A = np.ones((rows, cols), np.int8)          # one segment of 3000 rows per block: many cut pieces
    elif name == "zeros":
        A = np.zeros((rows, cols), np.int8)         # nothing stored, outputs still written
    elif name == "identity":
        rows = cols = 200
        A = np.eye(rows, dtype=np.int8)
    elif name == "equal_rows":
        A = np.tile(g.integers(-1, 2, size=(1, cols)).astype(np.int8), (rows, 1))
    elif name == "bin_k":
        k, rows, cols = 10, 1024, 10
        A = steps.bin_matrix(k).astype(np.int8)     # sigma = identity, every segment one row
    else:
        pats = g.integers(-1, 2, size=(2, cols)).astype(np.int8)
        A = pats[g.integers(0, 2, size=rows)]
    v = g.integers(-127, 128, size=A.shape[0], dtype=np.int8)
    with HostIndex(A, k) as h:
        S = R.rsr_host_streams(h.x)
        check_streams(h, S)
        assert np.array_equal(walk(h, S, v), dense.matvec_i8(A, v))
        if name == "zeros":
            assert h.info.stored_rows == 0 and h.info.work_units == h.info.nblocks
        if name == "bin_k":
            sigma, L = R.rsr_host_export_block(h.x, 0, 0)
            assert sigma.tolist() == list(range(1024)) and L.tolist() == list(range(1025))
