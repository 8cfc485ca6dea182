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
WINDOW, LANES, MAX_POS, ALIGN = 512, 64, 48, 128


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
    assert {"rsr_matvec_multi", "rsr_set_step2", "rsr_model_k", "rsr_autotune_k"} <= names
    lib = R.load()
    for n in sorted(names):
        assert hasattr(lib, n), f"{n} declared in rsr.h but not exported"
    dense_h = re.sub(r"/\*.*?\*/", "", open(os.path.join(ROOT, "include", "rsr_dense.h")).read(), flags=re.S)
    dnames = set(re.findall(r"\b(rsr_dense_[a-z0-9_]+)\s*\(", dense_h))
    assert {"rsr_dense_preprocess", "rsr_dense_matvec", "rsr_dense_matvec_i8", "rsr_dense_destroy"} <= dnames
    for n in sorted(dnames):
        assert hasattr(lib, n), f"{n} declared in rsr_dense.h but not exported"
    qbit_h = re.sub(r"/\*.*?\*/", "", open(os.path.join(ROOT, "include", "rsr_qbit.h")).read(), flags=re.S)
    qnames = set(re.findall(r"\b(rsr_qbit_[a-z0-9_]+)\s*\(", qbit_h))
    assert {"rsr_qbit_preprocess", "rsr_qbit_matvec", "rsr_qbit_matvec_i8", "rsr_qbit_destroy"} <= qnames
    assert {"rsr_matvec_acc", "rsr_matvec_acc_i8"} <= names
    for n in sorted(qnames):
        assert hasattr(lib, n), f"{n} declared in rsr_qbit.h but not exported"


def test_block_width_by_the_papers_cost_formula():
    # argmin over k of (n + 2^k) / k (Section 4.3), worked by hand: n = 1024: k=7 gives 164.6, k=8 160, k=9 170.7
    assert R.rsr_model_k(1024, 1, 16) == 8
    assert R.rsr_model_k(1024, 1, 6) == 6 and R.rsr_model_k(1024, 10, 12) == 10
    with pytest.raises(R.RsrError):
        R.rsr_model_k(1024, 0, 5)


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
    (2000, 20, 5, "binary", 8),     # long segments (about 62 rows): spread over many lanes
    (40000, 7, 3, "ternary", 9),    # more than 32768 rows: two row tiles
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
def unit_bytes(npos):
    raw = npos * 2 * LANES + (4 * LANES if npos else 0) + (2 * LANES if npos > 32 else 0)
    return -(-raw // ALIGN) * ALIGN


def unit_positions(stream, U):
    """The unit's row indices as an array [position][lane] and its flags [position][lane], undoing the
    granule order of the device."""
    npos = int(U["npos"])
    base = int(U["stream_off"]) * (ALIGN // 2)
    full = npos // 8
    pos = np.empty((npos, LANES), dtype=np.int64)
    if full:
        g = stream[base : base + full * 8 * LANES].reshape(full, LANES, 8)
        pos[: full * 8] = g.transpose(0, 2, 1).reshape(full * 8, LANES)
    rest = npos - full * 8
    if rest // 2:
        t = stream[base + full * 8 * LANES : base + (full * 8 + rest // 2 * 2) * LANES].reshape(rest // 2, LANES, 2)
        pos[full * 8 : full * 8 + rest // 2 * 2] = t.transpose(0, 2, 1).reshape(rest // 2 * 2, LANES)
    if npos & 1:
        pos[npos - 1] = stream[base + (npos - 1) * LANES : base + npos * LANES]
    flags = np.zeros((npos, LANES), dtype=np.int64)
    if npos:
        f = stream[base + npos * LANES : base + npos * LANES + 2 * LANES].astype(np.int64).reshape(LANES, 2)
        f0 = f[:, 0] | (f[:, 1] << 16)
        for p_ in range(min(npos, 32)):
            flags[p_] = (f0 >> (31 - p_)) & 1
        if npos > 32:
            f1 = stream[base + npos * LANES + 2 * LANES : base + npos * LANES + 3 * LANES].astype(np.int64)
            for p_ in range(32, npos):
                flags[p_] = (f1 >> (47 - p_)) & 1
    return pos, flags


def unit_entries(U, pos, flags):
    """Entries in the order the lanes own them (lane 0's run, then lane 1's ...): rows, flags, slots."""
    rows_ = pos.T.reshape(-1)
    fl = flags.T.reshape(-1)
    slots = int(U["slot0"]) + np.cumsum(fl)
    return rows_, fl, slots


def check_streams(h, S=None):
    """Invariants of the packed streams, over all row tiles (S: the streams of tile 0 if already fetched)."""
    info = h.info
    tiles = [S if (S is not None and t == 0) else R.rsr_host_streams(h.x, t) for t in range(info.row_tiles)]
    assert info.row_tiles == max(1, -(-info.rows // 32768))
    assert sum(T["rows"] for T in tiles) == info.rows and tiles[0]["row0"] == 0
    assert all(a["row0"] + a["rows"] == b["row0"] for a, b in zip(tiles, tiles[1:]))
    assert info.index_bytes + info.segment_bytes == sum(2 * len(T["stream"]) for T in tiles)
    assert info.work_units == sum(len(T["units"]) for T in tiles)
    assert info.schedule_bytes == sum(32 * len(T["units"]) + 4 * len(T["blk_unit"]) for T in tiles)
    totals = [check_tile(info, T) for T in tiles]
    assert sum(t[0] for t in totals) == info.stored_rows and sum(t[1] for t in totals) == info.segments
    assert sum(t[2] for t in totals) == info.segment_bytes


def check_tile(info, S):
    rows, k, kw = S["rows"], info.k, info.lo_bits
    units, stream, blk = S["units"], S["stream"], S["blk_unit"]
    assert kw == min(k, 9)
    assert len(stream) % (ALIGN // 2) == 0
    assert len(blk) == info.nblocks + 1 and blk[0] == 0 and blk[-1] == len(units)
    assert np.all(np.diff(blk.astype(np.int64)) >= 1)  # every block has a unit: its outputs get written
    stored = heads = flag_bytes = 0
    next_off = 0
    for b in range(info.nblocks):
        seen = [set(), set()]
        last_value = [-1, -1]
        for ui in range(blk[b], blk[b + 1]):
            U = units[ui]
            part = int(U["part"])
            assert U["block"] == b and part < info.parts
            assert U["units_in_block"] == blk[b + 1] - blk[b] and U["index_in_block"] == ui - blk[b]
            assert U["window"] < (1 << (k - kw))
            npos = int(U["npos"])
            assert npos <= MAX_POS
            assert int(U["stream_off"]) == next_off  # unit streams are back to back, 128-byte aligned
            next_off += unit_bytes(npos) // ALIGN
            flag_bytes += (4 * LANES if npos else 0) + (2 * LANES if npos > 32 else 0)
            if npos == 0:
                assert U["nentries"] == 0 and U["nrows"] == 0
                continue
            pos, flags = unit_positions(stream, U)
            rr, fl, slots = unit_entries(U, pos, flags)
            n = int(U["nentries"])
            assert 0 < n <= npos * LANES and npos == -(-n // LANES)  # no more positions than needed
            assert np.all(rr[n:] == rows) and np.all(fl[n:] == 0)  # the padding of the last lanes
            assert fl[0] == 0 and rr[0] < rows and rr[n - 1] < rows  # starts and ends with a row
            assert np.all(rr <= rows)
            assert slots[n - 1] < (1 << kw)  # every slot lies in the window
            real = rr[:n] < rows
            assert np.all(fl[:n][~real] == 1)  # a null entry stands for an absent value: it always moves on
            # (the order of the rows inside a segment is the packer's choice: it spreads them over the LDS banks)
            values = (int(U["window"]) << kw) + slots[:n][real]
            assert values[0] >= last_value[part]  # units of a part follow each other in value order
            last_value[part] = int(values[-1])
            got = rr[:n][real].tolist()
            assert len(set(got)) == len(got) and not (set(got) & seen[part])
            seen[part] |= set(got)
            assert len(got) == int(U["nrows"]) and int(fl.sum()) == int(U["nheads"])
            stored += len(got)
            heads += int(fl.sum()) + 1
    assert next_off * ALIGN == 2 * len(stream)
    return stored, heads, flag_bytes


@pytest.mark.parametrize("rows,cols,k,kind,seed", CASES)
def test_stream_invariants(rows, cols, k, kind, seed):
    A = make(rows, cols, kind, seed)
    with HostIndex(A, k) as h:
        check_streams(h, R.rsr_host_streams(h.x))


def walk(h, S, v):
    """numpy mirror of the kernel's traversal of the packed streams (int64 arithmetic): every lane walks
    its run with one running sum, stores it where a flag says that a new value starts, and what it is
    left with is added to its last slot afterwards.  The products of the row tiles add up."""
    info = h.info
    out = np.zeros(info.cols, dtype=np.int64)
    for t in range(info.row_tiles):
        T = S if t == 0 else R.rsr_host_streams(h.x, t)
        out += walk_tile(info, T, np.asarray(v)[T["row0"] : T["row0"] + T["rows"]])
    return out


def walk_tile(info, S, v):
    cols, k, kw = info.cols, info.k, info.lo_bits
    units, stream, blk = S["units"], S["stream"], S["blk_unit"]
    vl = np.concatenate([np.asarray(v, dtype=np.int64), [0]])
    out = np.zeros(cols, dtype=np.int64)
    value_bits = np.array([[(j >> b) & 1 for b in range(9)] for j in range(WINDOW)], dtype=np.int64)
    for b in range(info.nblocks):
        comb = np.zeros((2, 16), dtype=np.int64)
        for ui in range(blk[b], blk[b + 1]):
            U = units[ui]
            win = np.zeros(WINDOW, dtype=np.int64)
            npos = int(U["npos"])
            if npos:
                pos, flags = unit_positions(stream, U)
                nflag = flags.sum(axis=0)
                slot = int(U["slot0"]) + np.cumsum(nflag) - nflag  # the lane's first slot
                acc = np.zeros(LANES, dtype=np.int64)
                for p in range(npos):
                    f = flags[p].astype(bool)
                    win[slot[f]] = acc[f]          # plain stores: one lane per slot
                    assert len(set(slot[f].tolist())) == int(f.sum())
                    slot = slot + flags[p]
                    acc[f] = 0
                    acc += vl[pos[p]]
                np.add.at(win, slot, acc)          # the open segments
            r = win @ value_bits
            tot = win.sum()
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


def test_long_segments_and_big_windows_are_split_into_units():
    g = rng(5)
    # 4000 rows, block width 3: seven segments of about 500 rows, each spread over many lanes
    A = g.integers(0, 2, size=(4000, 6)).astype(np.int8)
    with HostIndex(A, 3) as h:
        S = R.rsr_host_streams(h.x)
        check_streams(h, S)
        assert 2 * h.info.stored_rows > 0.95 * h.info.index_bytes  # long segments still fill the lanes
    # 60000 equal rows: one segment spread over several units of the same window
    A = np.ones((60000, 2), np.int8)
    with HostIndex(A, 2) as h:
        S = R.rsr_host_streams(h.x)
        check_streams(h, S)
        assert h.info.row_tiles == 2 and S["rows"] == 30000   # two row tiles of equal height
        assert len(S["units"]) == -(-30000 // (MAX_POS * LANES)) and np.all(S["units"]["window"] == 0)
        assert 2 * h.info.stored_rows > 0.95 * h.info.index_bytes
        assert S["units"]["nheads"].sum() == 0
        v = g.integers(-127, 128, size=60000, dtype=np.int8)
        assert np.array_equal(walk(h, S, v), dense.matvec_i8(A, v))
        sigma, L = R.rsr_host_export_block(h.x, 0, 0)       # the tiles together are the index of the matrix
        assert sigma.tolist() == list(range(60000)) and L.tolist() == [0, 0, 0, 0, 60000]
    # the index of a random matrix is little more than 16 bits per row plus one flag bit
    A = g.integers(0, 2, size=(4096, 40)).astype(np.int8)
    with HostIndex(A, 10) as h:
        assert h.info.index_bytes + h.info.segment_bytes < 1.10 * (2 + 1 / 8) * h.info.stored_rows


@pytest.mark.parametrize("name", ["ones", "zeros", "identity", "equal_rows", "bin_k", "two_patterns"])
def test_degenerate_matrices(name):
    g = rng(77)
    rows, cols, k = 3000, 24, 6
    if name == "ones":
        A = np.ones((rows, cols), np.int8)          # one segment of 3000 rows per block: many pieces
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


def gather_passes(S, rows):
    """LDS cycles per half-wavefront gather of float activations (bank = row mod 32): for every position
    and half, the largest number of distinct rows that fall into one bank (the null index reads one
    shared word)."""
    units, stream = S["units"], S["stream"]
    total = count = 0
    for U in units:
        if int(U["npos"]) == 0:
            continue
        pos, _ = unit_positions(stream, U)
        for half in (0, 1):
            sub = pos[:, 32 * half : 32 * half + 32]
            for t in range(sub.shape[0]):
                rr = np.unique(sub[t])
                total += int(np.bincount(rr % 32, minlength=32).max())
                count += 1
    return total / max(count, 1)


def test_rows_of_a_half_wavefront_are_spread_over_the_lds_banks():
    # 32 random rows fall into 32 banks with about 3.5 in the fullest one.  The packer may reorder the rows
    # of a segment; with segments of four rows on average that must bring the mean clearly below.
    A = make(4096, 40, "binary", 11)
    with HostIndex(A, 10) as h:
        mean = gather_passes(R.rsr_host_streams(h.x), 4096)
    assert mean < 2.6, mean
