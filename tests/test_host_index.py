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
WINDOW, DUMMY, OVF_BASE, MAX_OVF, WIN_SLOTS, LANES, MAX_POS, ALIGN = 512, 8, 520, 256, 776, 64, 48, 256


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
    (2000, 20, 5, "binary", 8),     # long segments (about 62 rows): several pieces each
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
def unit_positions(stream, U):
    """The unit's stream as an array [position][lane], undoing the granule order of the device."""
    npos = int(U["npos"])
    base = int(U["stream_off"]) * (ALIGN // 2)
    full = npos // 8
    pos = np.empty((npos, LANES), dtype=np.int64)
    if full:
        g = stream[base : base + full * 8 * LANES].reshape(full, LANES, 8)
        pos[: full * 8] = g.transpose(0, 2, 1).reshape(full * 8, LANES)
    rest = npos - full * 8
    if rest:
        t = stream[base + full * 8 * LANES : base + npos * LANES].reshape(rest // 2, LANES, 2)
        pos[full * 8 :] = t.transpose(0, 2, 1).reshape(rest, LANES)
    return pos


def unit_groups(U, pos):
    """(parent positions, [(header position, index positions)]) of the unit."""
    hdr = (int(U["hdr_hi"]) << 32) | int(U["hdr_lo"])
    npar = int(U["npar"])
    heads = [p for p in range(int(U["npos"])) if (hdr >> p) & 1]
    assert hdr >> int(U["npos"]) == 0 and len(heads) == int(U["ngroups"])
    if heads:
        assert heads[0] == npar  # the parents come first, then the first group
    else:
        assert npar == 0
    return npar, [(h, list(range(h + 1, nxt))) for h, nxt in zip(heads, heads[1:] + [int(U["npos"])])]


def check_streams(h, S):
    info = h.info
    rows, k, kw = info.rows, info.k, info.lo_bits
    units, stream, blk = S["units"], S["stream"], S["blk_unit"]
    assert kw == min(k, 9)
    assert len(stream) % (ALIGN // 2) == 0
    assert len(blk) == info.nblocks + 1 and blk[0] == 0 and blk[-1] == len(units)
    assert np.all(np.diff(blk.astype(np.int64)) >= 1)  # every block has a unit: its outputs get written
    assert info.index_bytes + info.segment_bytes == 2 * len(stream)
    assert info.segment_bytes == 128 * int(units["ngroups"].astype(np.int64).sum())
    assert info.work_units == len(units)
    assert info.schedule_bytes == 32 * len(units) + 4 * len(blk)
    stored = pieces = 0
    next_off = 0
    for b in range(info.nblocks):
        seen = [set(), set()]
        for ui in range(blk[b], blk[b + 1]):
            U = units[ui]
            assert U["block"] == b and U["part"] < info.parts
            assert U["units_in_block"] == blk[b + 1] - blk[b] and U["index_in_block"] == ui - blk[b]
            assert U["window"] < (1 << (k - kw))
            npos = int(U["npos"])
            assert npos % 2 == 0 and npos <= MAX_POS and int(U["npar"]) <= MAX_OVF // LANES
            assert int(U["stream_off"]) == next_off  # unit streams are back to back, 256-byte aligned
            next_off += npos * LANES * 2 // ALIGN
            pos = unit_positions(stream, U)
            npar, groups = unit_groups(U, pos)
            parents = pos[:npar].reshape(-1)  # parent of overflow slot x, or the null index if x is unused
            assert np.all((parents < (1 << kw)) | (parents == rows))
            in_use = np.flatnonzero(parents < (1 << kw)) if rows >= (1 << kw) else None
            used_slots = []
            nidx = 0
            last_len = None
            for head, idxs in groups:
                slots = pos[head]
                assert np.all(slots < WIN_SLOTS)
                body = pos[idxs] if idxs else np.empty((0, LANES), dtype=np.int64)
                assert np.all(body <= rows)  # row index or the null index
                real = body < rows
                lens = real.sum(axis=0)
                # a piece may use any of its group's positions (its rows are summed); groups are ranked by
                # descending piece length: no piece is longer than the shortest piece of the group before
                owners = lens > 0
                assert last_len is None or lens.max() <= last_len
                last_len = lens[owners].min() if owners.any() else last_len
                assert np.all(slots[~owners] >= WINDOW) and np.all(slots[~owners] < OVF_BASE)  # dummies
                own = slots[owners]
                assert np.all((own < (1 << kw)) | ((own >= OVF_BASE) & (own < OVF_BASE + LANES * npar)))
                # only the unit's last group may carry one all-null position (even position count)
                assert lens.max() >= len(idxs) - (1 if head == groups[-1][0] else 0) and lens.max() >= 1
                used_slots += own.tolist()
                pieces += int(owners.sum())
                rr = body[real].tolist()
                assert len(set(rr)) == len(rr) and not (set(rr) & seen[U["part"]])
                seen[U["part"]] |= set(rr)
                nidx += len(rr)
            assert len(set(used_slots)) == len(used_slots)  # plain stores: one writer per slot and unit
            ovf = sorted(x - OVF_BASE for x in used_slots if x >= OVF_BASE)
            if in_use is not None:
                assert ovf == in_use.tolist()  # exactly the overflow slots that have a parent
            if npar:
                assert ovf and ovf[-1] >= LANES * (npar - 1)  # no parent position without need
            regular = set(x for x in used_slots if x < WINDOW)
            for x in ovf:
                par = int(parents[x])
                assert par in regular  # a further piece follows a first piece of its segment in the same unit
                assert (x % LANES) // 16 == par >> 7  # folded by a lane in the row of the parent's bits 7, 8
            assert nidx == int(U["nidx"]) and len(used_slots) == int(U["npieces"])
            stored += nidx
    assert next_off * ALIGN == 2 * len(stream)
    assert stored == info.stored_rows and pieces == info.segments


@pytest.mark.parametrize("rows,cols,k,kind,seed", CASES)
def test_stream_invariants(rows, cols, k, kind, seed):
    A = make(rows, cols, kind, seed)
    with HostIndex(A, k) as h:
        check_streams(h, R.rsr_host_streams(h.x))


def walk(h, S, v):
    """numpy mirror of the kernel's traversal of the packed streams (int64 arithmetic)."""
    info = h.info
    rows, cols, k, kw = info.rows, info.cols, info.k, info.lo_bits
    units, stream, blk = S["units"], S["stream"], S["blk_unit"]
    vl = np.concatenate([np.asarray(v, dtype=np.int64), [0]])
    out = np.zeros(cols, dtype=np.int64)
    value_bits = np.array([[(j >> b) & 1 for b in range(9)] for j in range(WINDOW)], dtype=np.int64)
    for b in range(info.nblocks):
        comb = np.zeros((2, 16), dtype=np.int64)
        for ui in range(blk[b], blk[b + 1]):
            U = units[ui]
            pos = unit_positions(stream, U)
            hdr = (int(U["hdr_hi"]) << 32) | int(U["hdr_lo"])
            win = np.zeros(WIN_SLOTS, dtype=np.int64)
            acc = np.zeros(LANES, dtype=np.int64)
            slot = WINDOW + (np.arange(LANES) & (DUMMY - 1))
            # (the kernel also gathers at the parent positions, into a dummy slot that is never read)
            npar = int(U["npar"])
            for p in range(npar, int(U["npos"])):
                if (hdr >> p) & 1:
                    win[slot] = acc
                    slot = pos[p].copy()
                    acc[:] = 0
                else:
                    acc += vl[pos[p]]
            win[slot] = acc
            r = win[:WINDOW] @ value_bits
            tot = win[:WINDOW].sum()
            parents = pos[:npar].reshape(-1)
            for o in range(LANES * npar):
                val = win[OVF_BASE + o]
                if val:  # unused overflow slots stay 0 (their parent is the null index)
                    r = r + val * value_bits[int(parents[o])]
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


def test_long_segments_are_cut_and_big_windows_split_into_units():
    g = rng(5)
    # 4000 rows, block width 3: seven segments of about 500 rows -> many pieces per segment
    A = g.integers(0, 2, size=(4000, 6)).astype(np.int8)
    with HostIndex(A, 3) as h:
        S = R.rsr_host_streams(h.x)
        check_streams(h, S)
        assert S["units"]["npar"].max() > 0 and h.info.segments > 2 * 7 * 2
        assert 2 * h.info.stored_rows > 0.75 * h.info.index_bytes  # long segments still fill the lanes
    # 60000 equal rows: one segment spread over several units of the same window
    A = np.ones((60000, 2), np.int8)
    with HostIndex(A, 2) as h:
        S = R.rsr_host_streams(h.x)
        check_streams(h, S)
        assert len(S["units"]) >= 60000 // (47 * 64) and np.all(S["units"]["window"] == 0)
        assert 2 * h.info.stored_rows > 0.9 * h.info.index_bytes
    # short segments only: nothing is cut more than once
    A = g.integers(0, 2, size=(1500, 9)).astype(np.int8)
    with HostIndex(A, 9) as h:
        S = R.rsr_host_streams(h.x)
        assert h.info.segments < 1.5 * 511


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
    """LDS passes per half-wavefront gather of float activations (bank = row mod 32): for every index
    position and half, the largest number of distinct rows that fall into one bank."""
    units, stream = S["units"], S["stream"]
    total, count, worst = 0, 0, 0
    conflict_free_possible, conflict_free = 0, 0
    for U in units:
        pos = unit_positions(stream, U)
        _, groups = unit_groups(U, pos)
        for head, idxs in groups:
            body = pos[idxs] if idxs else np.empty((0, LANES), dtype=np.int64)
            while body.shape[0] and np.all(body[-1] == rows):  # the position that makes the count even
                body = body[:-1]
            for half in (0, 1):
                sub = body[:, 32 * half : 32 * half + 32]
                real = sub[sub < rows]
                degree = np.bincount(real % 32, minlength=32).max() if real.size else 0
                passes = []
                for t in range(sub.shape[0]):
                    rr = np.unique(sub[t][sub[t] < rows])
                    passes.append(max(1, int(np.bincount(rr % 32, minlength=32).max()) if rr.size else 1))
                total += sum(passes)
                count += len(passes)
                worst = max(worst, max(passes, default=1))
                if sub.shape[0] and degree <= sub.shape[0]:  # no bank has more rows than there are positions
                    conflict_free_possible += 1
                    conflict_free += all(x == 1 for x in passes)
    return total / max(count, 1), worst, conflict_free_possible, conflict_free


def test_rows_of_a_half_wavefront_are_spread_over_the_lds_banks():
    # Random rows in random order cost about 3.5 passes per gather here.  The packer's placement must
    # stay clearly below, must never need more than two passes where no bank holds more than twice
    # the positions of its half group, and must be conflict-free wherever that is possible at all.
    A = make(4096, 80, "binary", 11)
    with HostIndex(A, 10) as h:
        S = R.rsr_host_streams(h.x)
        mean, worst, possible, achieved = gather_passes(S, 4096)
    assert mean < 2.0 and worst <= 2
    assert possible > 0 and achieved == possible
