"""GPU parity: the HIP library, called through the C ABI, against the CPU oracle.

int8 activations: bit-exact.  float activations: |gpu - oracle| <= 1e-5 * sum_i |v_i| per output,
oracle accumulating in float64.  Inputs are seeded and synthetic (workloads/), at the shapes of
the benchmark configurations; the bigger ones are checked in full because the C oracle finishes
them in seconds.
"""
import numpy as np
import pytest

import paper_2411_06360_amd as R
import workloads
from oracle import dense, steps
from tests.gpu_util import DeviceIndex, assert_f32_close

pytestmark = pytest.mark.gpu


def rng(seed):
    return np.random.default_rng(seed)


def note(msg):
    print(msg, flush=True)


# ---- configuration 1: binary 1024^2, k = 8, int8, bit-exact -----------------------------------------
def test_config1_binary_1k_int8_bit_exact():
    w = workloads.get("binary_1k")
    A, v = w.matrix(), w.activations(1, "i8")
    note(f"config1 {A.shape} k={w.k}")
    with DeviceIndex(A, w.k) as d:
        got = d.matvec(v)
        assert np.array_equal(got.astype(np.int64), dense.matvec_i8(A, v))
        # the float path on the same matrix
        vf = w.activations(1, "f32")
        assert_f32_close(d.matvec(vf), dense.matvec_f32(A, vf), vf)


# ---- configuration 2: ternary 4096^2, k = 10, float --------------------------------------------------
def test_config2_ternary_4k_f32():
    w = workloads.get("ternary_4k")
    A, v = w.matrix(), w.activations(1, "f32")
    note(f"config2 {A.shape} k={w.k}")
    with DeviceIndex(A, w.k) as d:
        assert d.info.parts == 2 and d.info.nblocks == 410 and d.info.last_block_width == 6
        worst = assert_f32_close(d.matvec(v), dense.matvec_f32(A, v), v)
        note(f"  worst error / bound = {worst:.3g}")
        v8 = w.activations(2, "i8")
        assert np.array_equal(d.matvec(v8).astype(np.int64), dense.matvec_i8(A, v8))


# ---- small shapes: several tiles, ragged tails, every k ------------------------------------------------
SMALL = [
    # rows, cols, k, kind
    (1, 1, 1, "binary"), (6, 6, 2, "binary"), (50, 37, 3, "ternary"), (300, 64, 8, "binary"),
    (257, 100, 10, "ternary"), (1024, 48, 12, "binary"), (700, 26, 13, "ternary"), (100, 33, 16, "ternary"),
    (2000, 20, 5, "binary"), (4097, 130, 9, "ternary"), (513, 1000, 7, "ternary"), (3, 5000, 4, "ternary"),
]


@pytest.mark.parametrize("rows,cols,k,kind", SMALL)
def test_small_shapes_int8_exact_and_f32_close(rows, cols, k, kind):
    g = rng(rows * 7 + cols * 3 + k)
    A = (g.integers(0, 2, size=(rows, cols)) if kind == "binary" else g.integers(-1, 2, size=(rows, cols))).astype(np.int8)
    note(f"small {rows}x{cols} k={k} {kind}")
    with DeviceIndex(A, k) as d:
        for batch in (1, 3):
            v8 = g.integers(-127, 128, size=(batch, rows), dtype=np.int8)
            assert np.array_equal(d.matvec(v8).astype(np.int64), dense.matvec_i8(A, v8))
            vf = g.standard_normal((batch, rows)).astype(np.float32)
            assert_f32_close(d.matvec(vf), dense.matvec_f32(A, vf), vf)


# ---- layout paths: many pieces per segment, several units per window, several rounds per workgroup ------
LAYOUT = [
    # name, rows, cols, k, what it exercises
    ("equal_rows", 30000, 4, 2, "one segment of 30000 rows: ~700 pieces, 4 parent positions, >10 units of one window"),
    ("seven_long_segments", 4000, 6, 3, "segments of ~500 rows: every unit full of pieces of the same few segments"),
    ("skewed_lengths", 5000, 40, 10, "ternary with 70 % zeros: segment lengths from 1 to ~150 in one window"),
    ("many_blocks", 200, 40000, 1, "40000 blocks: more than 64 blocks per workgroup, several rounds"),
    ("wide_k16", 3000, 64, 16, "k = 16: 128 windows per block, mostly empty"),
    ("two_patterns_ternary", 9000, 30, 10, "rows drawn from two patterns: two segments of ~4500 rows per part"),
]


@pytest.mark.parametrize("name,rows,cols,k,what", LAYOUT)
def test_layout_paths(name, rows, cols, k, what):
    g = rng(len(name) * 131 + rows)
    if name == "equal_rows":
        A = np.ones((rows, cols), np.int8)
    elif name == "skewed_lengths":
        A = g.choice(np.array([-1, 0, 1], np.int8), size=(rows, cols), p=[0.15, 0.7, 0.15])
    elif name == "two_patterns_ternary":
        A = g.integers(-1, 2, size=(2, cols)).astype(np.int8)[g.integers(0, 2, size=rows)]
    elif name in ("seven_long_segments", "many_blocks"):
        A = g.integers(0, 2, size=(rows, cols)).astype(np.int8)
    else:
        A = g.integers(-1, 2, size=(rows, cols)).astype(np.int8)
    note(f"layout {name}: {what}")
    with DeviceIndex(A, k) as d:
        for batch in (1, 2):
            v8 = g.integers(-127, 128, size=(batch, rows), dtype=np.int8)
            assert np.array_equal(d.matvec(v8).astype(np.int64), dense.matvec_i8(A, v8))
            vf = g.standard_normal((batch, rows)).astype(np.float32)
            assert_f32_close(d.matvec(vf), dense.matvec_f32(A, vf), vf)
        if name == "equal_rows":  # closed form: every output is the sum of v
            v1 = np.ones((1, rows), np.int8)
            assert np.all(d.matvec(v1) == rows)
    if name == "equal_rows":  # and twice the rows: one segment over two row tiles
        A2 = np.ones((60000, 2), np.int8)
        with DeviceIndex(A2, 2) as d:
            v8 = g.integers(-127, 128, size=(1, 60000), dtype=np.int8)
            assert np.array_equal(d.matvec(v8).astype(np.int64), dense.matvec_i8(A2, v8))
            vf = (g.random((1, 60000)) + 0.5).astype(np.float32)
            assert_f32_close(d.matvec(vf), dense.matvec_f32(A2, vf), vf)


def test_extreme_activations_int8_minus_128_and_coherent_float_signs():
    """Where the stated bounds are actually exercised: int8 activations all at -128 on a matrix whose
    rows all count (|sum| = 128 * rows, the largest magnitude the int32 accumulator sees), and float
    activations that are all positive on 30000 equal rows (every output is the sum of the whole vector,
    so rounding errors cannot cancel: the error bound 1e-5 * sum|v| is checked element by element)."""
    g = rng(61)
    rows = 30000
    A = np.ones((rows, 6), np.int8)
    A[:, 3:] = -1
    note("extremes: 30000 equal rows, int8 -128 and all-positive float")
    with DeviceIndex(A, 3) as d:
        v8 = np.full((2, rows), -128, np.int8)
        v8[1, ::2] = 127
        got = d.matvec(v8).astype(np.int64)
        assert np.array_equal(got, dense.matvec_i8(A, v8))
        assert got[0, 0] == -128 * rows and got[0, 5] == 128 * rows
        vf = (g.random((2, rows)) + 0.5).astype(np.float32)          # all in [0.5, 1.5)
        vf[1] *= np.float32(1000.0)
        worst = assert_f32_close(d.matvec(vf), dense.matvec_f32(A, vf), vf)
        note(f"  coherent signs: worst error / bound = {worst:.3g}")
    # the same on random binary rows with 16 rows per segment on average and all-positive activations
    B = g.integers(0, 2, size=(rows, 44)).astype(np.int8)
    with DeviceIndex(B, 11) as d:
        vf = (g.random((1, rows)) + 0.5).astype(np.float32)
        worst = assert_f32_close(d.matvec(vf), dense.matvec_f32(B, vf), vf)
        note(f"  random rows, positive activations: worst error / bound = {worst:.3g}")
        v8 = np.full((1, rows), -128, np.int8)
        assert np.array_equal(d.matvec(v8).astype(np.int64), dense.matvec_i8(B, v8))


def test_k_invariance_same_matrix_every_k():
    g = rng(41)
    A = g.integers(-1, 2, size=(600, 70)).astype(np.int8)
    v8 = g.integers(-127, 128, size=600, dtype=np.int8)
    vf = g.standard_normal(600).astype(np.float32)
    want8, wantf = dense.matvec_i8(A, v8), dense.matvec_f32(A, vf)
    for k in range(1, 17):
        note(f"k-invariance k={k}")
        with DeviceIndex(A, k) as d:
            assert np.array_equal(d.matvec(v8).astype(np.int64), want8), k
            assert_f32_close(d.matvec(vf), wantf, vf)


@pytest.mark.parametrize("name", ["ones", "zeros", "identity", "equal_rows", "bin_k", "paper"])
def test_degenerate_and_closed_form_matrices(name, golden):
    g = rng(43)
    rows, cols, k = 3000, 24, 6
    if name == "ones":
        A = np.ones((rows, cols), np.int8)
    elif name == "zeros":
        A = np.zeros((rows, cols), np.int8)
    elif name == "identity":
        rows = cols = 200
        A = np.eye(rows, dtype=np.int8)
    elif name == "equal_rows":
        A = np.tile(g.integers(-1, 2, size=(1, cols)).astype(np.int8), (rows, 1))
    elif name == "bin_k":
        k, rows, cols = 10, 1024, 10
        A = steps.bin_matrix(k).astype(np.int8)  # u = v: the product is the fold of v
    else:
        A = np.array(golden["matrix_B"]["rows"], dtype=np.int8)
        k = 2
    rows = A.shape[0]
    note(f"degenerate {name} {A.shape} k={k}")
    v8 = g.integers(-127, 128, size=rows, dtype=np.int8)
    vf = g.standard_normal(rows).astype(np.float32)
    with DeviceIndex(A, k) as d:
        got8 = d.matvec(v8).astype(np.int64)
        assert np.array_equal(got8, dense.matvec_i8(A, v8))
        gotf = d.matvec(vf)
        assert_f32_close(gotf, dense.matvec_f32(A, vf), vf)
        if name == "ones":
            assert np.all(got8 == int(v8.astype(np.int64).sum()))
        if name == "zeros":
            assert np.all(got8 == 0) and np.all(gotf == 0)
        if name == "identity":
            assert np.array_equal(got8, v8.astype(np.int64)) and np.array_equal(gotf, vf)
        if name == "paper":
            d8 = np.array(golden["derived_product"]["v"], dtype=np.int8)
            assert d.matvec(d8).tolist() == golden["derived_product"]["v_dot_B"]


def test_tables_on_the_device_are_the_papers_index(golden):
    B = np.array(golden["matrix_B"]["rows"], dtype=np.int8)
    with DeviceIndex(B, 2) as d:
        sigma, L = R.rsr_export_block(d.handle, 0, 0)
        assert (sigma + 1).tolist() == golden["example_3_3"]["sigma_1based"]
        assert (L[:-1] + 1).tolist() == golden["example_3_3"]["full_segmentation_1based"]
    g = rng(47)
    A = g.integers(-1, 2, size=(900, 45)).astype(np.int8)
    with DeviceIndex(A, 10) as d:
        for p, Bp in enumerate(steps.ternary_split(A)):
            for b, Bi in enumerate(steps.column_blocks(Bp, 10)):
                sigma, L = R.rsr_export_block(d.handle, p, b)
                assert np.array_equal(sigma, steps.binary_row_order(Bi))
                assert np.array_equal(L[:-1], steps.full_segmentation(Bi)) and L[-1] == 900


def test_results_are_reproducible_and_batch_equals_single_calls():
    w = workloads.get("ternary_4k")
    A = w.matrix()[:2048, :777].copy()
    g = rng(53)
    vf = g.standard_normal((5, 2048)).astype(np.float32)
    v8 = g.integers(-127, 128, size=(5, 2048), dtype=np.int8)
    with DeviceIndex(A, 10) as d:
        a, b = d.matvec(vf), d.matvec(vf)
        assert np.array_equal(a, b)  # fixed summation order
        singles = np.stack([d.matvec(vf[i]) for i in range(5)])
        assert np.array_equal(a, singles)
        assert np.array_equal(d.matvec(v8), np.stack([d.matvec(v8[i]) for i in range(5)]))


def test_product_captured_in_a_graph_gives_the_eager_result_on_every_replay():
    """rsr_matvec allocates nothing and enqueues one kernel: it can be captured in a HIP graph.  The graph
    is replayed several times with new activations and eager work in between; every replay must equal the
    eager product of the same activations bit for bit."""
    import torch

    g = rng(92)
    A = g.integers(-1, 2, size=(3000, 500)).astype(np.int8)
    note("graph capture 3000x500 k=9 batch 3")
    with DeviceIndex(A, 9) as d:
        dv = torch.zeros((3, 3000), dtype=torch.float32, device="cuda")
        out = torch.zeros((3, 500), dtype=torch.float32, device="cuda")
        eager = torch.zeros_like(out)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):  # warm-up on the capture stream
            R.rsr_matvec(d.handle, dv, out, 3, side.cuda_stream)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            R.rsr_matvec(d.handle, dv, out, 3, torch.cuda.current_stream().cuda_stream)
        for rep in range(4):
            v = g.standard_normal((3, 3000)).astype(np.float32)
            dv.copy_(torch.from_numpy(v).cuda())
            R.rsr_matvec(d.handle, dv, eager, 3, torch.cuda.current_stream().cuda_stream)
            torch.cuda.synchronize()
            out.fill_(float("nan"))
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(out, eager), f"replay {rep} differs from the eager product"
            assert_f32_close(out.cpu().numpy(), dense.matvec_f32(A, v), v)


def test_several_products_in_one_launch_equal_separate_launches():
    """rsr_matvec_multi: products of different shapes (and kinds) share one launch; every result is
    bit-identical to the product's own launch, and the oracle agrees."""
    import torch

    g = rng(71)
    shapes = [(700, 333, 9, "ternary"), (2560, 500, 10, "ternary"), (64, 2000, 4, "binary"), (5000, 40, 6, "ternary")]
    mats = [(g.integers(0, 2, size=(r, c)) if kind == "binary" else g.integers(-1, 2, size=(r, c))).astype(np.int8)
            for r, c, k, kind in shapes]
    hs = [R.rsr_preprocess(A, k) for A, (_, _, k, _) in zip(mats, shapes)]
    st = torch.cuda.current_stream().cuda_stream
    try:
        for batch in (1, 5):
            note(f"multi launch of {len(hs)} products, batch {batch}")
            vfs = [g.standard_normal((batch, A.shape[0])).astype(np.float32) for A in mats]
            dv = [torch.from_numpy(v).cuda() for v in vfs]
            single = [torch.full((batch, A.shape[1]), float("nan"), dtype=torch.float32, device="cuda") for A in mats]
            multi = [torch.full((batch, A.shape[1]), float("nan"), dtype=torch.float32, device="cuda") for A in mats]
            for h, v, o in zip(hs, dv, single):
                R.rsr_matvec(h, v, o, batch, st)
            R.rsr_matvec_multi(list(zip(hs, dv, multi)), batch, st)
            torch.cuda.synchronize()
            for A, v, a, b in zip(mats, vfs, single, multi):
                assert torch.equal(a, b)
                assert_f32_close(b.cpu().numpy(), dense.matvec_f32(A, v), v)
            v8s = [g.integers(-127, 128, size=(batch, A.shape[0]), dtype=np.int8) for A in mats]
            d8 = [torch.from_numpy(v).cuda() for v in v8s]
            o8 = [torch.full((batch, A.shape[1]), -7, dtype=torch.int32, device="cuda") for A in mats]
            R.rsr_matvec_multi_i8(list(zip(hs, d8, o8)), batch, st)
            torch.cuda.synchronize()
            for A, v, o in zip(mats, v8s, o8):
                assert np.array_equal(o.cpu().numpy().astype(np.int64), dense.matvec_i8(A, v))
        with pytest.raises(R.RsrError):
            R.rsr_matvec_multi([(hs[0], dv[0], multi[0])] * 9, 1, st)   # more than 8 products
        with pytest.raises(R.RsrError):
            R.rsr_matvec_multi([(hs[0], None, multi[0])], 1, st)
    finally:
        torch.cuda.synchronize()
        for h in hs:
            R.rsr_destroy(h)


def test_llm_block_stages_one_index_per_stage_every_output_slice():
    """Configuration 4 as the four stages of a decode step: q/k/v and gate/up are one index each (their
    columns side by side).  Every slice of every stage's output is checked against the oracle's product
    of the slice's own matrix, at batch 1 and 16, from separate launches and from one captured graph."""
    import torch

    stages = workloads.llm_block_stages()
    st = torch.cuda.current_stream().cuda_stream
    hs = []
    try:
        mats = [workloads.stage_matrix(members) for _, members in stages]
        hs = [R.rsr_preprocess(A, members[0].k) for A, (_, members) in zip(mats, stages)]
        for batch in (1, 16):
            note(f"llm block stages, batch {batch}")
            vs = [members[0].activations(batch, "f32") for _, members in stages]
            dv = [torch.from_numpy(v).cuda() for v in vs]
            outs = [torch.full((batch, A.shape[1]), float("nan"), dtype=torch.float32, device="cuda") for A in mats]
            for h, v, o in zip(hs, dv, outs):
                R.rsr_matvec(h, v, o, batch, st)
            torch.cuda.synchronize()
            for (name, members), v, o in zip(stages, vs, outs):
                got = o.cpu().numpy()
                c0 = 0
                for w in members:
                    A = w.matrix()
                    assert_f32_close(got[:, c0 : c0 + w.cols], dense.matvec_f32(A, v, threads=dense.host_threads()), v)
                    c0 += w.cols
                assert c0 == got.shape[1]
            # the four launches as one graph, replayed: same bits
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            gouts = [torch.zeros_like(o) for o in outs]
            with torch.cuda.stream(side):
                for h, v, o in zip(hs, dv, gouts):
                    R.rsr_matvec(h, v, o, batch, side.cuda_stream)
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                for h, v, o in zip(hs, dv, gouts):
                    R.rsr_matvec(h, v, o, batch, torch.cuda.current_stream().cuda_stream)
            for rep in range(3):
                for o in gouts:
                    o.fill_(float("nan"))
                torch.cuda.synchronize()
                graph.replay()
                torch.cuda.synchronize()
                for a, b in zip(outs, gouts):
                    assert torch.equal(a, b), f"graph replay {rep} differs"
    finally:
        torch.cuda.synchronize()
        for h in hs:
            R.rsr_destroy(h)


def test_plain_step2_gives_the_same_product_as_the_fold():
    """Step 2 of Algorithm 2 as printed (the plain product with Bin_[k]) against the RSR++ fold of Algorithm 3:
    the same product from the same index; int8 bit for bit."""
    g = rng(73)
    for rows, cols, k, kind in [(3000, 200, 11, "ternary"), (700, 26, 13, "ternary"), (300, 64, 8, "binary"), (50, 37, 3, "ternary")]:
        A = (g.integers(0, 2, size=(rows, cols)) if kind == "binary" else g.integers(-1, 2, size=(rows, cols))).astype(np.int8)
        note(f"plain step 2: {rows}x{cols} k={k}")
        with DeviceIndex(A, k) as d:
            v8 = g.integers(-127, 128, size=(2, rows), dtype=np.int8)
            vf = g.standard_normal((2, rows)).astype(np.float32)
            fold8, foldf = d.matvec(v8), d.matvec(vf)
            R.rsr_set_step2(d.handle, R.RSR_STEP2_PLAIN)
            plain8, plainf = d.matvec(v8), d.matvec(vf)
            R.rsr_set_step2(d.handle, R.RSR_STEP2_FOLD)
            assert np.array_equal(plain8, fold8) and np.array_equal(plain8.astype(np.int64), dense.matvec_i8(A, v8))
            assert_f32_close(plainf, dense.matvec_f32(A, vf), vf)
            assert np.array_equal(d.matvec(vf), foldf)
            with pytest.raises(R.RsrError):
                R.rsr_set_step2(d.handle, 7)


def test_autotuned_k_is_never_worse_than_a_fixed_k():
    """The empirical block width (Section 4.3's optimal k, chosen by measurement as in Appendix F.1): the k it
    returns is the fastest of the range it timed, so in particular not slower than the configuration's fixed k."""
    w = workloads.get("ternary_4k")
    A = w.matrix()[:, :1500].copy()
    note("autotune k on ternary 4096x1500")
    best, us = R.rsr_autotune_k(A, 1, 7, 13, reps=60, cold=False)
    note(f"  us per product by k: { {k: round(x, 2) for k, x in us.items()} } -> best k = {best}")
    assert 7 <= best <= 13 and us[best] == min(us.values())
    assert us[best] <= us[w.k]
    assert all(x > 0 for x in us.values())
    assert R.rsr_model_k(4096, 1, 16) == 9 and R.rsr_model_k(16384, 1, 16) == 11  # argmin of (n + 2^k) / k
    with DeviceIndex(A, best) as d:  # and the product at that k is the product
        vf = w.activations(1, "f32")
        assert_f32_close(d.matvec(vf), dense.matvec_f32(A, vf), vf)


def test_dense_bit_packed_comparator_against_the_oracle():
    """The comparator of include/rsr_dense.h (bit-packed matrix, table of sums per four rows) gives the same
    product: int8 exact, float within the bound; ragged row and column counts, batches, both kinds."""
    import torch

    g = rng(79)
    st = torch.cuda.current_stream().cuda_stream
    for rows, cols, kind in [(1, 1, "binary"), (37, 300, "ternary"), (2048, 256, "binary"), (2049, 257, "ternary"),
                             (5000, 1000, "ternary"), (16384, 700, "binary")]:
        A = (g.integers(0, 2, size=(rows, cols)) if kind == "binary" else g.integers(-1, 2, size=(rows, cols))).astype(np.int8)
        note(f"dense comparator {rows}x{cols} {kind}")
        h = R.rsr_dense_preprocess(A)
        try:
            planes = 2 if kind == "ternary" else 1
            assert R.rsr_dense_table_bytes(h) == planes * -(-rows // 32) * (-(-cols // 64) * 64) * 4
            for batch in (1, 3, 16):
                vf = g.standard_normal((batch, rows)).astype(np.float32)
                of = torch.full((batch, cols), float("nan"), dtype=torch.float32, device="cuda")
                R.rsr_dense_matvec(h, torch.from_numpy(vf).cuda(), of, batch, st)
                v8 = g.integers(-128, 128, size=(batch, rows), dtype=np.int8)
                o8 = torch.full((batch, cols), -7, dtype=torch.int32, device="cuda")
                R.rsr_dense_matvec_i8(h, torch.from_numpy(v8).cuda(), o8, batch, st)
                torch.cuda.synchronize()
                assert_f32_close(of.cpu().numpy(), dense.matvec_f32(A, vf), vf)
                assert np.array_equal(o8.cpu().numpy().astype(np.int64), dense.matvec_i8(A, v8))
            with pytest.raises(R.RsrError):
                R.rsr_dense_matvec(h, of, of, 17, st)
        finally:
            torch.cuda.synchronize()
            R.rsr_dense_destroy(h)
    with pytest.raises(R.RsrError):
        R.rsr_dense_preprocess(np.full((2, 2), 3, np.int8))


class DeviceBuiltIndex(DeviceIndex):
    """An index built by rsr_preprocess_device from a matrix uploaded with torch."""

    def __init__(self, A, k):
        import time
        import torch

        dA = torch.from_numpy(np.ascontiguousarray(A)).cuda()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        self.handle = R.rsr_preprocess_device(dA, A.shape[0], A.shape[1], k)
        self.seconds = time.perf_counter() - t0
        self.info = R.rsr_info(self.handle)


DEVICE_PREP = [
    (6, 6, 2, "binary"), (50, 37, 3, "ternary"), (300, 64, 8, "binary"), (257, 100, 10, "ternary"), (1024, 48, 12, "binary"),
    (700, 26, 13, "ternary"), (100, 33, 16, "ternary"), (40, 7, 1, "ternary"), (2000, 20, 5, "binary"), (40000, 7, 3, "ternary"),
    (4000, 6, 3, "binary"), (3000, 24, 6, "zeros"), (5000, 40, 10, "skewed"),
]


# ---- seeded random cases: shapes, k, value laws, batch sizes drawn at random ------------------------------
def test_random_cases_against_the_oracle():
    """40 seeded cases over odd shapes (1 .. 20000 rows, 1 .. 4000 columns), every k, five value laws (dense
    binary of random density, uniform ternary, rows copied from a few prototypes, 2 % non-zeros, all ones)
    and batch sizes 1 .. 33; both activation types, host- and device-built index alternating."""
    import torch

    g = rng(20241106)
    st = torch.cuda.current_stream().cuda_stream
    for case in range(40):
        rows = int(g.choice([1, 2, 5, 31, 33, 64, 65, 127, 500, 1000, 2047, 3000, 7000, 20000]))
        cols = int(g.choice([1, 7, 64, 300, 1500, 4000]))
        k = int(g.integers(1, 17))
        kind = str(g.choice(["bin", "ter", "proto", "sparse", "ones"]))
        if kind == "bin":
            A = (g.random((rows, cols)) < g.uniform(0.05, 0.95)).astype(np.int8)
        elif kind == "ter":
            A = g.integers(-1, 2, size=(rows, cols)).astype(np.int8)
        elif kind == "proto":
            P = g.integers(-1, 2, size=(int(g.integers(1, 6)), cols)).astype(np.int8)
            A = P[g.integers(0, len(P), size=rows)].copy()
            flip = g.random(A.shape) < 0.02
            A[flip] = g.integers(-1, 2, size=int(flip.sum()))
        elif kind == "sparse":
            A = ((g.random((rows, cols)) < 0.02) * g.choice([-1, 1], size=(rows, cols))).astype(np.int8)
        else:
            A = np.ones((rows, cols), np.int8)
        batch = int(g.choice([1, 2, 5, 9, 33]))
        on_device = case % 2 == 1
        note(f"random case {case}: {kind} {rows}x{cols} k={k} batch={batch} index built on the {'device' if on_device else 'host'}")
        v8 = g.integers(-128, 128, size=(batch, rows), dtype=np.int8)
        vf = g.standard_normal((batch, rows)).astype(np.float32)
        if on_device:
            dA = torch.from_numpy(A).cuda()
            h = R.rsr_preprocess_device(dA, rows, cols, k)
        else:
            h = R.rsr_preprocess(A, k)
        try:
            o8 = torch.full((batch, cols), -7, dtype=torch.int32, device="cuda")
            of = torch.full((batch, cols), float("nan"), dtype=torch.float32, device="cuda")
            R.rsr_matvec_i8(h, torch.from_numpy(v8).cuda(), o8, batch, st)
            R.rsr_matvec(h, torch.from_numpy(vf).cuda(), of, batch, st)
            torch.cuda.synchronize()
            assert np.array_equal(o8.cpu().numpy().astype(np.int64), dense.matvec_i8(A, v8)), case
            assert_f32_close(of.cpu().numpy(), dense.matvec_f32(A, vf), vf)
        finally:
            torch.cuda.synchronize()
            R.rsr_destroy(h)


# ---- out += scale * (v . A), and matrices with q bits per entry as weighted binary planes ---------------
def test_scaled_accumulation_into_the_result():
    import torch

    g = rng(151)
    A = g.integers(-1, 2, size=(1500, 333)).astype(np.int8)
    v8 = g.integers(-128, 128, size=(3, 1500), dtype=np.int8)
    vf = g.standard_normal((3, 1500)).astype(np.float32)
    st = torch.cuda.current_stream().cuda_stream
    with DeviceIndex(A, 9) as d:
        start8 = g.integers(-1000, 1000, size=(3, 333)).astype(np.int32)
        o8 = torch.from_numpy(start8.copy()).cuda()
        R.rsr_matvec_acc_i8(d.handle, torch.from_numpy(v8).cuda(), o8, -5, 3, st)
        R.rsr_matvec_acc_i8(d.handle, torch.from_numpy(v8).cuda(), o8, 1, 3, st)
        torch.cuda.synchronize()
        assert np.array_equal(o8.cpu().numpy().astype(np.int64), start8 - 4 * dense.matvec_i8(A, v8))
        startf = g.standard_normal((3, 333)).astype(np.float32)
        of = torch.from_numpy(startf.copy()).cuda()
        R.rsr_matvec_acc(d.handle, torch.from_numpy(vf).cuda(), of, 0.375, 3, st)
        torch.cuda.synchronize()
        want = startf.astype(np.float64) + 0.375 * dense.matvec_f32(A, vf)
        assert_f32_close(of.cpu().numpy(), want, vf)   # |scale| < 1: the bound of the plain product covers it
        with pytest.raises(R.RsrError):
            R.rsr_matvec_acc(d.handle, torch.from_numpy(vf).cuda(), of, float("inf"), 3, st)


@pytest.mark.parametrize("q,rows,cols,k", [(2, 700, 130, 8), (4, 2100, 257, 10), (8, 1024, 96, 8), (3, 40000, 40, 10)])
def test_qbit_matrix_as_weighted_binary_planes(q, rows, cols, k):
    import torch

    g = rng(160 + q)
    lo, hi = -(1 << (q - 1)), (1 << (q - 1)) - 1
    A = g.integers(lo, hi + 1, size=(rows, cols)).astype(np.int8)
    A[0, 0], A[1, 0] = lo, hi
    batch = 2
    v8 = g.integers(-128, 128, size=(batch, rows), dtype=np.int8)
    vf = g.standard_normal((batch, rows)).astype(np.float32)
    st = torch.cuda.current_stream().cuda_stream
    note(f"q-bit q={q} {rows}x{cols} k={k}")
    h = R.rsr_qbit_preprocess(A, k, q)
    try:
        assert R.rsr_qbit_planes(h) == q and R.rsr_qbit_table_bytes(h) > 0
        o8 = torch.full((batch, cols), -7, dtype=torch.int32, device="cuda")
        R.rsr_qbit_matvec_i8(h, torch.from_numpy(v8).cuda(), o8, batch, st)
        of = torch.full((batch, cols), float("nan"), dtype=torch.float32, device="cuda")
        R.rsr_qbit_matvec(h, torch.from_numpy(vf).cuda(), of, batch, st)
        torch.cuda.synchronize()
        assert np.array_equal(o8.cpu().numpy().astype(np.int64), dense.matvec_i8(A, v8, qbits=q))
        # q planes, each within 1e-5 * sum|v| of its exact product, weights 2^i: together below 2^q * 1e-5 * sum|v|;
        # the stated bound is half of that
        assert_f32_close(of.cpu().numpy(), dense.matvec_f32(A, vf, qbits=q), vf, rel=1e-5 * (1 << (q - 1)))
    finally:
        torch.cuda.synchronize()
        R.rsr_qbit_destroy(h)
    with pytest.raises(R.RsrError):
        R.rsr_qbit_preprocess(np.full((4, 4), 2, np.int8), 2, 2)   # 2 does not fit in 2 bits
    with pytest.raises(R.RsrError):
        R.rsr_qbit_preprocess(A, k, 9)


@pytest.mark.parametrize("rows,cols,k,kind", DEVICE_PREP)
def test_device_side_preprocess_builds_the_same_index(rows, cols, k, kind):
    """Algorithm 1 on the GPU: the tables exported from the device-built index are the paper's sigma and L
    (the oracle's, entry by entry), and its products are those of the host-built index."""
    g = rng(rows * 11 + cols * 5 + k)
    if kind == "binary":
        A = g.integers(0, 2, size=(rows, cols)).astype(np.int8)
    elif kind == "zeros":
        A = np.zeros((rows, cols), np.int8)
    elif kind == "skewed":
        A = g.choice(np.array([-1, 0, 1], np.int8), size=(rows, cols), p=[0.15, 0.7, 0.15])
    else:
        A = g.integers(-1, 2, size=(rows, cols)).astype(np.int8)
    note(f"device preprocess {rows}x{cols} k={k} {kind}")
    parts = steps.ternary_split(A) if (A < 0).any() else (A,)
    with DeviceBuiltIndex(A, k) as d, DeviceIndex(A, k) as hst:
        assert d.info.parts == len(parts) == hst.info.parts and d.info.nblocks == hst.info.nblocks
        assert d.info.stored_rows == hst.info.stored_rows and d.info.row_tiles == hst.info.row_tiles
        for p_, Bp in enumerate(parts):
            for b, Bi in enumerate(steps.column_blocks(Bp, k)):
                if rows * (1 << Bi.shape[1]) > 40_000_000:
                    continue  # (the oracle's L counts rows per value one by one)
                sigma, L = R.rsr_export_block(d.handle, p_, b)
                assert np.array_equal(sigma, steps.binary_row_order(Bi)), (p_, b)
                assert np.array_equal(L[:-1], steps.full_segmentation(Bi)) and L[-1] == rows
                s2, L2 = R.rsr_export_block(hst.handle, p_, b)
                assert np.array_equal(sigma, s2) and np.array_equal(L, L2)
        for batch in (1, 3):
            v8 = g.integers(-127, 128, size=(batch, rows), dtype=np.int8)
            assert np.array_equal(d.matvec(v8).astype(np.int64), dense.matvec_i8(A, v8))
            vf = g.standard_normal((batch, rows)).astype(np.float32)
            assert_f32_close(d.matvec(vf), dense.matvec_f32(A, vf), vf)


def test_device_side_preprocess_at_the_benchmark_configurations():
    """Configurations 1 to 3 indexed on the device: product parity at full size, and the time Algorithm 1
    takes on the GPU next to the host packer's."""
    import time

    for name in ("binary_1k", "ternary_4k", "binary_16k"):
        w = workloads.get(name)
        A = w.matrix()
        t0 = time.perf_counter()
        hx = R.rsr_host_pack(A, w.k)
        host_s = time.perf_counter() - t0
        R.rsr_host_free(hx)
        with DeviceBuiltIndex(A, w.k) as d:
            note(f"preprocess {name}: device {d.seconds * 1e3:.1f} ms, host packer {host_s * 1e3:.1f} ms; "
                 f"device-built tables {d.info.table_bytes / 1e6:.2f} MB")
            v8 = w.activations(1, "i8")
            assert np.array_equal(d.matvec(v8).astype(np.int64), dense.matvec_i8(A, v8, threads=dense.host_threads()))
            vf = w.activations(2, "f32")
            assert_f32_close(d.matvec(vf), dense.matvec_f32(A, vf, threads=dense.host_threads()), vf)
            sigma, L = R.rsr_export_block(d.handle, 0, 3)
            Bi = steps.column_blocks(steps.ternary_split(A)[0] if (A < 0).any() else A, w.k)[3]
            assert np.array_equal(sigma, steps.binary_row_order(Bi))


def test_unaligned_activation_pointer_and_odd_row_count():
    import torch

    g = rng(59)
    rows, cols, k = 1001, 90, 8
    A = g.integers(-1, 2, size=(rows, cols)).astype(np.int8)
    with DeviceIndex(A, k) as d:
        vf = g.standard_normal((3, rows)).astype(np.float32)  # lanes 1, 2 start at a non-16-byte offset
        assert_f32_close(d.matvec(vf), dense.matvec_f32(A, vf), vf)
        v8 = g.integers(-127, 128, size=(3, rows), dtype=np.int8)
        assert np.array_equal(d.matvec(v8).astype(np.int64), dense.matvec_i8(A, v8))
        # a base pointer that is itself only 4-byte aligned
        buf = torch.zeros(rows + 1, dtype=torch.float32, device="cuda")
        buf[1:] = torch.from_numpy(vf[0]).cuda()
        out = torch.empty(cols, dtype=torch.float32, device="cuda")
        R.rsr_matvec(d.handle, buf[1:], out, 1, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        assert_f32_close(out.cpu().numpy(), dense.matvec_f32(A, vf[0]), vf[0])


def test_more_than_32768_rows_two_row_tiles_float_and_int8():
    """Matrices above 32768 rows are indexed in two row tiles (one launch each, results add up): the float
    path serves every row count the index accepts, and the exported tables are those of the whole matrix."""
    g = rng(67)
    for rows, cols, k in [(41000, 24, 4), (60000, 33, 11), (65534, 5, 5)]:
        A = g.integers(-1, 2, size=(rows, cols)).astype(np.int8)
        note(f"row tiles {rows}x{cols} k={k}")
        with DeviceIndex(A, k) as d:
            assert d.info.row_tiles == 2
            for batch in (1, 3):
                vf = g.standard_normal((batch, rows)).astype(np.float32)
                assert_f32_close(d.matvec(vf), dense.matvec_f32(A, vf), vf)
                v8 = g.integers(-127, 128, size=(batch, rows), dtype=np.int8)
                assert np.array_equal(d.matvec(v8).astype(np.int64), dense.matvec_i8(A, v8))
            if cols < 10:
                for p_, Bp in enumerate(steps.ternary_split(A)):
                    sigma, L = R.rsr_export_block(d.handle, p_, 0)
                    Bi = steps.column_blocks(Bp, k)[0]
                    assert np.array_equal(sigma, steps.binary_row_order(Bi))
                    assert np.array_equal(L[:-1], steps.full_segmentation(Bi))


def test_errors_from_the_device_entry_points():
    import torch

    A = np.zeros((300, 8), np.int8)
    A[::2] = 1
    with DeviceIndex(A, 4) as d:
        v = torch.zeros(300, dtype=torch.float32, device="cuda")
        out = torch.zeros(8, dtype=torch.float32, device="cuda")
        with pytest.raises(R.RsrError):
            R.rsr_matvec(d.handle, v, out, 0, None)
        with pytest.raises(R.RsrError):
            R.rsr_matvec(d.handle, None, out, 1, None)
        with pytest.raises(R.RsrError):
            R.rsr_matvec(d.handle, v, out, 70000, None)
        with pytest.raises(R.RsrError):
            R.rsr_matvec_i8(d.handle, v, None, 1, None)


# ---- the big configurations, in full ----------------------------------------------------------------------
def test_config3_binary_16k_f32_and_int8_batches():
    w = workloads.get("binary_16k")
    A = w.matrix()
    note(f"config3 {A.shape} k={w.k}")
    with DeviceIndex(A, w.k) as d:
        assert d.info.nblocks == 1366 and d.info.last_block_width == 4 and d.info.parts == 1
        for batch in (1, 8):
            vf = w.activations(batch, "f32")
            worst = assert_f32_close(d.matvec(vf), dense.matvec_f32(A, vf, threads=dense.host_threads()), vf)
            note(f"  f32 batch {batch}: worst error / bound = {worst:.3g}")
            v8 = w.activations(batch, "i8")
            assert np.array_equal(d.matvec(v8).astype(np.int64), dense.matvec_i8(A, v8, threads=dense.host_threads()))


@pytest.mark.parametrize("idx", range(7))
def test_config4_llm_block_matrices(idx):
    w = workloads.CONFIGS[4][idx]
    A = w.matrix()
    note(f"config4 {w.name} {A.shape} k={w.k}")
    with DeviceIndex(A, w.k) as d:
        assert d.info.parts == 2
        for batch in (1, 16):
            vf = w.activations(batch, "f32")
            assert_f32_close(d.matvec(vf), dense.matvec_f32(A, vf, threads=dense.host_threads()), vf)


def test_config5_correlated_ternary_32k_batch4():
    w = workloads.get("ternary_32k_correlated")
    A = w.matrix()
    note(f"config5 {A.shape} k={w.k}")
    with DeviceIndex(A, w.k) as d:
        assert d.info.nblocks == 2521 and d.info.last_block_width == 8 and d.info.parts == 2
        vf = w.activations(4, "f32")
        worst = assert_f32_close(d.matvec(vf), dense.matvec_f32(A, vf, threads=dense.host_threads()), vf)
        note(f"  worst error / bound = {worst:.3g}")
