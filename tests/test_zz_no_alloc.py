"""The entry point that allocates nothing (rsr_dense_matvec_static, include/rsr_dense.h): called through the
C ABI, its output must equal that of the entry point it is a variant of (rsr_dense_matvec) bit for bit -
same kernels, same order of additions, only the buffer of partial sums differs - on two calls in a row,
the second with a smaller input (the shared static buffer then still holds the first call's partial sums,
which must not leak into the result), and the oracle must agree with both."""
import numpy as np
import pytest

import paper_2411_06360_amd as R
from oracle import dense
from tests.gpu_util import assert_f32_close

pytestmark = pytest.mark.gpu


def run_both(A, v):
    import torch

    batch = v.shape[0]
    st = torch.cuda.current_stream().cuda_stream
    h = R.rsr_dense_preprocess(A)
    try:
        dv = torch.from_numpy(v).cuda()
        ref = torch.full((batch, A.shape[1]), float("nan"), dtype=torch.float32, device="cuda")
        got = torch.full((batch, A.shape[1]), float("nan"), dtype=torch.float32, device="cuda")
        R.rsr_dense_matvec(h, dv, ref, batch, st)
        R.rsr_dense_matvec_static(h, dv, got, batch, st)
        torch.cuda.synchronize()
        return ref.cpu().numpy(), got.cpu().numpy()
    finally:
        torch.cuda.synchronize()
        R.rsr_dense_destroy(h)


def test_static_buffer_entry_point_equals_the_allocating_one_twice_in_a_row():
    import torch

    g = np.random.default_rng(83)
    print("no-alloc entry point: 5000x3000 ternary batch 3, then 700x129 binary batch 1", flush=True)
    A1 = g.integers(-1, 2, size=(5000, 3000)).astype(np.int8)
    v1 = g.standard_normal((3, 5000)).astype(np.float32)
    ref1, got1 = run_both(A1, v1)
    assert np.array_equal(ref1, got1)
    assert_f32_close(got1, dense.matvec_f32(A1, v1), v1)
    A2 = g.integers(0, 2, size=(700, 129)).astype(np.int8)   # smaller: fewer tiles, fewer columns, one vector
    v2 = g.standard_normal((1, 700)).astype(np.float32)
    ref2, got2 = run_both(A2, v2)
    assert np.array_equal(ref2, got2)
    assert_f32_close(got2, dense.matvec_f32(A2, v2), v2)
    # sizes beyond the static buffer are refused with a clear message, and nothing is launched
    A3 = np.ones((512 * 9, 16384), np.int8)                  # 9 tiles x 8 vectors x 16384 columns x 4 bytes > 4 MiB
    h = R.rsr_dense_preprocess(A3)
    try:
        v3 = torch.zeros((8, A3.shape[0]), dtype=torch.float32, device="cuda")
        o3 = torch.zeros((8, 16384), dtype=torch.float32, device="cuda")
        with pytest.raises(R.RsrError) as e:
            R.rsr_dense_matvec_static(h, v3, o3, 8, None)
        assert e.value.code == -2 and "exceed" in str(e.value)
        R.rsr_dense_matvec_static(h, v3, o3, 7, None)         # 7 vectors fit exactly below the limit
        torch.cuda.synchronize()
    finally:
        torch.cuda.synchronize()
        R.rsr_dense_destroy(h)
