"""The seeded input generators: shapes, value sets, laws and reproducibility (small sizes only)."""
import numpy as np

import workloads
from workloads import configs as C


def test_config_table_matches_the_benchmark_description():
    w = workloads.get("binary_1k")
    assert (w.rows, w.cols, w.k, w.kind) == (1024, 1024, 8, "binary")
    w = workloads.get("ternary_4k")
    assert (w.rows, w.cols, w.k, w.kind) == (4096, 4096, 10, "ternary")
    w = workloads.get("binary_16k")
    assert (w.rows, w.cols, w.k, w.batches, w.dtypes) == (16384, 16384, 12, (1, 8), ("f32", "i8"))
    shapes = [(x.rows, x.cols) for x in workloads.CONFIGS[4]]
    assert shapes == [(2560, 2560)] * 4 + [(2560, 6912)] * 2 + [(6912, 2560)]
    assert all(x.k == 10 and x.p_zero == 0.5 for x in workloads.CONFIGS[4])
    assert len({x.seed for x in workloads.CONFIGS[4]}) == 7
    w = workloads.get("ternary_32k_correlated")
    assert (w.rows, w.cols, w.k, w.batches) == (32768, 32768, 13, (4,))
    assert workloads.seed_for(3, 0) == 2411063630


def test_generators_are_reproducible_and_have_the_stated_laws():
    g = np.random.default_rng(5)
    B = C.binary_matrix(g, 300, 400)
    assert B.dtype == np.int8 and B.shape == (300, 400) and set(np.unique(B)) == {0, 1}
    assert abs(B.mean() - 0.5) < 0.01
    T = C.ternary_matrix(np.random.default_rng(6), 300, 400, p_zero=0.5)
    assert set(np.unique(T)) == {-1, 0, 1}
    assert abs((T == 0).mean() - 0.5) < 0.01 and abs((T == 1).mean() - 0.25) < 0.01
    T2 = C.ternary_matrix(np.random.default_rng(6), 300, 400, p_zero=0.5)
    assert np.array_equal(T, T2)
    K = C.correlated_ternary_matrix(np.random.default_rng(7), 2000, 130, p_zero=0.6, n_prototypes=8, p_resample=0.05)
    assert set(np.unique(K)) <= {-1, 0, 1} and abs((K == 0).mean() - 0.6) < 0.05
    # rows cluster around few prototypes: far fewer distinct 13-column patterns than rows
    pats = {bytes(r) for r in K[:, :13]}
    assert len(pats) < 700


def test_activations():
    w = workloads.get("binary_1k")
    v = w.activations(1, "i8")
    assert v.dtype == np.int8 and v.shape == (1, 1024) and v.min() >= -127 and v.max() <= 127
    f = w.activations(3, "f32")
    assert f.dtype == np.float32 and f.shape == (3, 1024) and abs(float(f.std()) - 1.0) < 0.05
    assert np.array_equal(f, w.activations(3, "f32"))
    small = workloads.CONFIGS[1][0]
    A = small.matrix()
    assert A.shape == (1024, 1024) and np.array_equal(A, small.matrix())


def test_bench_refuses_more_than_one_gpu():
    """The build runs on one device: `bench.py --gpus N` with N > 1 says so and exits with an error."""
    import os
    import subprocess
    import sys

    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    proc = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                          stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, timeout=120)
    assert proc.returncode != 0 and proc.stdout.strip() == ""
    assert "one GPU" in proc.stderr
