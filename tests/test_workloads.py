"""The seeded input generators: reproducible, exact counts, well-formed CSR."""
import numpy as np

from paper_2005_14469_amd import workloads


def _check_csr(w):
    assert w.row_ptr.dtype == np.int32 and w.col_idx.dtype == np.int32 and w.vals.dtype == np.float32
    assert w.row_ptr[0] == 0 and np.all(np.diff(w.row_ptr) >= 0) and w.row_ptr[-1] == w.col_idx.size
    assert w.col_idx.min() >= 0 and w.col_idx.max() < w.k
    for i in range(0, w.m, max(1, w.m // 50)):
        c = w.col_idx[w.row_ptr[i]:w.row_ptr[i + 1]]
        assert np.all(np.diff(c) > 0)
    assert w.B.shape == (w.k, w.N) and w.B.dtype == np.float32


def test_config0_exact_count_and_reproducible():
    a, b = workloads.config(0), workloads.config(0)
    assert a.nnz == round(0.1 * 256 * 256) == 6554
    assert np.array_equal(a.col_idx, b.col_idx) and np.array_equal(a.vals, b.vals) and np.array_equal(a.B, b.B)
    _check_csr(a)


def test_uniform_dist_range():
    w = workloads.uniform_random(64, 64, 8, 0.5, 1, dist="uniform")
    assert np.abs(w.vals).max() <= 1 and np.abs(w.B).max() <= 1 and w.vals.min() < 0
    _check_csr(w)


def test_zipf_rows_shape():
    w = workloads.zipf_rows(2048, 2048, 16, seed=3, row_max=512)
    lens = np.diff(w.row_ptr)
    assert lens.min() >= 1 and lens.max() <= 512 and np.median(lens) <= 3
    _check_csr(w)


def test_diagonal():
    w = workloads.diagonal(33, 4, 0)
    assert w.nnz == 33 and np.array_equal(w.col_idx, np.arange(33))
    _check_csr(w)
