"""Pins of the oracle's product functions: Equation 1 by brute force, closed-form special
cases, a library cross-check, invariants, and the error measure itself."""
import numpy as np
import pytest
import scipy.sparse as sp

from oracle import gcoo_oracle as orc
from paper_2005_14469_amd import workloads


def _rand(m, k, N, density, seed):
    rng = np.random.default_rng(seed)
    A = ((rng.random((m, k)) < density) * rng.standard_normal((m, k))).astype(np.float32)
    B = rng.standard_normal((k, N)).astype(np.float32)
    S = sp.csr_matrix(A)
    S.sort_indices()
    return A, B, S.indptr.astype(np.int32), S.indices.astype(np.int32), S.data.astype(np.float32)


def test_dense_gemm_hand_worked():
    """Equation 1 on a 2x3 by 3x2 product worked by hand (asymmetric, so a transposed
    operand or a swapped index cannot pass)."""
    A = np.array([[1, 2, 3], [4, 5, 6]], np.float32)
    B = np.array([[7, 8], [9, 10], [11, 12]], np.float32)
    assert orc.dense_gemm(A, B).tolist() == [[58, 64], [139, 154]]


@pytest.mark.parametrize("m", [1, 2, 5, 17])
@pytest.mark.parametrize("k", [1, 3, 8, 17])
@pytest.mark.parametrize("N", [1, 4, 9])
def test_spdm_equals_brute_force(m, k, N):
    A, B, rp, ci, va = _rand(m, k, N, 0.4, 100 * m + 10 * k + N)
    ref = orc.dense_gemm(A, B)
    # independent of the oracle: exact rational arithmetic is overkill; python floats are fp64
    py = [[sum(float(A[i, l]) * float(B[l, j]) for l in range(k)) for j in range(N)] for i in range(m)]
    assert np.allclose(ref, np.array(py), rtol=0, atol=1e-12)
    C64, D64 = orc.spdm_csr(k, N, rp, ci, va, B)
    assert np.allclose(C64, ref, rtol=0, atol=1e-12)
    assert np.allclose(D64, np.abs(A).astype(np.float64) @ np.abs(B).astype(np.float64), rtol=1e-14, atol=0)
    for p in (1, 2, 4, 8, 16, 32):
        G = orc.gcoo_from_csr(m, k, rp, ci, va, p)
        assert np.allclose(orc.spdm_gcoo(G, B, N), ref, rtol=0, atol=1e-12)


def test_library_cross_check_scipy():
    w = workloads.uniform_random(300, 200, 37, 0.9, 5)
    S = sp.csr_matrix((w.vals.astype(np.float64), w.col_idx, w.row_ptr), shape=(w.m, w.k))
    ref = S @ w.B.astype(np.float64)
    C64, D64 = orc.spdm_csr(w.k, w.N, w.row_ptr, w.col_idx, w.vals, w.B)
    assert np.max(np.abs(C64 - ref) / np.maximum(D64, 1e-300)) < 1e-14
    refD = abs(S) @ np.abs(w.B).astype(np.float64)
    assert np.allclose(D64, refD, rtol=1e-13, atol=0)


def test_row_range_is_a_slice_of_the_full_result():
    w = workloads.uniform_random(64, 50, 11, 0.8, 9)
    C64, D64 = orc.spdm_csr(w.k, w.N, w.row_ptr, w.col_idx, w.vals, w.B)
    c, d = orc.spdm_csr(w.k, w.N, w.row_ptr, w.col_idx, w.vals, w.B, 10, 23)
    assert np.array_equal(c, C64[10:23]) and np.array_equal(d, D64[10:23])


def test_leading_dimension_of_B():
    w = workloads.uniform_random(20, 30, 16, 0.7, 2)
    C64, _ = orc.spdm_csr(w.k, 5, w.row_ptr, w.col_idx, w.vals, w.B)     # first 5 columns, ldb = 16
    full, _ = orc.spdm_csr(w.k, 16, w.row_ptr, w.col_idx, w.vals, w.B)
    assert np.array_equal(C64, full[:, :5])


def test_special_cases_exact():
    rng = np.random.default_rng(1)
    n, N = 23, 7
    B = rng.standard_normal((n, N)).astype(np.float32)
    eye = sp.identity(n, dtype=np.float32, format="csr")
    C64, D64 = orc.spdm_csr(n, N, eye.indptr, eye.indices, eye.data, B)
    assert np.array_equal(C64, B.astype(np.float64))                      # A = I gives C = B
    assert np.array_equal(D64, np.abs(B).astype(np.float64))
    perm = rng.permutation(n)
    P = sp.csr_matrix((np.ones(n, np.float32), (np.arange(n), perm)), shape=(n, n))
    C64, _ = orc.spdm_csr(n, N, P.indptr, P.indices, P.data, B)
    assert np.array_equal(C64, B[perm].astype(np.float64))                # permutation of rows
    Z = sp.csr_matrix((n, n), dtype=np.float32)
    C64, D64 = orc.spdm_csr(n, N, Z.indptr, Z.indices, Z.data, B)
    assert not C64.any() and not D64.any()                                # A = 0 gives C = 0
    d = rng.standard_normal(n).astype(np.float32)
    Dg = sp.diags(d, format="csr", dtype=np.float32)
    C64, _ = orc.spdm_csr(n, N, Dg.indptr, Dg.indices, Dg.data, B)
    assert np.array_equal(C64, d.astype(np.float64)[:, None] * B.astype(np.float64))
    one = sp.csr_matrix((np.array([2.5], np.float32), ([4], [9])), shape=(n, n))
    C64, _ = orc.spdm_csr(n, N, one.indptr, one.indices, one.data, B)
    exp = np.zeros((n, N))
    exp[4] = 2.5 * B[9].astype(np.float64)
    assert np.array_equal(C64, exp)


def test_linearity_in_B():
    w = workloads.uniform_random(40, 60, 9, 0.8, 4)
    rng = np.random.default_rng(8)
    B2 = rng.standard_normal(w.B.shape).astype(np.float32)
    f = lambda B: orc.spdm_csr(w.k, w.N, w.row_ptr, w.col_idx, w.vals, B)[0]
    # B + B2 rounded to fp32 would break exactness: use a power-of-two scale and disjoint supports
    assert np.array_equal(f(w.B * np.float32(4.0)), 4.0 * f(w.B))
    Bz = w.B.copy(); Bz[::2] = 0
    B2z = B2.copy(); B2z[1::2] = 0
    assert np.allclose(f(Bz + B2z), f(Bz) + f(B2z), rtol=1e-13, atol=1e-13)


def test_structural_zeros_are_skipped_not_multiplied():
    """An Inf in a row of B that no stored entry touches must not reach C (0*Inf never formed)."""
    A = np.array([[1, 0], [0, 0]], np.float32)
    B = np.array([[2, 3], [np.inf, np.nan]], np.float32)
    S = sp.csr_matrix(A)
    C64, D64 = orc.spdm_csr(2, 2, S.indptr, S.indices, S.data, B)
    assert C64.tolist() == [[2, 3], [0, 0]] and D64.tolist() == [[2, 3], [0, 0]]


def test_max_scaled_error_measure():
    C64 = np.array([[1.0, -2.0], [0.0, 4.0]])
    D64 = np.array([[2.0, 2.0], [0.0, 8.0]])
    C = np.array([[1.0, -2.0], [0.0, 4.0]], np.float32)
    assert orc.max_scaled_error(C, C64, D64) == (0.0, 0)
    C[0, 1] = -2.5                                  # off by 0.5 where the scale is 2
    assert orc.max_scaled_error(C, C64, D64) == (0.25, 0)
    C[1, 0] = 1e-30                                 # must be exactly zero where the scale is zero
    assert orc.max_scaled_error(C, C64, D64) == (0.25, 1)
    C[1, 0] = -0.0
    C[1, 1] = np.nan
    assert orc.max_scaled_error(C, C64, D64) == (0.25, 1)


def test_fp32_reference_sits_far_inside_the_tolerance():
    """Sanity of the 1e-5 bar: a plain fp32 computation of config 0 lands near 1e-7 of the scale,
    and a single dropped entry is seen as a violation far above it."""
    w = workloads.config(0)
    C64, D64 = orc.spdm_csr(w.k, w.N, w.row_ptr, w.col_idx, w.vals, w.B)
    S = sp.csr_matrix((w.vals, w.col_idx, w.row_ptr), shape=(w.m, w.k))
    C32 = (S @ w.B).astype(np.float32)
    err, bad = orc.max_scaled_error(C32, C64, D64)
    assert bad == 0 and err < 2e-6
    v = w.vals.copy()
    v[w.nnz // 2] = 0
    S2 = sp.csr_matrix((v, w.col_idx, w.row_ptr), shape=(w.m, w.k))
    err2, _ = orc.max_scaled_error((S2 @ w.B).astype(np.float32), C64, D64)
    assert err2 > 1e-3
