"""The band schedule format on the CPU: streams built by the Python model, multiplied by the
model's executor (which follows the kernel's steps and sees nothing but the streams), against
the oracle."""
import numpy as np
import pytest

from oracle import gcoo_oracle as orc
from paper_2005_14469_amd import workloads
from tests import band_model


@pytest.mark.parametrize("m,k,N,p,s", [
    (100, 300, 8, 32, 0.9), (257, 1000, 4, 32, 0.99), (70, 200, 4, 16, 0.3), (64, 64, 4, 32, 0.0), (33, 50, 4, 8, 0.95),
    (300, 70, 4, 32, 0.6), (1, 1, 1, 1, 0.0), (20, 130, 2, 32, 1.0),
    (300, 500, 4, 16, 0.5), (257, 1000, 4, 16, 0.99), (120, 90, 4, 17, 0.7), (530, 200, 4, 12, 0.8),
])
def test_streams_multiply_like_the_oracle(m, k, N, p, s):
    w = workloads.uniform_random(m, k, N, s, seed=m + k)
    G = orc.gcoo_from_csr(w.m, w.k, w.row_ptr, w.col_idx, w.vals, p)
    streams, info = band_model.build(m, k, p, G.gIdxes, G.rows, G.cols, G.values)
    C = band_model.execute(m, k, p, N, streams, info, w.B)
    C64, D64 = orc.spdm_csr(w.k, N, w.row_ptr, w.col_idx, w.vals, w.B)
    assert np.abs(C - C64).max() <= 1e-12 * max(D64.max(), 1.0)
    # space: a stream fits the closed-form bound the device layout relies on
    for q, st in enumerate(streams):
        nnz_q = int(G.gIdxes[q + 1] - G.gIdxes[q]) if q < G.g else 0
        assert len(st) <= 3 * nnz_q + 56 * ((k + 63) // 64 + 2)
        assert len(st) % 4 == 0


def test_pieces_of_run_cover_the_run():
    for ell in range(1, 300):
        pcs = band_model.pieces_of_run(ell)
        assert sum(t for _, t in pcs) == ell and all(t in (1, 2, 4, 8) for _, t in pcs)
        assert [x for x, _ in pcs] == list(np.cumsum([0] + [t for _, t in pcs])[:-1])


def repeated_coordinates_workload():
    """A CSR input whose rows repeat one coordinate many times: runs far longer than a group is tall."""
    rng = np.random.default_rng(11)
    m, k, N = 40, 90, 3
    rows = []
    for i in range(m):
        cols_i = list(rng.choice(k, 5, replace=False))
        if i % 7 == 0:
            cols_i += [17] * 45 + [18] * 70            # the same coordinate again and again
        rows.append(np.array(cols_i, np.int32))
    row_ptr = np.concatenate([[0], np.cumsum([len(r) for r in rows])]).astype(np.int32)
    col_idx = np.concatenate(rows).astype(np.int32)
    vals = rng.standard_normal(len(col_idx)).astype(np.float32)
    B = rng.standard_normal((k, N)).astype(np.float32)
    return m, k, N, row_ptr, col_idx, vals, B


@pytest.mark.parametrize("p", [1, 8, 16, 32])
def test_runs_longer_than_a_group_is_tall(p):
    m, k, N, row_ptr, col_idx, vals, B = repeated_coordinates_workload()
    G = orc.gcoo_from_csr(m, k, row_ptr, col_idx, vals, p)
    streams, info = band_model.build(m, k, p, G.gIdxes, G.rows, G.cols, G.values)
    C = band_model.execute(m, k, p, N, streams, info, B)
    C64, D64 = orc.spdm_csr(k, N, row_ptr, col_idx, vals, B)
    assert np.abs(C - C64).max() <= 1e-12 * max(D64.max(), 1.0)
    for q, st in enumerate(streams):
        nnz_q = int(G.gIdxes[q + 1] - G.gIdxes[q]) if q < G.g else 0
        assert len(st) <= 3 * nnz_q + 56 * ((k + 63) // 64 + 2)
