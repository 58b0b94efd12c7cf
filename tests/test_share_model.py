"""The share schedule on the CPU: built by the Python model, multiplied by the model's executor (which
follows the kernel's steps and sees nothing but the schedule), against the oracle."""
import numpy as np
import pytest

from oracle import gcoo_oracle as orc
from paper_2005_14469_amd import workloads
from tests import share_model


@pytest.mark.parametrize("m,k,N,p,s", [
    (100, 300, 8, 32, 0.9), (257, 1000, 4, 42, 0.99), (70, 200, 4, 16, 0.3), (64, 64, 4, 48, 0.0), (33, 50, 4, 8, 0.95),
    (300, 70, 4, 32, 0.6), (1, 1, 1, 1, 0.0), (20, 130, 2, 32, 1.0), (700, 500, 4, 48, 0.5), (530, 200, 4, 12, 0.8),
])
def test_schedule_multiplies_like_the_oracle(m, k, N, p, s):
    w = workloads.uniform_random(m, k, N, s, seed=m + k)
    G = orc.gcoo_from_csr(w.m, w.k, w.row_ptr, w.col_idx, w.vals, p)
    info, streams = share_model.build(m, k, p, G.gIdxes, G.rows, G.cols, G.values)
    C = share_model.execute(m, k, p, N, info, streams, w.B)
    C64, D64 = orc.spdm_csr(w.k, N, w.row_ptr, w.col_idx, w.vals, w.B)
    assert np.abs(C - C64).max() <= 1e-12 * max(D64.max(), 1.0)
    # every entry is listed exactly once, and the blocks fit the bound the device layout relies on
    listed = sum(int(((b[:, :, 1] != share_model.SINK)).sum()) for bands in streams for (_, _, b) in bands)
    assert listed == G.nnz
    g = (m + p - 1) // p
    blocks = sum(len(b) for bands in streams for (_, _, b) in bands)
    pairs = min(G.nnz, ((g + 7) // 8) * 8 * ((k + 63) // 64))
    assert blocks <= G.nnz // 16 + 2 * pairs


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


@pytest.mark.parametrize("p", [1, 8, 16, 48])
def test_runs_longer_than_a_group_is_tall(p):
    m, k, N, row_ptr, col_idx, vals, B = repeated_coordinates_workload()
    G = orc.gcoo_from_csr(m, k, row_ptr, col_idx, vals, p)
    info, streams = share_model.build(m, k, p, G.gIdxes, G.rows, G.cols, G.values)
    C = share_model.execute(m, k, p, N, info, streams, B)
    C64, D64 = orc.spdm_csr(k, N, row_ptr, col_idx, vals, B)
    assert np.abs(C - C64).max() <= 1e-12 * max(D64.max(), 1.0)


def test_stretches_cover_a_band():
    cols = np.array([3] * 70 + [5] + [9] * 4 + [11] * 33)
    st = share_model.stretches(cols)
    assert st == [(0, 32), (32, 64), (64, 70), (70, 71), (71, 75), (75, 107), (107, 108)]
