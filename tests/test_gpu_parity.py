"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.

Integer work (the GCOO arrays) must be bit-identical.  The product must satisfy
max |C_gpu - C64| / (|A|.|B|) <= 1e-5 elementwise, and be exactly zero where |A|.|B| is zero.
"""
import numpy as np
import pytest
import scipy.sparse as sp

torch = pytest.importorskip("torch")

from oracle import gcoo_oracle as orc
from paper_2005_14469_amd import binding, workloads

pytestmark = pytest.mark.gpu

TOL = 1e-5
DEV = "cuda:0"


def _say(msg):
    print(msg, flush=True)


@pytest.fixture
def share_always():
    """Conversions inside the test build the share schedule whenever the workgroup-shared kernel could run."""
    binding.gcoo_set_share_policy(binding.SHARE_ALWAYS)
    yield
    binding.gcoo_set_share_policy(binding.SHARE_AUTO)


def _assert_arrays_equal(exp, G):
    assert np.array_equal(exp["rows"], G.rows)
    assert np.array_equal(exp["cols"], G.cols)
    assert np.array_equal(exp["values"].view(np.uint32), G.values.view(np.uint32))     # bit patterns
    assert np.array_equal(exp["gIdxes"], G.gIdxes.astype(np.int64))
    assert np.array_equal(exp["nnzPerGroup"], G.nnzPerGroup)


def _check_product(w, p, variant, Bt=None, r0=0, r1=None, A=None):
    """Run the GPU path on workload w and compare rows [r0, r1) with the oracle."""
    A = A or binding.gcoo_from_csr(w.m, w.k, w.row_ptr, w.col_idx, w.vals, p, device=DEV)
    Bt = Bt if Bt is not None else torch.from_numpy(w.B).to(DEV)
    Cg = torch.full((w.m, Bt.shape[1]), float("nan"), dtype=torch.float32, device=DEV)   # must be fully overwritten
    binding.gcoo_spdm(A, Bt, Cg, variant=variant)
    torch.cuda.synchronize()
    Ch = Cg.cpu().numpy()
    r1 = w.m if r1 is None else r1
    C64, D64 = orc.spdm_csr(w.k, Bt.shape[1], w.row_ptr, w.col_idx, w.vals, Bt.cpu().numpy(), r0, r1)
    err, bad = orc.max_scaled_error(Ch[r0:r1], C64, D64)
    assert bad == 0, f"{bad} elements are NaN or nonzero where the scale is zero"
    assert err <= TOL, f"scaled error {err:.3e} > {TOL}"
    return err, A, Ch


REG_MAX_P = 64


def _variants_for(p, N):
    """The kernels that serve group height p and N columns (torch tensors are 16-byte aligned)."""
    v = [binding.VARIANT_LDS]
    if (p <= 38 and N >= 4) or (p <= REG_MAX_P and N >= 2):       # four columns per lane, or two
        v += [binding.VARIANT_REG]
    if p > REG_MAX_P and N >= 4:      # groups taller than 64 rows: the register kernel runs on the copy regrouped at 32 rows
        v += [binding.VARIANT_REG]
    return v


# ------------------------------------------------------------------ conversion (bit-exact)

@pytest.mark.parametrize("p", [1, 2, 3, 8, 32, 64, 100, 256])
@pytest.mark.parametrize("shape", [(1, 1), (50, 40), (129, 300), (256, 256), (1000, 70000)])
def test_gcoo_from_csr_bit_exact(p, shape):
    m, k = shape
    if k > 60000 and p not in (8, 100):
        pytest.skip("the three-pass radix case is run for two group heights only")
    _say(f"gcoo_from_csr m={m} k={k} p={p}")
    w = workloads.uniform_random(m, k, 1, 0.9 if m * k > 100 else 0.3, seed=7 * m + p)
    G = orc.gcoo_from_csr(w.m, w.k, w.row_ptr, w.col_idx, w.vals, p)
    for on_device, known_nnz in ((False, False), (True, False), (True, True)):
        if on_device:
            args = [torch.from_numpy(x).to(DEV) for x in (w.row_ptr, w.col_idx, w.vals)]
        else:
            args = [w.row_ptr, w.col_idx, w.vals]
        A = binding.gcoo_from_csr(w.m, w.k, *args, p, device=DEV, known_nnz=known_nnz)
        assert A.info() == dict(m=m, k=k, nnz=w.nnz, p=p, g=G.g)
        _assert_arrays_equal(A.export(), G)
        A.free()


@pytest.mark.parametrize("m,k,p,s", [(256, 3000, 128, 0.8), (300, 40000, 64, 0.9), (100, 65536, 100, 0.8), (200, 257, 200, 0.1)])
def test_gcoo_from_csr_large_groups_bit_exact(m, k, p, s):
    """Groups of 6000 entries and more with 257 .. 65536 columns are sorted high digit first, bucket by bucket."""
    _say(f"gcoo_from_csr, large groups m={m} k={k} p={p}")
    w = workloads.uniform_random(m, k, 1, s, seed=m + k + p)
    assert w.nnz / ((m + p - 1) // p) >= 6000
    rng = np.random.default_rng(m)
    rp, ci, va = w.row_ptr.copy(), w.col_idx.copy(), w.vals.copy()
    for i in range(0, m, 3):                            # every third row: columns out of order, one coordinate repeated
        b, e = rp[i], rp[i + 1]
        if e - b > 2:
            perm = rng.permutation(e - b)
            ci[b:e] = ci[b:e][perm]
            va[b:e] = va[b:e][perm]
            ci[b + 1] = ci[b]
    G = orc.gcoo_from_csr(m, k, rp, ci, va, p)
    args = [torch.from_numpy(x).to(DEV) for x in (rp, ci, va)]
    A = binding.gcoo_from_csr(m, k, *args, p, device=DEV, known_nnz=True)
    _assert_arrays_equal(A.export(), G)
    A.free()


def test_gcoo_from_csr_unsorted_repeated_and_explicit_zero_entries():
    _say("gcoo_from_csr unsorted/duplicate input")
    rng = np.random.default_rng(5)
    m, k, p = 70, 33, 16
    w = workloads.uniform_random(m, k, 1, 0.6, seed=3)
    rp, ci, va = w.row_ptr.copy(), w.col_idx.copy(), w.vals.copy()
    for i in range(m):
        s, e = rp[i], rp[i + 1]
        if e - s > 2:
            perm = rng.permutation(e - s)
            ci[s:e] = ci[s:e][perm]
            va[s:e] = va[s:e][perm]
            ci[s + 1] = ci[s]                       # repeated coordinate, order of input must survive
    va[::9] = 0.0
    va[4::9] = -0.0
    va[5::31] = np.nan
    G = orc.gcoo_from_csr(m, k, rp, ci, va, p)
    A = binding.gcoo_from_csr(m, k, rp, ci, va, p, device=DEV)
    _assert_arrays_equal(A.export(), G)


def test_gcoo_empty_shapes():
    _say("gcoo_from_csr empty shapes")
    for m, k in [(0, 5), (5, 3), (5, 0)]:
        rp = np.zeros(m + 1, np.int32)
        A = binding.gcoo_from_csr(m, k, rp, np.zeros(0, np.int32), np.zeros(0, np.float32), 2, device=DEV)
        G = orc.gcoo_from_csr(m, k, rp, np.zeros(0, np.int32), np.zeros(0, np.float32), 2)
        _assert_arrays_equal(A.export(), G)
        if k > 0:
            B = torch.randn(k, 8, device=DEV)
            C = binding.gcoo_spdm(A, B)
            torch.cuda.synchronize()
            assert C.shape == (m, 8) and not C.any()


@pytest.mark.parametrize("p", [1, 4, 32, 50, 128, 256])
@pytest.mark.parametrize("shape", [(1, 1), (37, 29), (256, 256), (300, 1111), (2000, 3001)])
def test_gcoo_from_dense_bit_exact(p, shape):
    m, k = shape
    _say(f"gcoo_from_dense m={m} k={k} p={p}")
    rng = np.random.default_rng(m + k + p)
    Ah = ((rng.random((m, k)) < 0.2) * rng.standard_normal((m, k))).astype(np.float32)
    Ah[0, 0] = -0.0                                   # dropped
    if m > 1:
        Ah[1, k - 1] = np.nan                         # kept
    G = orc.gcoo_from_dense(Ah, p)
    Ad = torch.from_numpy(Ah).to(DEV)
    assert binding.gcoo_dense_nnz(Ad) == G.nnz
    A = binding.gcoo_from_dense(Ad, p)
    assert A.info()["nnz"] == G.nnz
    _assert_arrays_equal(A.export(), G)
    # a view with a leading dimension larger than k
    big = torch.zeros((m, k + 5), dtype=torch.float32, device=DEV)
    big[:, :k] = Ad
    A2 = binding.gcoo_from_dense(big[:, :k], p)
    _assert_arrays_equal(A2.export(), G)


# ------------------------------------------------------------------ product

@pytest.mark.parametrize("p", [1, 2, 8, 16, 32, 33, 38, 39, 64, 128, 256])
def test_config0_all_variants(p):
    w = workloads.config(0)
    for variant in _variants_for(p, w.N):
        _say(f"config0 p={p} variant={variant}")
        err, _, _ = _check_product(w, p, variant)
        assert err < 2e-6          # rounding alone sits near 1e-7; more means a lost or misplaced entry


@pytest.mark.parametrize("m,k,N,p", [
    (1, 1, 1, 1), (5, 7, 3, 2), (33, 65, 64, 32), (100, 90, 260, 32), (129, 257, 516, 64),
    (300, 200, 1028, 16), (77, 500, 250, 128), (64, 64, 4, 8), (130, 40, 1000, 20), (513, 100, 768, 32),
    (400, 300, 516, 38), (77, 90, 260, 36), (1000, 2000, 256, 38),
    # N not a multiple of the columns per lane: the lane at the end of a row computes the last columns instead
    (100, 90, 261, 32), (300, 200, 1027, 16), (400, 300, 517, 38), (129, 257, 515, 64), (64, 64, 5, 8), (50, 60, 4, 32),
    (90, 70, 257, 32), (90, 70, 258, 24), (90, 70, 259, 38), (40, 30, 2, 48), (40, 30, 3, 64), (70, 50, 7, 3), (300, 300, 769, 40),
])
def test_ragged_shapes_all_variants(m, k, N, p):
    w = workloads.uniform_random(m, k, N, 0.8, seed=m * 1000 + N)
    for variant in _variants_for(p, N):
        _say(f"ragged m={m} k={k} N={N} p={p} variant={variant}")
        _check_product(w, p, variant)


def test_register_kernel_refuses_what_it_does_not_serve():
    _say("REG variant: a single column is refused, AUTO falls back to the LDS kernel")
    w = workloads.uniform_random(256, 256, 64, 0.9, seed=5)
    Bt = torch.from_numpy(w.B).to(DEV)
    for p, N in [(128, 1), (32, 1), (48, 1)]:
        A = binding.gcoo_from_csr(w.m, w.k, w.row_ptr, w.col_idx, w.vals, p, device=DEV)
        Bv = Bt[:, :N].contiguous()
        Cv = torch.empty((w.m, N), device=DEV)
        assert binding.gcoo_spdm_pick(A, Bv, Cv) == binding.VARIANT_LDS
        with pytest.raises(binding.GcooError):
            binding.gcoo_spdm(A, Bv, Cv, variant=binding.VARIANT_REG)
        torch.cuda.synchronize()


@pytest.mark.parametrize("p", [65, 100, 128, 256])
def test_groups_taller_than_64_rows_run_the_fast_kernels(p):
    """p > 64: the conversion keeps a second copy of the matrix regrouped at 32 rows and the product runs on it, through
    every route into the library; the exported arrays are those of the caller's p."""
    w = workloads.uniform_random(700, 900, 260, 0.93, seed=p)
    _say(f"tall groups p={p}: CSR from the host, CSR on the device, dense, the entry point that allocates nothing")
    G = orc.gcoo_from_csr(w.m, w.k, w.row_ptr, w.col_idx, w.vals, p)
    Bt = torch.from_numpy(w.B).to(DEV)
    dev = [torch.from_numpy(x).to(DEV) for x in (w.row_ptr, w.col_idx, w.vals)]
    Ah = np.zeros((w.m, w.k), np.float32)
    Ah[np.repeat(np.arange(w.m), np.diff(w.row_ptr)), w.col_idx] = w.vals
    handles = [binding.gcoo_from_csr(w.m, w.k, w.row_ptr, w.col_idx, w.vals, p, device=DEV),
               binding.gcoo_from_csr(w.m, w.k, *dev, p, device=DEV, known_nnz=True),
               binding.gcoo_from_csr_device_static(w.m, w.k, *dev, p),
               binding.gcoo_from_dense(torch.from_numpy(Ah).to(DEV), p)]
    C64, D64 = orc.spdm_csr(w.k, w.N, w.row_ptr, w.col_idx, w.vals, w.B)
    for A in handles:
        Cg = torch.full((w.m, w.N), float("nan"), device=DEV)
        assert binding.gcoo_spdm_pick(A, Bt, Cg) == binding.VARIANT_REG
        for variant in (binding.VARIANT_AUTO, binding.VARIANT_REG, binding.VARIANT_LDS):
            Cg.fill_(float("nan"))
            binding.gcoo_spdm(A, Bt, Cg, variant=variant)
            torch.cuda.synchronize()
            err, bad = orc.max_scaled_error(Cg.cpu().numpy(), C64, D64)
            assert bad == 0 and err <= TOL, (variant, err, bad)
        E = A.export()
        assert np.array_equal(E["gIdxes"], G.gIdxes) and np.array_equal(E["cols"], G.cols) and np.array_equal(E["rows"], G.rows)
        assert np.array_equal(E["values"].view(np.uint32), G.values.view(np.uint32))


@pytest.mark.skip(reason="the one-column-per-lane register kernel (65 <= p <= 128) is not part of the library any more: "
                         "one run of it at 8000 x 8000, p = 128 ended in a GPU memory fault whose cause was never found")
def test_register_kernel_one_column_per_lane():
    w = workloads.config(3)
    _check_product(w, 128, binding.VARIANT_REG, r0=0, r1=128)


@pytest.mark.parametrize("m,k,N,p,sparsity", [
    (64, 6000, 256, 32, 0.5), (40, 3000, 520, 16, 0.7), (128, 5000, 128, 64, 0.8), (33, 9000, 64, 32, 0.97),
    (256, 2500, 1024, 32, 0.9),
])
def test_heavy_groups_shared_by_a_workgroup(m, k, N, p, sparsity):
    """Few (group, tile) items with thousands of entries each: the register kernel hands such groups
    to eight waves that split the entries and add their partial sums in a fixed order."""
    w = workloads.uniform_random(m, k, N, sparsity, seed=m + k + N)
    _say(f"heavy groups m={m} k={k} N={N} p={p} nnz={w.nnz}")
    err, A, c1 = _check_product(w, p, binding.VARIANT_REG)
    assert err < 2e-6
    _, _, c2 = _check_product(w, p, binding.VARIANT_REG, A=A)
    assert np.array_equal(c1, c2)                        # same bits on every run


def test_auto_variant_and_strided_operands():
    _say("strided B and C")
    w = workloads.uniform_random(200, 150, 96, 0.9, seed=21)
    A = binding.gcoo_from_csr(w.m, w.k, w.row_ptr, w.col_idx, w.vals, 32, device=DEV)
    Bbig = torch.zeros((w.k, 200), device=DEV)
    Bbig[:, 4:100] = torch.from_numpy(w.B).to(DEV)
    Cbig = torch.full((w.m, 160), 7.0, device=DEV)
    for off in (4, 5):                                # 16-byte aligned and unaligned column offsets
        Bv = Bbig[:, off:off + 96]
        if off != 4:
            Bv.copy_(torch.from_numpy(w.B).to(DEV))
        Cv = Cbig[:, 8:104]
        binding.gcoo_spdm(A, Bv, Cv)
        torch.cuda.synchronize()
        C64, D64 = orc.spdm_csr(w.k, 96, w.row_ptr, w.col_idx, w.vals, w.B)
        err, bad = orc.max_scaled_error(Cv.cpu().numpy(), C64, D64)
        assert bad == 0 and err <= TOL
        assert torch.all(Cbig[:, :8] == 7.0) and torch.all(Cbig[:, 104:] == 7.0)       # nothing outside C touched


def test_special_cases_bit_exact():
    """Products that are exact in fp32: the GPU result must equal them bit for bit."""
    _say("special cases")
    rng = np.random.default_rng(3)
    n, N = 150, 132
    B = rng.standard_normal((n, N)).astype(np.float32)
    Bt = torch.from_numpy(B).to(DEV)
    perm = rng.permutation(n)
    d = rng.standard_normal(n).astype(np.float32)
    cases = {
        "identity": (sp.identity(n, dtype=np.float32, format="csr"), B),
        "permutation": (sp.csr_matrix((np.ones(n, np.float32), (np.arange(n), perm)), shape=(n, n)), B[perm]),
        "zero": (sp.csr_matrix((n, n), dtype=np.float32), np.zeros_like(B)),
        "diagonal": (sp.diags(d, format="csr", dtype=np.float32), d[:, None] * B),
        "single": (sp.csr_matrix((np.array([2.5], np.float32), ([4], [9])), shape=(n, n)), None),
    }
    single = np.zeros_like(B)
    single[4] = np.float32(2.5) * B[9]
    cases["single"] = (cases["single"][0], single)
    for name, (S, expect) in cases.items():
        S = sp.csr_matrix(S)
        for p in (8, 32, 64):
            A = binding.gcoo_from_csr(n, n, S.indptr.astype(np.int32), S.indices.astype(np.int32),
                                      S.data.astype(np.float32), p, device=DEV)
            for variant in _variants_for(p, N):
                C = binding.gcoo_spdm(A, Bt, variant=variant)
                torch.cuda.synchronize()
                assert np.array_equal(C.cpu().numpy(), expect), (name, p, variant)


def test_unstored_entries_are_skipped_not_multiplied():
    _say("non-finite B rows that A never touches")
    w = workloads.uniform_random(64, 64, 128, 0.98, seed=9)
    untouched = np.setdiff1d(np.arange(w.k), w.col_idx)
    assert untouched.size > 0
    B = w.B.copy()
    B[untouched] = np.inf
    B[untouched[0]] = np.nan
    w.B = B
    for variant in _variants_for(32, w.N):
        _check_product(w, 32, variant)


def test_independent_of_p_and_deterministic():
    _say("p independence / determinism")
    w = workloads.uniform_random(256, 256, 256, 0.9, seed=13)
    Bt = torch.from_numpy(w.B).to(DEV)
    C64, D64 = orc.spdm_csr(w.k, w.N, w.row_ptr, w.col_idx, w.vals, w.B)
    for p in (8, 32, 64, 128):
        A = binding.gcoo_from_csr(w.m, w.k, w.row_ptr, w.col_idx, w.vals, p, device=DEV)
        for variant in _variants_for(p, w.N):
            c1 = binding.gcoo_spdm(A, Bt, variant=variant).cpu().numpy()
            c2 = binding.gcoo_spdm(A, Bt, variant=variant).cpu().numpy()
            assert np.array_equal(c1, c2)                    # no atomics anywhere: same bits on every run
            err, bad = orc.max_scaled_error(c1, C64, D64)    # the order of the sum depends on p, the value does not
            assert bad == 0 and err <= TOL


def test_linearity_in_B_power_of_two_scale():
    _say("linearity")
    w = workloads.uniform_random(128, 128, 128, 0.9, seed=17)
    A = binding.gcoo_from_csr(w.m, w.k, w.row_ptr, w.col_idx, w.vals, 32, device=DEV)
    Bt = torch.from_numpy(w.B).to(DEV)
    c1 = binding.gcoo_spdm(A, Bt).cpu().numpy()
    c4 = binding.gcoo_spdm(A, Bt * 4.0).cpu().numpy()
    assert np.array_equal(c4, c1 * np.float32(4.0))


@pytest.mark.parametrize("index,p", [(1, 32), (4, 32), (4, 64)])
def test_mid_size_configs_full_check(index, p):
    """4000^2 s=0.95 and the skewed 16384^2 x 512 workload, every element against the oracle."""
    w = workloads.config(index)
    _say(f"config{index} p={p} nnz={w.nnz}")
    _check_product(w, p, binding.VARIANT_AUTO)


@pytest.mark.parametrize("shape", [(300, 200, 1028), (77, 500, 250), (1, 1, 1)])
def test_csr_baseline_kernel(shape):
    """The comparison kernel of the benchmark is held to the same bound as the path itself."""
    m, k, N = shape
    _say(f"csr baseline m={m} k={k} N={N}")
    w = workloads.uniform_random(m, k, N, 0.8, seed=m + N)
    args = [torch.from_numpy(x).to(DEV) for x in (w.row_ptr, w.col_idx, w.vals)]
    Bt = torch.from_numpy(w.B).to(DEV)
    Cg = torch.full((m, N), float("nan"), dtype=torch.float32, device=DEV)
    binding.gcoo_csr_spmm_baseline(m, k, *args, Bt, Cg)
    torch.cuda.synchronize()
    C64, D64 = orc.spdm_csr(w.k, N, w.row_ptr, w.col_idx, w.vals, w.B)
    err, bad = orc.max_scaled_error(Cg.cpu().numpy(), C64, D64)
    assert bad == 0 and err <= TOL


def test_tune_p_returns_a_measured_candidate():
    _say("gcoo_tune_p")
    w = workloads.uniform_random(512, 512, 256, 0.9, seed=4)
    args = [torch.from_numpy(x).to(DEV) for x in (w.row_ptr, w.col_idx, w.vals)]
    best, times = binding.gcoo_tune_p(w.m, w.k, *args, torch.from_numpy(w.B).to(DEV), candidates=(8, 32, 128), reps=2)
    assert set(times) == {8, 32, 128} and best in times and all(t > 0 for t in times.values())
    assert binding.gcoo_default_p(w.m, w.k, w.nnz, w.N) == 32



# ------------------------------------------------------------------ the workgroup-shared kernel and its schedule

def _check_share_schedule(A, m, k, p, G):
    """The share schedule written by the HIP builder equals the Python model record for record."""
    from tests import share_model
    sh = A.export_share()
    assert sh is not None
    info, streams = share_model.build(m, k, p, G.gIdxes, G.rows, G.cols, G.values)
    g = (m + p - 1) // p
    nQ = (g + 7) // 8
    blocks = sh["blocks"].reshape(-1, 16, 4)
    used = []
    for Q in range(nQ):
        ucols, NB = info[Q]
        first = int(G.gIdxes[Q * 8])
        assert sh["ucount"][Q] == len(ucols)
        assert np.array_equal(sh["ucols"][first:first + len(ucols)], ucols)
        hb = first // share_model.BAND + Q
        cap = int(G.gIdxes[min(Q * 8 + 8, g)]) // share_model.BAND + Q + 1 - hb
        assert NB <= cap
        for w in range(8):
            q = Q * 8 + w
            at = int(sh["sbase"][q])
            start = at
            for b, (nq, ns4, blk) in enumerate(streams[q]):
                assert sh["hdr"][2 * (8 * hb + w * cap + b)] == nq, (Q, w, b)
                assert sh["hdr"][2 * (8 * hb + w * cap + b) + 1] == ns4, (Q, w, b)
                assert np.array_equal(blocks[at:at + len(blk)], blk), (Q, w, b)
                at += len(blk)
            used.append((start, at))
    used.sort()
    for (a0, a1), (b0, b1) in zip(used, used[1:]):
        assert a1 <= b0, "streams overlap"
    assert used[-1][1] + 16 <= len(blocks)


@pytest.mark.parametrize("m,k,N,p,s", [
    (100, 300, 8, 32, 0.9), (257, 1000, 260, 42, 0.99), (70, 200, 4, 16, 0.3), (64, 64, 64, 48, 0.0), (33, 50, 4, 8, 0.95),
    (300, 70, 12, 32, 0.6), (1, 1, 4, 1, 0.0), (20, 130, 4, 32, 1.0), (700, 500, 516, 48, 0.5), (530, 2000, 300, 12, 0.98),
    (1000, 3000, 1024, 42, 0.995), (3000, 900, 64, 16, 0.95), (64, 4000, 256, 32, 0.999), (100, 300, 8, 2, 0.95),
    # one, two and three bands, full and with one column over (the kernel asks for the rows of two bands beyond the last
    # one as for any other: their columns repeat the last one)
    (336, 48, 256, 42, 0.5), (336, 49, 256, 42, 0.5), (400, 96, 260, 42, 0.7), (400, 97, 512, 48, 0.7), (336, 145, 256, 42, 0.9),
])
def test_share_schedule_and_variant(share_always, m, k, N, p, s):
    """The kernel whose eight waves share the rows of B through LDS: its schedule against the model, its product
    against the oracle, the same bits on a second run."""
    _say(f"share: m={m} k={k} N={N} p={p} s={s}")
    w = workloads.uniform_random(m, k, N, s, seed=m + k)
    G = orc.gcoo_from_csr(w.m, w.k, w.row_ptr, w.col_idx, w.vals, p)
    A = binding.gcoo_from_csr(w.m, w.k, w.row_ptr, w.col_idx, w.vals, p, device=DEV)
    if w.nnz == 0:
        assert A.export_share() is None
        return
    _check_share_schedule(A, m, k, p, G)
    err, _, c1 = _check_product(w, p, binding.VARIANT_SHARE, A=A)
    assert err < 2e-6
    _, _, c2 = _check_product(w, p, binding.VARIANT_SHARE, A=A)
    assert np.array_equal(c1, c2)


@pytest.mark.parametrize("p", [16, 32, 48])
def test_share_variant_skewed_rows_and_diagonal(share_always, p):
    """Power-law row lengths (a few groups with thousands of entries in one band: many blocks per band, ring
    pieces requested in the middle of a band) and a diagonal matrix (one entry per column)."""
    w = workloads.zipf_rows(700, 3000, 260, seed=17, row_max=2500)
    _say(f"share variant, skewed rows p={p} nnz={w.nnz}")
    err, A, c1 = _check_product(w, p, binding.VARIANT_SHARE)
    assert err < 2e-6
    _, _, c2 = _check_product(w, p, binding.VARIANT_SHARE, A=A)
    assert np.array_equal(c1, c2)
    d = workloads.diagonal(1000, 516, seed=3)
    _say(f"share variant, diagonal p={p}")
    err, _, _ = _check_product(d, p, binding.VARIANT_SHARE)
    assert err < 2e-6


def test_share_schedule_of_a_very_sparse_matrix(share_always):
    """So few entries that the per-group column bitmaps of the conversion do not fit its scratch area: the column
    lists are then made by one workgroup per super-group.  Schedule against the model, product against the oracle."""
    m, k, p = 3000, 40000, 24
    w = workloads.uniform_random(m, k, 64, 1.0 - 300.0 / (m * k), seed=77)
    assert ((m + p - 1) // p) * ((k + 31) // 32) * 4 > 12 * w.nnz
    _say(f"share variant, very sparse: nnz={w.nnz}")
    A = binding.gcoo_from_csr(w.m, w.k, w.row_ptr, w.col_idx, w.vals, p, device=DEV)
    G = orc.gcoo_from_csr(w.m, w.k, w.row_ptr, w.col_idx, w.vals, p)
    _check_share_schedule(A, m, k, p, G)
    err, _, _ = _check_product(w, p, binding.VARIANT_SHARE, A=A)
    assert err < 2e-6


def test_share_variant_repeated_coordinates_and_strides(share_always):
    from tests.test_share_model import repeated_coordinates_workload
    m, k, N, row_ptr, col_idx, vals, B = repeated_coordinates_workload()
    _say("share variant: repeated coordinates, strided operands")
    k2, N2 = 4000, 12
    rng = np.random.default_rng(2)
    Bh = rng.standard_normal((k2, N2)).astype(np.float32)
    Bbig = torch.zeros((k2, 40), device=DEV)
    Bbig[:, 8:8 + N2] = torch.from_numpy(Bh).to(DEV)
    C64, D64 = orc.spdm_csr(k2, N2, row_ptr, col_idx, vals, Bh)
    for p in (8, 48):
        G = orc.gcoo_from_csr(m, k2, row_ptr, col_idx, vals, p)
        A = binding.gcoo_from_csr(m, k2, row_ptr, col_idx, vals, p, device=DEV)
        _check_share_schedule(A, m, k2, p, G)
        Cbig = torch.full((m, 32), 7.0, device=DEV)
        binding.gcoo_spdm(A, Bbig[:, 8:8 + N2], Cbig[:, 4:4 + N2], variant=binding.VARIANT_SHARE)
        torch.cuda.synchronize()
        err, bad = orc.max_scaled_error(Cbig[:, 4:4 + N2].cpu().numpy(), C64, D64)
        assert bad == 0 and err <= TOL
        assert torch.all(Cbig[:, :4] == 7.0) and torch.all(Cbig[:, 4 + N2:] == 7.0)
    with pytest.raises(binding.GcooError):                  # rows not 16-byte aligned
        binding.gcoo_spdm(A, Bbig[:, 9:9 + N2], Cbig[:, 4:4 + N2], variant=binding.VARIANT_SHARE)
    torch.cuda.synchronize()


def test_share_policy_and_automatic_choice():
    """By default a matrix gets a share schedule only where the workgroup-shared kernel is the automatic choice;
    the register kernel's schedule is always there, so either kernel can run on the same handle."""
    _say("share policy")
    w = workloads.uniform_random(4096, 12000, 3072, 0.97, seed=8)      # 12000 columns, 3 % dense
    Bt = torch.from_numpy(w.B).to(DEV)
    Cg = torch.empty((w.m, w.N), device=DEV)
    for p in (32, 24):                                                  # 16 x 12 and 22 x 12 workgroups
        A = binding.gcoo_from_csr(w.m, w.k, w.row_ptr, w.col_idx, w.vals, p, device=DEV)
        assert A.export_share() is not None and binding.gcoo_spdm_pick(A, Bt, Cg) == binding.VARIANT_SHARE
        # too few blocks of C for the workgroups of that kernel to occupy the chip
        assert binding.gcoo_spdm_pick(A, Bt[:, :256], Cg[:, :256]) == binding.VARIANT_REG
        err, _, cfull = _check_product(w, p, binding.VARIANT_AUTO, A=A)
        assert err < 2e-6
        Cn = torch.full((w.m, 256), float("nan"), device=DEV)
        binding.gcoo_spdm(A, Bt[:, :256], Cn)
        torch.cuda.synchronize()
        scale = float(np.abs(w.B).max()) * float(np.abs(w.vals).max())
        assert float((Cn - torch.from_numpy(cfull[:, :256]).to(DEV)).abs().max()) <= 1e-4 * scale * 8
    w2 = workloads.uniform_random(64, 3000, 256, 0.97, seed=8)         # too few columns for that kernel to pay
    A2 = binding.gcoo_from_csr(w2.m, w2.k, w2.row_ptr, w2.col_idx, w2.vals, 32, device=DEV)
    assert A2.export_share() is None
    assert binding.gcoo_spdm_pick(A2, torch.from_numpy(w2.B).to(DEV), Cg[:64, :256]) == binding.VARIANT_REG
    w3 = workloads.uniform_random(64, 8000, 256, 0.98, seed=9)
    assert binding.gcoo_from_csr(w3.m, w3.k, w3.row_ptr, w3.col_idx, w3.vals, 48, device=DEV).export_share() is not None
    assert binding.gcoo_from_csr(w3.m, w3.k, w3.row_ptr, w3.col_idx, w3.vals, 49, device=DEV).export_share() is None
    binding.gcoo_set_share_policy(binding.SHARE_NEVER)
    try:
        A3 = binding.gcoo_from_csr(w.m, w.k, w.row_ptr, w.col_idx, w.vals, 32, device=DEV)
        assert A3.export_share() is None and binding.gcoo_spdm_pick(A3, Bt, Cg) == binding.VARIANT_REG
    finally:
        binding.gcoo_set_share_policy(binding.SHARE_AUTO)


# ------------------------------------------------------------------ the benchmark's launches, every element

def _every_element(w, A, Bt, variant, chunk=1000):
    """C = A x B at full size against the oracle, every element, in row chunks; returns the largest scaled error."""
    Cg = torch.full((w.m, w.N), float("nan"), dtype=torch.float32, device=DEV)
    binding.gcoo_spdm(A, Bt, Cg, variant=variant)
    torch.cuda.synchronize()
    Ch = Cg.cpu().numpy()
    worst = 0.0
    for r0 in range(0, w.m, chunk):
        r1 = min(r0 + chunk, w.m)
        C64, D64 = orc.spdm_csr(w.k, w.N, w.row_ptr, w.col_idx, w.vals, w.B, r0, r1)
        err, bad = orc.max_scaled_error(Ch[r0:r1], C64, D64)
        assert bad == 0 and err <= TOL, (r0, err, bad)
        worst = max(worst, err)
    return worst, Cg


@pytest.mark.parametrize("index", [2, 3])
def test_full_size_configs_every_element(index):
    """8000^2 at s=0.9 and s=0.995 in the launch configuration the benchmark times (group height from
    gcoo_default_p, automatic variant, device CSR with nnz given): all five GCOO arrays and every element of C
    against the oracle, and the same bits on a second launch."""
    w = workloads.config(index)
    p = binding.gcoo_default_p(w.m, w.k, w.nnz, w.N)
    assert p == (38 if index == 2 else 42)
    _say(f"config{index} nnz={w.nnz} p={p}")
    dev = [torch.from_numpy(x).to(DEV) for x in (w.row_ptr, w.col_idx, w.vals)]
    A = binding.gcoo_from_csr(w.m, w.k, *dev, p, device=DEV, known_nnz=True)
    _assert_arrays_equal(A.export(), orc.gcoo_from_csr(w.m, w.k, w.row_ptr, w.col_idx, w.vals, p))
    Bt = torch.from_numpy(w.B).to(DEV)
    Cp = torch.empty((w.m, w.N), dtype=torch.float32, device=DEV)
    assert binding.gcoo_spdm_pick(A, Bt, Cp) == (binding.VARIANT_REG if index == 2 else binding.VARIANT_SHARE)
    worst, C1 = _every_element(w, A, Bt, binding.VARIANT_AUTO)
    _say(f"  every element within {worst:.2e}")
    _, C2 = _every_element(w, A, Bt, binding.VARIANT_AUTO)
    assert torch.equal(C1, C2)
    if index == 3:                       # the register kernel at its best height, as before the workgroup-shared one took over here
        A32 = binding.gcoo_from_csr(w.m, w.k, *dev, 32, device=DEV, known_nnz=True)
        worst, _ = _every_element(w, A32, Bt, binding.VARIANT_REG)
        _say(f"  register kernel, p = 32: every element within {worst:.2e}")


def test_full_size_sweep_point_every_element():
    """8000^2 at s=0.98, N = 8000, as the benchmark's sweeps run it: group height from gcoo_default_p, automatic
    variant (the workgroup-shared kernel); arrays and every element of C against the oracle."""
    n, s = 8000, 0.98
    w = workloads.uniform_random(n, n, n, s, workloads.BASE_SEED + n, name="uniform_8000_0.98")
    p = binding.gcoo_default_p(w.m, w.k, w.nnz, w.N)
    _say(f"uniform 8000 s=0.98 nnz={w.nnz} default p={p}")
    assert p == 42
    A = binding.gcoo_from_csr(w.m, w.k, w.row_ptr, w.col_idx, w.vals, p, device=DEV)
    _assert_arrays_equal(A.export(), orc.gcoo_from_csr(w.m, w.k, w.row_ptr, w.col_idx, w.vals, p))
    Bt = torch.from_numpy(w.B).to(DEV)
    Cp = torch.empty((w.m, w.N), dtype=torch.float32, device=DEV)
    assert binding.gcoo_spdm_pick(A, Bt, Cp) == binding.VARIANT_SHARE
    worst, _ = _every_element(w, A, Bt, binding.VARIANT_AUTO)
    _say(f"  every element within {worst:.2e}")


@pytest.mark.parametrize("p", [32, 48])
def test_skewed_config_through_the_share_variant(share_always, p):
    """The 16384^2 power-law workload through the workgroup-shared kernel, every element."""
    w = workloads.config(4)
    _say(f"config4 share p={p} nnz={w.nnz}")
    A = binding.gcoo_from_csr(w.m, w.k, w.row_ptr, w.col_idx, w.vals, p, device=DEV)
    worst, _ = _every_element(w, A, torch.from_numpy(w.B).to(DEV), binding.VARIANT_SHARE, chunk=4096)
    assert worst < 2e-6


def test_zipf_config_every_element_default_path():
    """The 16384^2 power-law workload as the benchmark runs it (library default height, automatic variant): a launch of
    few items, so the register kernel takes the groups in order of falling size, splits the heavy ones over the
    waves of a workgroup and bundles the others.  Every element against the oracle; the same bits twice."""
    w = workloads.config(4)
    p = binding.gcoo_default_p(w.m, w.k, w.nnz, w.N)
    _say(f"config4 default path p={p} nnz={w.nnz}")
    A = binding.gcoo_from_csr(w.m, w.k, w.row_ptr, w.col_idx, w.vals, p, device=DEV)
    Bt = torch.from_numpy(w.B).to(DEV)
    assert binding.gcoo_spdm_pick(A, Bt, torch.empty((w.m, w.N), device=DEV)) == binding.VARIANT_REG
    worst, C1 = _every_element(w, A, Bt, binding.VARIANT_AUTO, chunk=4096)
    assert worst < 2e-6
    _, C2 = _every_element(w, A, Bt, binding.VARIANT_AUTO, chunk=4096)
    assert torch.equal(C1, C2)


@pytest.mark.parametrize("p", [4, 16, 32, 64])
@pytest.mark.parametrize("N", [64, 260, 1031])
def test_skewed_rows_few_items(p, N):
    """Power-law rows in launches of few items, from all groups heavy (one tile, tall groups) to a mix of heavy
    groups and bundles of light ones, with N that is no multiple of the columns per lane."""
    w = workloads.zipf_rows(900, 5000, N, seed=23 + p, row_max=3000)
    _say(f"skewed rows, few items: p={p} N={N} nnz={w.nnz}")
    err, A, c1 = _check_product(w, p, binding.VARIANT_REG)
    assert err < 2e-6
    _, _, c2 = _check_product(w, p, binding.VARIANT_REG, A=A)
    assert np.array_equal(c1, c2)


# ------------------------------------------------------------------ dispatch corners

@pytest.mark.parametrize("p", [8, 32, 38, 48])
def test_register_kernel_with_any_n_and_alignment(p):
    """N that is no multiple of the columns per lane, and views that start 4, 8 or 12 bytes into a row with odd leading
    dimensions: the register kernel serves them all (unaligned 16-byte accesses, the last lane of a row shifted
    inside), and nothing outside the N columns of C is written."""
    w = workloads.uniform_random(300, 400, 1031, 0.9, seed=31)
    _say(f"register kernel, ragged N and alignment, p={p}")
    A = binding.gcoo_from_csr(w.m, w.k, w.row_ptr, w.col_idx, w.vals, p, device=DEV)
    Bt = torch.from_numpy(w.B).to(DEV)
    for N2, shift, pitch in [(1031, 0, 1031), (1030, 0, 1030), (1029, 1, 1041), (1024, 2, 1040), (1027, 3, 1039), (1024, 1, 1027),
                             (513, 5, 1031)]:
        Bbig = torch.zeros((w.k, pitch), device=DEV)
        Bbig[:, shift:shift + N2] = Bt[:, :N2]
        Cbig = torch.full((w.m, pitch), 7.0, device=DEV)
        Bv, Cv = Bbig[:, shift:shift + N2], Cbig[:, shift:shift + N2]
        assert binding.gcoo_spdm_pick(A, Bv, Cv) == binding.VARIANT_REG
        binding.gcoo_spdm(A, Bv, Cv, variant=binding.VARIANT_AUTO)
        torch.cuda.synchronize()
        C64, D64 = orc.spdm_csr(w.k, N2, w.row_ptr, w.col_idx, w.vals, np.ascontiguousarray(w.B[:, :N2]))
        err, bad = orc.max_scaled_error(Cv.cpu().numpy(), C64, D64)
        assert bad == 0 and err <= TOL, (N2, shift, pitch, err, bad)
        assert torch.all(Cbig[:, :shift] == 7.0) and torch.all(Cbig[:, shift + N2:] == 7.0), (N2, shift, pitch)


def test_skewed_matrix_through_the_tall_layout():
    """Power-law row lengths at p = 38 (the tall accumulator layout, which never splits a heavy group)."""
    w = workloads.zipf_rows(700, 3000, 260, seed=17, row_max=2500)
    _say(f"skewed rows, p = 38, nnz={w.nnz}")
    err, A, c1 = _check_product(w, 38, binding.VARIANT_REG)
    assert err < 2e-6
    _, _, c2 = _check_product(w, 38, binding.VARIANT_REG, A=A)
    assert np.array_equal(c1, c2)


def test_one_handle_two_host_threads_two_streams(share_always):
    """A handle is read-only after conversion: two host threads multiply with it at once, each on a stream of
    its own, through different kernels, and both get the oracle's result."""
    import threading
    w = workloads.uniform_random(1500, 4000, 1024, 0.98, seed=12)
    _say("one handle, two threads, two streams")
    A = binding.gcoo_from_csr(w.m, w.k, w.row_ptr, w.col_idx, w.vals, 32, device=DEV)
    Bt = torch.from_numpy(w.B).to(DEV)
    torch.cuda.synchronize()
    C64, D64 = orc.spdm_csr(w.k, w.N, w.row_ptr, w.col_idx, w.vals, w.B)
    outs, errors = {}, []

    def work(name, variant):
        try:
            st = torch.cuda.Stream(device=DEV)
            for _ in range(5):
                Cg = torch.full((w.m, w.N), float("nan"), dtype=torch.float32, device=DEV)
                binding.gcoo_spdm(A, Bt, Cg, variant=variant, stream=st)
            st.synchronize()
            outs[name] = Cg.cpu().numpy()
        except Exception as e:                                   # surfaced below
            errors.append((name, e))
    threads = [threading.Thread(target=work, args=("share", binding.VARIANT_SHARE)),
               threading.Thread(target=work, args=("reg", binding.VARIANT_REG)),
               threading.Thread(target=work, args=("auto", binding.VARIANT_AUTO))]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    for name, Ch in outs.items():
        err, bad = orc.max_scaled_error(Ch, C64, D64)
        assert bad == 0 and err <= TOL, name


def test_dense_count_on_two_streams_at_once():
    """gcoo_dense_nnz takes a counter of its own per call: two host threads on two streams get their own counts."""
    import threading
    _say("gcoo_dense_nnz from two threads")
    rng = np.random.default_rng(6)
    mats = [torch.from_numpy(((rng.random((3000, 2000)) < d) * 1.0).astype(np.float32)).to(DEV) for d in (0.1, 0.3)]
    want = [int((x != 0).sum().item()) for x in mats]
    got = [[], []]

    def work(i):
        st = torch.cuda.Stream(device=DEV)
        for _ in range(20):
            got[i].append(binding.gcoo_dense_nnz(mats[i], stream=st))
    threads = [threading.Thread(target=work, args=(i,)) for i in (0, 1)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert got[0] == [want[0]] * 20 and got[1] == [want[1]] * 20


def test_device_csr_with_a_column_out_of_range_is_clamped_and_reported():
    """Device input is not validated on the host; a column outside [0, k) is stored clamped (so no kernel leaves
    B) and gcoo_export says GCOO_EBOUNDS."""
    _say("device CSR, column out of range")
    w = workloads.uniform_random(100, 200, 64, 0.9, seed=2)
    ci = w.col_idx.copy()
    ci[5] = 200
    ci[17] = -3
    dev = [torch.from_numpy(x).to(DEV) for x in (w.row_ptr, ci, w.vals)]
    A = binding.gcoo_from_csr(w.m, w.k, *dev, 16, device=DEV, known_nnz=True)
    with pytest.raises(binding.GcooError) as e:
        A.export()
    assert e.value.status == binding.GCOO_EBOUNDS
    Cg = binding.gcoo_spdm(A, torch.from_numpy(w.B).to(DEV))           # stays inside B: columns 199 and 0 were used
    torch.cuda.synchronize()
    ci[5], ci[17] = 199, 0
    order = np.lexsort((ci, np.repeat(np.arange(w.m), np.diff(w.row_ptr))))
    C64, D64 = orc.spdm_csr(w.k, w.N, w.row_ptr, ci[order].astype(np.int32), w.vals[order], w.B)
    err, bad = orc.max_scaled_error(Cg.cpu().numpy(), C64, D64)
    assert bad == 0 and err <= TOL
