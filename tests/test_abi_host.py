"""Host-only checks of the C ABI: the library loads, exports every symbol the header declares,
and the argument checks that need no device behave as the header says.  No kernel is launched."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2005_14469_amd import binding, build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(binding.LIB_PATH):
        build.build()
    return binding.lib()


def _declared(header):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return set(re.findall(r"\b(gcoo_[a-z_]+)\s*\(", text))


def test_header_symbols_are_exported(L):
    declared = _declared("gcoo.h")
    assert declared == set(binding.SYMBOLS)
    for name in declared:
        assert hasattr(L, name), name
    base = _declared("gcoo_baseline.h")
    assert base == set(binding.BASELINE_SYMBOLS)
    for name in base:
        assert hasattr(binding.baseline_lib(), name), name
        assert not hasattr(L, name), "the comparison routine is not part of the product library"
    assert sorted(os.listdir(os.path.join(ROOT, "include"))) == ["gcoo.h", "gcoo_baseline.h"]


def test_device_bytes_covers_table_1_footprint(L):
    for m, k, nnz, p in [(4, 4, 6, 2), (8000, 8000, 6400000, 32), (1, 1, 0, 1), (16384, 16384, 868447, 64)]:
        b = L.gcoo_device_bytes(m, k, nnz, p)
        g = (m + p - 1) // p
        assert b >= 4 * (3 * nnz + 2 * g + 1) and b % 256 == 0
    assert L.gcoo_device_bytes(-1, 4, 0, 2) == 0
    assert L.gcoo_device_bytes(4, 4, 0, 0) == 0
    assert L.gcoo_device_bytes(4, 4, 0, binding.GCOO_MAX_P + 1) == 0
    assert L.gcoo_device_bytes(4, 4, 2 ** 31, 2) == 0


def test_strerror_and_free_null(L):
    assert L.gcoo_strerror(0) == b"ok"
    for s in (-1, -2, -3, -4, -99):
        assert len(L.gcoo_strerror(s)) > 0
    assert L.gcoo_free(None) == 0
    assert L.gcoo_last_hip_error() is not None


def test_from_csr_rejects_bad_arguments_before_touching_the_device(L):
    out = C.c_void_p()
    rp = np.array([0, 1, 2], np.int32)
    ci = np.array([0, 1], np.int32)
    va = np.ones(2, np.float32)
    fake = C.c_void_p(256 * 1024)          # aligned, never dereferenced on these paths
    call = lambda **kw: L.gcoo_from_csr(kw.get("m", 2), kw.get("k", 2), kw.get("rp", rp).ctypes.data,
                                        kw.get("ci", ci).ctypes.data, va.ctypes.data, 0, kw.get("p", 2),
                                        kw.get("buf", fake), kw.get("bytes", 1 << 20), None, C.byref(out))
    assert call(p=0) == binding.GCOO_EINVAL
    assert call(p=257) == binding.GCOO_EINVAL
    assert call(m=-1) == binding.GCOO_EINVAL
    assert call(buf=C.c_void_p(0)) == binding.GCOO_EINVAL
    assert call(buf=C.c_void_p(256 * 1024 + 4)) == binding.GCOO_EINVAL          # misaligned
    assert call(rp=np.array([0, 2, 1], np.int32)) == binding.GCOO_EBOUNDS       # decreasing
    assert call(rp=np.array([1, 1, 2], np.int32)) == binding.GCOO_EBOUNDS       # does not start at 0
    assert call(ci=np.array([0, 2], np.int32)) == binding.GCOO_EBOUNDS          # column == k
    assert call(ci=np.array([-1, 0], np.int32)) == binding.GCOO_EBOUNDS
    assert call(bytes=16) == binding.GCOO_ENOMEM
    assert out.value is None
    assert L.gcoo_from_csr(2, 2, None, None, None, 0, 2, fake, 1 << 20, None, C.byref(out)) == binding.GCOO_EINVAL
    assert L.gcoo_from_csr(2, 2, rp.ctypes.data, ci.ctypes.data, va.ctypes.data, 0, 2, fake, 1 << 20, None, None) \
        == binding.GCOO_EINVAL


def test_spdm_and_info_reject_null_handle(L):
    assert L.gcoo_spdm(None, None, 4, 4, None, 4, None) == binding.GCOO_EINVAL
    assert L.gcoo_spdm_variant(None, None, 4, 4, None, 4, None, 0) == binding.GCOO_EINVAL
    assert L.gcoo_info(None, None, None, None, None, None) == binding.GCOO_EINVAL
    assert L.gcoo_export(None, None, None, None, None, None, None) == binding.GCOO_EINVAL
    n = C.c_int64()
    assert L.gcoo_dense_nnz(-1, 2, None, 2, None, C.byref(n)) == binding.GCOO_EINVAL
    assert L.gcoo_dense_nnz(2, 4, None, 2, None, C.byref(n)) == binding.GCOO_EINVAL     # lda < k
    out = C.c_void_p()
    assert L.gcoo_from_dense(2, 2, None, 2, 2, C.c_void_p(4096), 1 << 20, None, C.byref(out)) == binding.GCOO_EINVAL


def test_newer_entry_points_reject_bad_arguments_on_the_host(L):
    out = C.c_void_p()
    fake = C.c_void_p(256 * 1024)
    # device-CSR conversion with nnz supplied: the count must fit the 32-bit index arrays
    assert L.gcoo_from_csr_device(2, 2, -1, fake, fake, fake, 2, fake, 1 << 20, None, C.byref(out)) == binding.GCOO_EINVAL
    assert L.gcoo_from_csr_device(2, 2, 2 ** 31, fake, fake, fake, 2, fake, 1 << 40, None, C.byref(out)) \
        == binding.GCOO_EINVAL
    assert L.gcoo_from_csr_device(2, 2, 1, fake, fake, fake, 0, fake, 1 << 20, None, C.byref(out)) == binding.GCOO_EINVAL
    assert L.gcoo_from_csr_device(2, 2, 1, fake, fake, fake, 2, fake, 16, None, C.byref(out)) == binding.GCOO_ENOMEM
    assert L.gcoo_from_csr_device(2, 2, 1, fake, None, None, 2, fake, 1 << 20, None, C.byref(out)) == binding.GCOO_EINVAL
    assert out.value is None
    # share schedule policy and introspection
    assert L.gcoo_set_share_policy(-1) == binding.GCOO_EINVAL
    assert L.gcoo_set_share_policy(3) == binding.GCOO_EINVAL
    assert L.gcoo_set_share_policy(binding.SHARE_AUTO) == 0
    assert L.gcoo_export_share(None, None, None, None, None, None, None, None, None) == binding.GCOO_EINVAL
    # the conversion without device allocations: its limit is checked on the host, before any device call
    big = binding.GCOO_STATIC_MAX_NNZ + 1
    assert L.gcoo_static_handle_bytes(4000, 4000, big, 32) == 0
    assert L.gcoo_from_csr_device_static(4000, 4000, big, fake, fake, fake, 32, fake, 1 << 40, None, C.byref(out)) \
        == binding.GCOO_ELIMIT
    assert out.value is None and b"2097152" in L.gcoo_strerror(binding.GCOO_ELIMIT)
    assert 0 < L.gcoo_static_handle_bytes(4000, 4000, 1000, 32) < L.gcoo_device_bytes(4000, 4000, 1000, 32)
    assert L.gcoo_spdm_pick(None, None, 4, 4, None, 4) == binding.GCOO_EINVAL
    for variant in (-1, 4):
        assert L.gcoo_spdm_variant(None, None, 4, 4, None, 4, None, variant) == binding.GCOO_EINVAL
    # CSR baseline kernel (library of its own): shapes are checked before anything is launched
    Lb = binding.baseline_lib()
    assert Lb.gcoo_csr_spmm_baseline(-1, 2, fake, fake, fake, fake, 4, 4, fake, 4, None) == binding.GCOO_EINVAL
    assert Lb.gcoo_csr_spmm_baseline(2, 2, None, fake, fake, fake, 4, 4, fake, 4, None) == binding.GCOO_EINVAL
    assert Lb.gcoo_csr_spmm_baseline(2, 2, fake, fake, fake, fake, 3, 4, fake, 4, None) == binding.GCOO_EINVAL   # ldb < N
    assert Lb.gcoo_csr_spmm_baseline(2, 2, fake, fake, fake, fake, 4, 4, None, 4, None) == binding.GCOO_EINVAL
    assert Lb.gcoo_csr_spmm_baseline(0, 2, fake, fake, fake, fake, 4, 4, None, 4, None) == 0                     # nothing to do


def _share_height(m, N):
    """The header's rule for the workgroup-shared kernel: the p in 24..48 that minimises
    ceil(workgroups / 256) x (p + 24), the taller one on a tie."""
    best, cost = None, None
    for p in range(48, 23, -1):
        g = (m + p - 1) // p
        items = ((g + 7) // 8) * ((N + 255) // 256)
        c = ((items + 255) // 256) * (p + 24)
        if cost is None or c < cost:
            best, cost = p, c
    return best


def test_default_p_rule(L):
    """32 (the register kernel's best height) unless the workgroup-shared kernel or the tall register instance
    was measured faster: the cases below sit on both sides of every limit the header states."""
    def dp(n, s, N=None, m=None):
        m = n if m is None else m
        return L.gcoo_default_p(m, n, int(m * n * (1 - s)), n if N is None else N)
    assert dp(8000, 0.995) == 42            # the headline workload: 8000 columns at 0.5 %
    assert dp(8000, 0.98) == 42 and dp(8000, 0.99) == 42 and dp(8000, 0.95) == 42      # 24 super-groups x 32 tiles = 3 rounds of 256
    assert dp(8000, 0.996) == 42 and dp(8000, 0.997) == 32          # from 7000 columns on: 0.35 % and more
    assert dp(6000, 0.99) == _share_height(6000, 6000) and dp(6000, 0.995) == 32    # from 5500 on: 0.8 % and more
    assert dp(5000, 0.98) == _share_height(5000, 5000) and dp(5000, 0.99) == 32     # from 3500 on: 1.5 % and more
    assert dp(14000, 0.995) == 48 and dp(12000, 0.997) == 32 and dp(10000, 0.995) != 32
    assert dp(16384, 1 - 868447 / 16384 ** 2, N=512) == 32 and dp(16384, 1 - 868447 / 16384 ** 2) == 32   # the skewed workload's shape
    assert dp(14000, 0.98) == 48 and dp(4000, 0.98) == 32
    for n in (4000, 5000, 7000, 8000, 10000, 14000):
        assert dp(n, 0.98) == _share_height(n, n), n
    assert dp(8000, 0.9) == 38 and dp(8000, 0.93) == 38 and dp(14000, 0.9) == 38      # 6 .. 12 % dense: the tall register instance
    assert dp(8000, 0.8) == 32 and dp(4000, 0.9) == 32 and dp(8000, 0.9, N=8002) == 32
    assert dp(4000, 0.995) == 32            # below 5500 columns only from 1.5 % on
    assert dp(6000, 0.98) in (32, _share_height(6000, 6000))
    assert dp(3000, 0.98) == 32 and dp(2000, 0.98) == 32
    assert dp(12000, 0.98, N=256) == 32     # too few workgroups
    assert dp(12000, 0.98, N=12002) == 32   # rows of B not 16-byte aligned
    for m, k, nnz, n in [(0, 0, 0, 0), (1, 1, 1, 1), (256, 256, 6000, 256)]:
        assert L.gcoo_default_p(m, k, nnz, n) == 32
    # no height for a kernel that the policy rules out
    assert L.gcoo_set_share_policy(binding.SHARE_NEVER) == 0
    try:
        assert dp(8000, 0.995) == 32 and dp(14000, 0.98) == 32 and dp(8000, 0.9) == 38
    finally:
        assert L.gcoo_set_share_policy(binding.SHARE_AUTO) == 0
    assert L.gcoo_default_p(-1, 1, 1, 1) == 0
    assert L.gcoo_default_p(1, 1, -1, 1) == 0
