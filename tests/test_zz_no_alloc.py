"""The conversion that allocates no device memory (gcoo_from_csr_device_static) against the existing entry point
(gcoo_from_csr_device): same arrays, same schedules, same product, on two calls in a row of which the second
is the smaller one (the library's scratch keeps what the first call left in it)."""
import ctypes as C

import numpy as np
import pytest

torch = pytest.importorskip("torch")

from paper_2005_14469_amd import binding, workloads

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _convert_both(w, p):
    """One matrix through both entry points, called through the C ABI with buffers allocated beforehand."""
    L = binding.lib()
    dev = [torch.from_numpy(x).to(DEV) for x in (w.row_ptr, w.col_idx, w.vals)]
    need_ref = int(L.gcoo_device_bytes(w.m, w.k, w.nnz, p))
    need_new = int(L.gcoo_static_handle_bytes(w.m, w.k, w.nnz, p))
    assert 0 < need_new < need_ref                      # the handle alone, without the conversion's scratch
    buf_ref = torch.empty(need_ref, dtype=torch.uint8, device=DEV)
    buf_new = torch.full((need_new,), 0xA5, dtype=torch.uint8, device=DEV)
    sp = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    h_ref, h_new = C.c_void_p(), C.c_void_p()
    assert L.gcoo_from_csr_device(w.m, w.k, w.nnz, dev[0].data_ptr(), dev[1].data_ptr(), dev[2].data_ptr(), p,
                                  buf_ref.data_ptr(), need_ref, sp, C.byref(h_ref)) == 0
    assert L.gcoo_from_csr_device_static(w.m, w.k, w.nnz, dev[0].data_ptr(), dev[1].data_ptr(), dev[2].data_ptr(), p,
                                         buf_new.data_ptr(), need_new, sp, C.byref(h_new)) == 0
    return binding.GcooMatrix(h_ref.value, buf_ref), binding.GcooMatrix(h_new.value, buf_new)


def _same(A_ref, A_new, w):
    E0, E1 = A_ref.export(), A_new.export()
    for key in ("rows", "cols", "gIdxes", "nnzPerGroup"):
        assert np.array_equal(E0[key], E1[key]), key
    assert np.array_equal(E0["values"].view(np.uint32), E1["values"].view(np.uint32))
    S0, S1 = A_ref.export_share(), A_new.export_share()
    assert (S0 is None) == (S1 is None)
    if S0 is not None:
        # (headers of bands a super-group does not have, and the places of the streams, are not defined: the
        # products below, bit for bit, are the check of headers and records)
        assert np.array_equal(S0["ucount"], S1["ucount"])
        for Q, n in enumerate(S0["ucount"]):
            first = int(E0["gIdxes"][8 * Q])
            assert np.array_equal(S0["ucols"][first:first + n], S1["ucols"][first:first + n])
    Bt = torch.from_numpy(w.B).to(DEV)
    variants = [binding.VARIANT_AUTO, binding.VARIANT_REG] + ([binding.VARIANT_SHARE] if S0 is not None else [])
    for variant in variants:
        C0 = torch.full((w.m, w.N), float("nan"), dtype=torch.float32, device=DEV)
        C1 = torch.full((w.m, w.N), float("nan"), dtype=torch.float32, device=DEV)
        binding.gcoo_spdm(A_ref, Bt, C0, variant=variant)
        binding.gcoo_spdm(A_new, Bt, C1, variant=variant)
        torch.cuda.synchronize()
        assert not torch.isnan(C0).any() and torch.equal(C0, C1), variant     # the same bits: same arrays, same schedules


def test_static_conversion_matches_the_existing_one_twice_in_a_row():
    binding.gcoo_set_share_policy(binding.SHARE_ALWAYS)
    try:
        first = workloads.uniform_random(3000, 5000, 512, 0.97, seed=41)       # 450 000 entries, two radix passes
        second = workloads.uniform_random(700, 200, 260, 0.9, seed=42)         # smaller: one pass, fewer groups
        for w, p in ((first, 32), (second, 16)):
            print(f"static conversion: {w.m} x {w.k}, nnz {w.nnz}, p {p}", flush=True)
            A_ref, A_new = _convert_both(w, p)
            torch.cuda.synchronize()
            _same(A_ref, A_new, w)
    finally:
        binding.gcoo_set_share_policy(binding.SHARE_AUTO)


def test_static_conversion_refuses_what_its_scratch_cannot_hold():
    L = binding.lib()
    big = binding.GCOO_STATIC_MAX_NNZ + 1
    assert L.gcoo_static_handle_bytes(4000, 4000, big, 32) == 0
    out = C.c_void_p()
    fake = C.c_void_p(256 * 1024)
    assert L.gcoo_from_csr_device_static(4000, 4000, big, fake, fake, fake, 32, fake, 1 << 40, None, C.byref(out)) == binding.GCOO_ELIMIT
    assert out.value is None and b"2097152" in L.gcoo_strerror(binding.GCOO_ELIMIT)
    assert L.gcoo_static_handle_bytes(4000, 4000, binding.GCOO_STATIC_MAX_NNZ, 32) > 0
