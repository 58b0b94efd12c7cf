"""The whole step (the conversion that allocates nothing + the product) recorded into a HIP graph and replayed:
gcoo_from_csr_device_static and gcoo_spdm launch kernels on the caller's stream and do nothing else, so a
stream capture can take them.  Every replay is checked against the same calls made eagerly, with the program's
own eager work and synchronisations between the replays, on inputs that change from replay to replay."""
import ctypes as C

import numpy as np
import pytest

torch = pytest.importorskip("torch")

from paper_2005_14469_amd import binding, workloads

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _step(L, w, p, dev, buf, B, Cout, variant, stream_ptr):
    h = C.c_void_p()
    rc = L.gcoo_from_csr_device_static(w.m, w.k, w.nnz, dev[0].data_ptr(), dev[1].data_ptr(), dev[2].data_ptr(), p,
                                       buf.data_ptr(), buf.numel(), stream_ptr, C.byref(h))
    assert rc == 0, rc
    rc = L.gcoo_spdm_variant(h, B.data_ptr(), B.stride(0), B.shape[1], Cout.data_ptr(), Cout.stride(0), stream_ptr, variant)
    assert rc == 0, rc
    return h


@pytest.mark.parametrize("case", ["register", "shared", "few_items", "tall_groups"])
def test_conversion_and_product_in_a_graph(case):
    L = binding.lib()
    if case == "register":
        w, p, variant = workloads.uniform_random(1500, 2000, 516, 0.97, seed=1), 32, binding.VARIANT_REG
    elif case == "shared":
        w, p, variant = workloads.uniform_random(1500, 2000, 512, 0.97, seed=2), 42, binding.VARIANT_SHARE
    elif case == "few_items":
        w, p, variant = workloads.zipf_rows(600, 3000, 260, seed=3, row_max=2000), 32, binding.VARIANT_REG
    else:
        w, p, variant = workloads.uniform_random(900, 1200, 260, 0.95, seed=4), 128, binding.VARIANT_AUTO
    print(f"graph: {case} p={p} nnz={w.nnz}", flush=True)
    binding.gcoo_set_share_policy(binding.SHARE_ALWAYS if case == "shared" else binding.SHARE_AUTO)
    try:
        dev = [torch.from_numpy(x).to(DEV) for x in (w.row_ptr, w.col_idx, w.vals)]
        B = torch.from_numpy(w.B).to(DEV)
        need = int(L.gcoo_static_handle_bytes(w.m, w.k, w.nnz, p))
        assert need > 0
        buf_g = torch.empty(need, dtype=torch.uint8, device=DEV)
        buf_e = torch.empty(need, dtype=torch.uint8, device=DEV)
        C_g = torch.empty((w.m, w.N), device=DEV)
        C_e = torch.empty((w.m, w.N), device=DEV)
        # once eagerly first: the library takes the address of its scratch and raises kernel limits on its first call
        sp = C.c_void_p(torch.cuda.current_stream().cuda_stream)
        L.gcoo_free(_step(L, w, p, dev, buf_e, B, C_e, variant, sp))
        torch.cuda.synchronize()

        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            sp_c = C.c_void_p(torch.cuda.current_stream().cuda_stream)
            h_g = _step(L, w, p, dev, buf_g, B, C_g, variant, sp_c)
        vals0 = dev[2].clone()
        for replay in range(4):
            # new values of A and of B for this replay; the structure (and so every launch shape) stays
            dev[2].copy_(vals0 * (1.0 + 0.25 * replay))
            B.add_(0.5 * replay)
            C_g.fill_(float("nan"))
            graph.replay()
            torch.cuda.synchronize()
            C_e.fill_(float("nan"))
            h_e = _step(L, w, p, dev, buf_e, B, C_e, variant, sp)
            torch.cuda.synchronize()
            L.gcoo_free(h_e)
            assert torch.equal(C_g, C_e), f"replay {replay}"
            assert not torch.isnan(C_g).any()
            # eager work of the program between the replays
            (C_g.sum() + B.sum()).item()
        L.gcoo_free(h_g)
    finally:
        binding.gcoo_set_share_policy(binding.SHARE_AUTO)
