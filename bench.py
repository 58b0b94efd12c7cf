#!/usr/bin/env python3
"""Benchmark of the GCOO SpDM hot path on one MI355X.

A step is one pass of the whole path over one synthetic input that is already resident in
HBM: CSR (device) -> GCOO conversion kernels -> SpDM kernel -> C.  Prints ONE JSON line.

  metric / value   effective GFLOP/s of the step, 2*nnz*N / t_step (Equation 2 of the paper
                   generalised to m x k times k x N), conversion included
  spdm             the SpDM kernel alone (the paper's "kernel calculation" part of its
                   breakdown, Section 4.3): time from HIP events around each launch on the
                   launch stream, effective GFLOP/s, and the same for the conversion
  roofline         for the dominant kernel (SpDM): algorithmic bytes 12*nnz + 4*k*N + 4*m*N per
                   launch over its measured duration, against 8 TB/s
  cpu_baseline     the CPU oracle, timed as it stands on the host cores on a bounded sample
  dense            rocBLAS/hipBLASLt SGEMM (torch.mm, fp32) on the densified A, for the crossover
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

KERNEL_NAMES = {1: "gcoo::spdm_lds", 2: "gcoo::spdm_sched", 3: "gcoo::spdm_share"}
KERNEL_FILES = {1: "spdm_lds", 2: "spdm_sched", 3: "spdm_share"}
HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
FP32_VECTOR_PEAK_TF = 157.3    # published (packed fp32); plain v_fma_f32 reaches half of it


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="config3",
                    help="config0..config4 (the five named workloads; config3 = 8000^2, sparsity 0.995), or "
                         "uniform_<n>_<sparsity> for a square uniform random A with N = n")
    ap.add_argument("--p", type=int, default=0, help="group height; 0 = library default for the workload")
    ap.add_argument("--variant", type=int, default=0, help="0 auto, 1 partial sums in LDS, 2 partial sums in registers, 3 the same with the rows of B shared through LDS by the eight groups of a workgroup")
    ap.add_argument("--share", choices=["auto", "always", "never"], default="auto",
                    help="when the conversion also builds the schedule of variant 3: where the library expects that kernel to be "
                         "picked (auto), wherever it can run (always: needed to force --variant 3 elsewhere), or never")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing")
    ap.add_argument("--no-dense", action="store_true", help="skip the dense SGEMM timing")
    ap.add_argument("--secondary", default="config2", help="second workload reported in the same line ('' = none)")
    ap.add_argument("--crossover", action="store_true",
                    help="instead of the headline run: sweep the sparsity of an 8000^2 uniform random A and report where "
                         "the path overtakes the dense SGEMM (the time-against-sparsity comparison of Section 4.2 of the paper)")
    ap.add_argument("--sweep", choices=["sparsity", "size"], default=None,
                    help="instead of the headline run, one of the paper's sweeps on uniform random square matrices: "
                         "'sparsity' = time against sparsity at n = 4000 and 14000 with the dense SGEMM beside it "
                         "(Section 4.2); 'size' = GFLOP/s against n at sparsity 0.98 and 0.995 (Section 4.2)")
    ap.add_argument("--eo-kc", action="store_true",
                    help="instead of the headline run: dense A on the device -> GCOO (Algorithm 1) -> SpDM at n = 4000 and "
                         "14000, sparsity 0.95..0.99: the split of Section 4.3 into extra overhead (conversion) and kernel")
    ap.add_argument("--kernels", action="store_true",
                    help="instead of the headline run: the register kernel (p = 32, 38) against the workgroup-shared kernel "
                         "(p = 32, 42, 48) on uniform random square matrices, kernel and conversion times: the grid behind "
                         "the library's choice between the two")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain 256 MiB device copy a few times: the reference launch against which the "
                         "FETCH_SIZE / WRITE_SIZE counters of rocprofv3 --pmc are scaled")
    return ap.parse_args()


def time_path(torch, binding, w, dev, p, variant, steps, warmup):
    """Times `steps` passes of convert + multiply; returns per-step and per-kernel times in ms."""
    rp = torch.from_numpy(w.row_ptr).to(dev)
    ci = torch.from_numpy(w.col_idx).to(dev)
    va = torch.from_numpy(w.vals).to(dev)
    B = torch.from_numpy(w.B).to(dev)
    C = torch.empty((w.m, w.N), dtype=torch.float32, device=dev)
    need = binding.gcoo_device_bytes(w.m, w.k, w.nnz, p)
    buf = torch.empty(need, dtype=torch.uint8, device=dev)
    import ctypes as Cc
    L = binding.lib()
    stream = torch.cuda.current_stream()
    sp = Cc.c_void_p(stream.cuda_stream)

    def convert():
        out = Cc.c_void_p()
        # the CSR arrays are on the device and nnz is known: the conversion reads nothing back
        rc = L.gcoo_from_csr_device(w.m, w.k, w.nnz, rp.data_ptr(), ci.data_ptr(), va.data_ptr(), p, buf.data_ptr(), need, sp,
                                    Cc.byref(out))
        if rc != 0:
            raise binding.GcooError(rc, "gcoo_from_csr_device")
        return out

    def multiply(h):
        rc = L.gcoo_spdm_variant(h, B.data_ptr(), B.stride(0), w.N, C.data_ptr(), C.stride(0), sp, variant)
        if rc != 0:
            raise binding.GcooError(rc, "gcoo_spdm")

    for _ in range(warmup):
        h = convert()
        multiply(h)
        L.gcoo_free(h)
    torch.cuda.synchronize()
    # HIP events around the conversion and the product of every fifth step of the timed region (of every step when
    # there are fewer than ten): an event record costs the stream some 5 us, and three per step were 4 % of a 0.45 ms step
    every = 5 if steps >= 10 else 1
    ev = {i: [torch.cuda.Event(enable_timing=True) for _ in range(3)] for i in range(0, steps, every)}
    t0 = time.perf_counter()
    for i in range(steps):
        e = ev.get(i)
        if e:
            e[0].record(stream)
        h = convert()
        if e:
            e[1].record(stream)
        multiply(h)
        if e:
            e[2].record(stream)
        L.gcoo_free(h)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    conv = [e[0].elapsed_time(e[1]) for e in ev.values()]
    mult = [e[1].elapsed_time(e[2]) for e in ev.values()]
    h = convert()
    picked = L.gcoo_spdm_pick(h, B.data_ptr(), B.stride(0), w.N, C.data_ptr(), C.stride(0)) if variant == 0 else variant
    L.gcoo_free(h)
    torch.cuda.synchronize()
    return dict(ms_per_step=(t1 - t0) * 1e3 / steps, convert_ms=sum(conv) / len(conv), spdm_ms=sum(mult) / len(mult),
                spdm_ms_min=min(mult), variant=int(picked), B=B, C=C)


def dense_ms(torch, w, dev, reps=5):
    """fp32 SGEMM on the densified A (library GEMM; context for the crossover, not part of the path)."""
    import numpy as np
    A = np.zeros((w.m, w.k), np.float32)
    rows = np.repeat(np.arange(w.m), np.diff(w.row_ptr))
    A[rows, w.col_idx] = w.vals
    Ad = torch.from_numpy(A).to(dev)
    B = torch.from_numpy(w.B).to(dev)
    torch.backends.cuda.matmul.allow_tf32 = False
    for _ in range(2):
        torch.mm(Ad, B)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        torch.mm(Ad, B)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def cpu_baseline(w, p, budget_flops=1.2e11):
    """The oracle as it stands (conversion + product, fp64 sums) on a row slice of the workload."""
    from oracle import gcoo_oracle as orc
    flops_full = 2.0 * w.nnz * w.N
    rows = w.m if flops_full <= budget_flops else max(p, int(w.m * budget_flops / flops_full) // p * p)
    rp = (w.row_ptr[:rows + 1] - w.row_ptr[0]).astype("int32")
    nnz = int(rp[-1])
    ci, va = w.col_idx[:nnz], w.vals[:nnz]
    t0 = time.perf_counter()
    orc.gcoo_from_csr(rows, w.k, rp, ci, va, p)
    t1 = time.perf_counter()
    orc.spdm_csr(w.k, w.N, rp, ci, va, w.B, 0, rows, want_scale=False)
    t2 = time.perf_counter()
    return dict(value=2.0 * nnz * w.N / (t2 - t0) / 1e9, unit="GFLOP/s", cores=orc.num_threads(), kind="oracle",
                sample=f"rows 0..{rows - 1} of {w.m} ({nnz} nonzeros): conversion {1e3 * (t1 - t0):.0f} ms + "
                       f"product {1e3 * (t2 - t1):.0f} ms, fp64 sums, OpenMP over rows")


def traffic_file(kernel: str, workload: str) -> str:
    return os.path.join("profiles", f"{kernel}_{workload}_pmc.txt")


def read_traffic(kernel: str, workload: str):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary of this kernel on this workload, if there
    is one (the counters cannot be read from inside this run: the line names the file in traffic_source)."""
    path = os.path.join(ROOT, traffic_file(kernel, workload))
    if not os.path.exists(path):
        return None
    vals = {}
    for line in open(path):
        if "=" in line and not line.startswith("#"):
            k, v = line.split("=", 1)
            try:
                vals[k.strip()] = float(v.split()[0])
            except ValueError:
                pass
    if "FETCH_BYTES_PER_LAUNCH" in vals and "WRITE_BYTES_PER_LAUNCH" in vals:
        return vals["FETCH_BYTES_PER_LAUNCH"] + vals["WRITE_BYTES_PER_LAUNCH"]
    return None


def run_one(torch, binding, workloads, name, args, dev, steps, warmup):
    if name.startswith("uniform_"):                       # uniform_<n>_<sparsity>: square uniform random A, N = n
        _, n_, s_ = name.split("_")
        w = workloads.uniform_random(int(n_), int(n_), int(n_), float(s_), workloads.BASE_SEED + int(n_), name=name)
    else:
        w = workloads.config(int(name.replace("config", "")))
    p = args.p or binding.gcoo_default_p(w.m, w.k, w.nnz, w.N)
    r = time_path(torch, binding, w, dev, p, args.variant, steps, warmup)
    flops = 2.0 * w.nnz * w.N
    alg_bytes = 12.0 * w.nnz + 4.0 * w.k * w.N + 4.0 * w.m * w.N
    out = dict(
        workload=name, m=w.m, k=w.k, N=w.N, nnz=w.nnz, p=p, variant=r["variant"],
        ms_per_step=r["ms_per_step"], gflops=flops / r["ms_per_step"] / 1e6,
        convert_ms=r["convert_ms"], spdm_ms=r["spdm_ms"], spdm_ms_min=r["spdm_ms_min"],
        spdm_gflops=flops / r["spdm_ms"] / 1e6,
        hbm_gbs=alg_bytes / r["spdm_ms"] / 1e6, hbm_frac=alg_bytes / r["spdm_ms"] / 1e6 / HBM_PEAK_GBS,
        valu_frac_of_published=flops / r["spdm_ms"] / 1e9 / FP32_VECTOR_PEAK_TF,
        alg_bytes=alg_bytes,
    )
    return w, out


def crossover(torch, binding, workloads, args, dev, n=8000):
    """Time vs. sparsity at n = 8000 against the dense SGEMM; crossover by linear interpolation in log(1-s)."""
    import math
    rows = []
    dense = None
    for s in (0.5, 0.6, 0.7, 0.8, 0.85, 0.9, 0.95, 0.98, 0.99, 0.995, 0.999):
        w = workloads.uniform_random(n, n, n, s, workloads.BASE_SEED + int(round(s * 10000)), name=f"uniform_{n}_s{s}")
        p = args.p or binding.gcoo_default_p(n, n, w.nnz, n)
        r = time_path(torch, binding, w, dev, p, args.variant, 5, 2)
        if dense is None:
            dense = dense_ms(torch, w, dev)
        rows.append(dict(sparsity=s, nnz=w.nnz, p=p, variant=r["variant"], spdm_ms=r["spdm_ms"], convert_ms=r["convert_ms"],
                         step_ms=r["ms_per_step"],
                         spdm_gflops=2.0 * w.nnz * n / r["spdm_ms"] / 1e6))
        del w, r

    def cross(key):
        prev = None
        for row in rows:
            if row[key] <= dense:
                if prev is None:
                    return row["sparsity"]
                # interpolate log(time) against log(1-s)
                x0, x1 = math.log(1 - prev["sparsity"]), math.log(1 - row["sparsity"])
                y0, y1 = math.log(prev[key] / dense), math.log(row[key] / dense)
                x = x0 + (0 - y0) * (x1 - x0) / (y1 - y0)
                return 1 - math.exp(x)
            prev = row
        return None

    return {"metric": "sparsity at which the GCOO path overtakes the dense fp32 SGEMM, n=8000", "dense_sgemm_ms": dense,
            "crossover_sparsity_spdm_kernel": cross("spdm_ms"), "crossover_sparsity_whole_path": cross("step_ms"),
            "p": args.p or "library default per row", "rows": rows}


def copy_bandwidth_gbs(torch, dev):
    """What a plain device copy of 1 GiB sustains on this machine (bytes read + bytes written per second)."""
    src = torch.empty(256 * 1024 * 1024, dtype=torch.float32, device=dev).fill_(1.0)
    dst = torch.empty_like(src)
    t = _event_ms(torch, lambda: dst.copy_(src), 5)
    return 2.0 * src.numel() * 4 / t / 1e6


def _event_ms(torch, fn, reps, warmup=2):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    ts = []
    for _ in range(reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fn()
        e1.record()
        torch.cuda.synchronize()
        ts.append(e0.elapsed_time(e1))
    ts.sort()
    return ts[len(ts) // 2]


def _square_case(torch, binding, workloads, dev, n, sparsity, p, variant, Bd, Cd, reps=5):
    """Device-resident uniform random n x n A (CSR) times a device B: conversion and kernel time in ms."""
    w = workloads.uniform_random(n, n, 1, sparsity, workloads.BASE_SEED + n + int(round(sparsity * 10000)), name="sweep")
    rp, ci, va = [torch.from_numpy(x).to(dev) for x in (w.row_ptr, w.col_idx, w.vals)]
    holder = {}

    def convert():
        holder["A"] = binding.gcoo_from_csr(n, n, rp, ci, va, p)

    t_conv = _event_ms(torch, convert, reps)
    A = holder["A"]
    t_kern = _event_ms(torch, lambda: binding.gcoo_spdm(A, Bd, Cd, variant=variant), reps)
    A.free()
    # context: the plain CSR row-split kernel of this library and the vendor CSR routine behind torch.sparse
    t_csr = _event_ms(torch, lambda: binding.gcoo_csr_spmm_baseline(n, n, rp, ci, va, Bd, Cd), reps)
    t_vendor = None
    try:
        As = torch.sparse_csr_tensor(rp, ci, va, size=(n, n))
        t_vendor = _event_ms(torch, lambda: torch.sparse.mm(As, Bd), 3, warmup=1)
        del As
    except Exception as e:                                   # not every build of torch ships the sparse backend
        print(f"torch.sparse.mm unavailable: {e}", file=sys.stderr)
    return dict(n=n, sparsity=sparsity, nnz=w.nnz, p=p, convert_ms=t_conv, spdm_ms=t_kern,
                spdm_gflops=2.0 * w.nnz * n / t_kern / 1e6, step_gflops=2.0 * w.nnz * n / (t_kern + t_conv) / 1e6,
                csr_rowsplit_ms=t_csr, vendor_csr_ms=t_vendor)


def _dense_square_ms(torch, dev, n, Bd):
    Ad = torch.randn((n, n), device=dev, dtype=torch.float32)
    torch.backends.cuda.matmul.allow_tf32 = False
    t = _event_ms(torch, lambda: torch.mm(Ad, Bd), 5)
    del Ad
    return t


def sweep(torch, binding, workloads, args, dev):
    rows, dense = [], {}
    if args.sweep == "sparsity":
        plan = [(n, s) for n in (4000, 14000) for s in (0.8, 0.9, 0.95, 0.96, 0.97, 0.98, 0.99, 0.995, 0.999)]
    else:
        plan = [(n, s) for s in (0.98, 0.995) for n in (400, 800, 1600, 2400, 3200, 4000, 6000, 8000, 10000, 12000, 14000)]
    cur_n, Bd, Cd = None, None, None
    for n, s in sorted(plan, key=lambda t: t[0]):
        if n != cur_n:
            del Bd, Cd
            g = torch.Generator(device=dev)
            g.manual_seed(workloads.BASE_SEED + n)
            Bd = torch.randn((n, n), generator=g, device=dev, dtype=torch.float32)
            Cd = torch.empty((n, n), device=dev, dtype=torch.float32)
            dense[n] = _dense_square_ms(torch, dev, n, Bd)
            cur_n = n
        p = args.p or binding.gcoo_default_p(n, n, int(round(n * n * (1.0 - s))), n)
        r = _square_case(torch, binding, workloads, dev, n, s, p, args.variant, Bd, Cd)
        print(f"sweep n={n} sparsity={s}: spdm {r['spdm_ms']:.3f} ms, csr {r['csr_rowsplit_ms']:.3f} ms, vendor csr "
              f"{r['vendor_csr_ms']}, dense {dense[n]:.3f} ms", file=sys.stderr, flush=True)
        r["dense_sgemm_ms"] = dense[n]
        r["speedup_over_dense"] = dense[n] / r["spdm_ms"]
        rows.append(r)
    rows.sort(key=lambda r: (r["sparsity"], r["n"]) if args.sweep == "size" else (r["n"], r["sparsity"]))
    return {"metric": f"uniform random square A, fp32, sweep over {args.sweep}", "p": args.p or "library default per row",
            "rows": rows}


def kernels_compared(torch, binding, workloads, args, dev):
    """Register kernel against workgroup-shared kernel on the same matrices (uniform random, N = n)."""
    rows = []
    plan = [(4000, 0.98), (4000, 0.995), (8000, 0.9), (8000, 0.95), (8000, 0.98), (8000, 0.99), (8000, 0.995), (8000, 0.999),
            (14000, 0.98), (14000, 0.995)]
    cur_n, Bd, Cd = None, None, None
    binding.gcoo_set_share_policy(binding.SHARE_ALWAYS)
    try:
        for n, sp in plan:
            if n != cur_n:
                del Bd, Cd
                g = torch.Generator(device=dev)
                g.manual_seed(workloads.BASE_SEED + n)
                Bd = torch.randn((n, n), generator=g, device=dev, dtype=torch.float32)
                Cd = torch.empty((n, n), device=dev, dtype=torch.float32)
                cur_n = n
            w = workloads.uniform_random(n, n, 1, sp, workloads.BASE_SEED + n + int(round(sp * 10000)), name="kernels")
            rp, ci, va = [torch.from_numpy(x).to(dev) for x in (w.row_ptr, w.col_idx, w.vals)]
            row = dict(n=n, sparsity=sp, nnz=w.nnz)
            for name, variant, p in (("reg32", binding.VARIANT_REG, 32), ("reg38", binding.VARIANT_REG, 38),
                                     ("share32", binding.VARIANT_SHARE, 32), ("share42", binding.VARIANT_SHARE, 42),
                                     ("share48", binding.VARIANT_SHARE, 48)):
                holder = {}

                def convert():
                    holder["A"] = binding.gcoo_from_csr(n, n, rp, ci, va, p)

                t_conv = _event_ms(torch, convert, 3)
                A = holder["A"]
                row[name + "_ms"] = _event_ms(torch, lambda: binding.gcoo_spdm(A, Bd, Cd, variant=variant), 5)
                row[name + "_convert_ms"] = t_conv      # with both schedules built (the policy above)
                A.free()
            print("kernels " + " ".join(f"{k}={v:.3f}" if isinstance(v, float) else f"{k}={v}" for k, v in row.items()),
                  file=sys.stderr, flush=True)
            rows.append(row)
    finally:
        binding.gcoo_set_share_policy(binding.SHARE_AUTO)
    return {"metric": "register kernel against workgroup-shared kernel, uniform random square A, N = n, fp32, ms", "rows": rows}


def eo_kc(torch, binding, workloads, args, dev):
    """Dense device matrix -> GCOO -> product: conversion time against kernel time (Section 4.3)."""
    rows = []
    for n in (4000, 14000):
        g = torch.Generator(device=dev)
        g.manual_seed(workloads.BASE_SEED + n)
        B = torch.randn((n, n), generator=g, device=dev, dtype=torch.float32)
        C = torch.empty((n, n), device=dev, dtype=torch.float32)
        for s in (0.95, 0.96, 0.97, 0.98, 0.99):
            w = workloads.uniform_random(n, n, 1, s, workloads.BASE_SEED + n + int(round(s * 1000)), name="eo_kc")
            Ad = torch.zeros((n, n), device=dev, dtype=torch.float32)
            r = torch.repeat_interleave(torch.arange(n, device=dev), torch.from_numpy(w.row_ptr[1:] - w.row_ptr[:-1]).to(dev))
            Ad[r, torch.from_numpy(w.col_idx).to(dev).long()] = torch.from_numpy(w.vals).to(dev)
            del r
            holder = {}
            p = args.p or binding.gcoo_default_p(n, n, w.nnz, n)

            def convert():
                holder["A"] = binding.gcoo_from_dense(Ad, p)      # count, size the buffer, count per block, fill, schedule

            t_count = _event_ms(torch, lambda: binding.gcoo_dense_nnz(Ad), 5)
            t_eo = _event_ms(torch, convert, 5)
            A = holder["A"]
            t_kc = _event_ms(torch, lambda: binding.gcoo_spdm(A, B, C, variant=args.variant), 5)
            dense_bytes = 4.0 * n * n
            rows.append(dict(n=n, sparsity=s, nnz=w.nnz, p=p, count_ms=t_count, eo_ms=t_eo, kc_ms=t_kc,
                             eo_share=t_eo / (t_eo + t_kc),
                             eo_gbs=(3 * dense_bytes + 12.0 * w.nnz) / t_eo / 1e6))
            A.free()
            del Ad, w
        del B, C
    return {"metric": "dense -> GCOO conversion (EO) against SpDM kernel (KC), fp32, A on the device",
            "note": "eo_ms includes the count that sizes the buffer (three reads of A in all); eo_gbs = (3*4*n*n + 12*nnz)/eo_ms",
            "rows": rows}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path needs no second one); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2005_14469_amd import binding, build, workloads

    if not os.path.exists(binding.LIB_PATH):
        build.build()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    binding.gcoo_set_share_policy({"auto": binding.SHARE_AUTO, "always": binding.SHARE_ALWAYS, "never": binding.SHARE_NEVER}[args.share])
    if args.copy_calibration:
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": {"bytes_read": src.numel() * 4, "bytes_written": dst.numel() * 4, "launches": 5}}))
        return

    if args.crossover:
        print(json.dumps(crossover(torch, binding, workloads, args, dev)))
        return
    if args.eo_kc:
        print(json.dumps(eo_kc(torch, binding, workloads, args, dev)))
        return
    if args.kernels:
        print(json.dumps(kernels_compared(torch, binding, workloads, args, dev)))
        return
    if args.sweep:
        print(json.dumps(sweep(torch, binding, workloads, args, dev)))
        return
    w, head = run_one(torch, binding, workloads, args.workload, args, dev, args.steps, args.warmup)
    line = {
        "metric": "fp32 SpDM effective GFLOP/s (2*nnz*N/t, whole path: CSR->GCOO conversion + SpDM kernel)",
        "value": head["gflops"], "unit": "GFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{args.workload}: A {w.m}x{w.k} uniform random, nnz={w.nnz}, B {w.k}x{w.N}, fp32",
                   "p": head["p"], "variant": head["variant"]},
        "spdm": {"ms": head["spdm_ms"], "ms_min": head["spdm_ms_min"], "gflops": head["spdm_gflops"],
                 "convert_ms": head["convert_ms"], "frac_of_fp32_vector_peak": head["valu_frac_of_published"]},
        "roofline": {"bound": "hbm", "achieved": head["hbm_gbs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": head["hbm_frac"], "traffic": read_traffic(KERNEL_FILES.get(head["variant"], "spdm_sched"), args.workload),
                     "traffic_source": (traffic_file(KERNEL_FILES.get(head["variant"], "spdm_sched"), args.workload)
                                        if read_traffic(KERNEL_FILES.get(head["variant"], "spdm_sched"), args.workload) is not None
                                        else None),
                     "kernel": KERNEL_NAMES.get(head["variant"], "?"), "algorithmic_bytes_per_launch": head["alg_bytes"]},
    }
    if not args.no_dense:
        bw = copy_bandwidth_gbs(torch, dev)
        line["roofline"]["measured_copy_gbs"] = bw             # the same algorithmic bytes against what a copy sustains here
        line["roofline"]["frac_of_measured_copy"] = head["hbm_gbs"] / bw
        d = dense_ms(torch, w, dev)
        line["dense"] = {"sgemm_ms": d, "spdm_speedup_over_dense": d / head["spdm_ms"]}
    if args.secondary and args.secondary != args.workload:
        w2, sec = run_one(torch, binding, workloads, args.secondary, args, dev, max(5, args.steps // 5), 2)
        line["secondary"] = {k: sec[k] for k in ("workload", "nnz", "p", "variant", "ms_per_step", "gflops", "convert_ms",
                                                 "spdm_ms", "spdm_gflops", "hbm_frac", "valu_frac_of_published")}
        line["secondary"]["roofline"] = {"bound": "alu", "achieved": sec["spdm_gflops"] / 1e3, "peak": FP32_VECTOR_PEAK_TF,
                                         "unit": "TFLOP/s", "frac": sec["valu_frac_of_published"]}
        if not args.no_dense:
            d2 = dense_ms(torch, w2, dev)
            line["secondary"]["dense_sgemm_ms"] = d2
        del w2
    if not args.no_cpu:
        line["cpu_baseline"] = cpu_baseline(w, head["p"])
    print(json.dumps(line))


if __name__ == "__main__":
    main()
