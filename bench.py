#!/usr/bin/env python3
"""Benchmark of libcsr5 on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 2] [--sigma 0]

One "step" is one y = A*x on the CSR5 form of the workload (the tile kernel plus
the carry fix-up kernel, i.e. one csr5_spmv call) with every input resident in HBM.
The CSR -> CSR5 conversion is timed in the same run and reported in units of one
SpMV.  Prints ONE JSON line.  The headline value is SpMV GFLOP/s = 2*nnz / t.

The CPU oracle is used for two things only: a correctness check of the timed
configuration, and the `cpu_baseline` figure (the oracle timed as it stands on
one host core).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published peak


def bytes_model(m, nnz, info, n_ref, vb=8, ib=4):
    """Algorithmic bytes of one SpMV: val + col_idx (vb + 4 B per nonzero), packed
    descriptors, tile_ptr, empty_offset and its per-tile starts, every
    referenced x entry once, y written once.  vb = bytes per value (8 or 4),
    ib = bytes per tile_ptr / empty_offset_ptr entry (8 in the 64-bit index variant)."""
    W, p, pc, E = info["desc_words_per_lane"], info["p"], info["p_complete"], info["empty_offset_len"]
    return ((vb + 4) * nnz + 4 * W * 64 * pc + ib * (p + 1) + ib * (pc + 1) + 4 * E + vb * n_ref + vb * m)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--workload", type=int, default=2,
                    help="1..5 = the five configurations (default 2: the 27-point stencil); 6 = the paper's dense "
                         "2000x2000 matrix; 7 = the 2.2e9-nonzero matrix of the 64-bit index variant, generated "
                         "in GPU memory; 8 = configuration 4 with fewer dense rows (12 M nonzeros)")
    ap.add_argument("--sigma", type=int, default=0, help="tile height, 0 = the library's rule")
    ap.add_argument("--dtype", choices=["f64", "f32"], default="f64",
                    help="f64 is the headline; f32 runs the single-precision instantiation")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=10.0)
    ap.add_argument("--quick", action="store_true", help="skip the conversion/cold/batch extras")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run plain 256 MiB device copies (a kernel of known traffic, "
                         "to scale rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (the method has no multi-GPU part); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_1503_05032_amd import binding as B
    from paper_1503_05032_amd import build as libbuild
    from paper_1503_05032_amd import workloads as wl

    if not os.path.exists(B.LIB_PATH):
        libbuild.build(verbose=False)
    B.load()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(0)

    if args.copy_probe:
        src = torch.ones(1 << 25, dtype=torch.float64, device=dev)      # 256 MiB
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)                                               # 256 MiB read + 256 MiB written
        torch.cuda.synchronize()
        del src, dst

    f32 = args.dtype == "f32"
    tdt = torch.float32 if f32 else torch.float64
    vb = 4 if f32 else 8
    convert_ex = B.csr5s_convert_ex if f32 else B.csr5_convert_ex
    spmv_ex = B.csr5s_spmv_ex if f32 else B.csr5_spmv_ex
    spmv_profile = B.csr5s_spmv_profile if f32 else B.csr5_spmv_profile

    wide = args.workload == 7
    if wide:
        if f32:
            print("bench.py: the 64-bit index variant is double precision only", file=sys.stderr)
            sys.exit(2)
        from paper_1503_05032_amd import workloads_device as wd
        A = wd.huge_mixed(dev)
        a = None
        m, n, nnz, name = A["m"], A["n"], A["nnz"], A["name"]
        row_ptr, col0, val0, x = A["row_ptr"], A["col_idx"], A["val"], A["x"]
        row_ptr_h = row_ptr.cpu().numpy()
        lens = np.diff(row_ptr_h)
        st = {"row_len_min": int(lens.min()), "row_len_avg": float(lens.mean()), "row_len_max": int(lens.max()),
              "empty_rows": int((lens == 0).sum())}
        seen = torch.zeros(n, dtype=torch.bool, device=dev)
        for e0 in range(0, nnz, 1 << 28):
            seen[col0[e0:e0 + (1 << 28)].long()] = True
        n_ref = int(seen.sum().item())
        del seen
        convert_ex, workspace_bytes = B.csr5l_convert_ex, B.csr5l_workspace_bytes
    else:
        a = wl.config(args.workload)
        if f32:
            a.val = a.val.astype(np.float32)
            a.x = a.x.astype(np.float32)
        m, n, nnz, name = a.m, a.n, a.nnz, a.name
        st = a.stats()
        n_ref = int(np.unique(a.col_idx).size)
        row_ptr = torch.from_numpy(a.row_ptr).to(dev)
        col0 = torch.from_numpy(a.col_idx).to(dev)        # pristine CSR copies
        val0 = torch.from_numpy(a.val).to(dev)
        x = torch.from_numpy(a.x).to(dev)
        workspace_bytes = B.csr5_workspace_bytes
    col = col0.clone()
    val = val0.clone()
    y = torch.empty(m, dtype=tdt, device=dev)

    sigma = args.sigma or B.csr5_sigma_auto(nnz, m)
    ws = torch.empty(workspace_bytes(m, nnz, sigma), dtype=torch.uint8, device=dev)

    def ev():
        return torch.cuda.Event(enable_timing=True)

    # ---------------------------------------------------------------- conversion
    conv_ms, conv_alloc_ms = [], []
    h = None
    nconv = 1 if args.quick else 7
    for it in range(nconv):
        if h is not None:
            B.csr5_free(h)
        col.copy_(col0)
        val.copy_(val0)
        torch.cuda.synchronize()
        e0, e1 = ev(), ev()
        e0.record()
        h = convert_ex(m, n, nnz, row_ptr, col, val, sigma=sigma, workspace=ws,
                       flags=B.CSR5_FLAG_NO_HOST_CHECK)
        e1.record()
        torch.cuda.synchronize()
        conv_ms.append(e0.elapsed_time(e1))
    if not args.quick:
        for it in range(5):           # the plain entry point: hipMalloc + host check inside
            c2, v2 = col0.clone(), val0.clone()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            h2 = convert_ex(m, n, nnz, row_ptr, c2, v2, sigma=sigma)
            torch.cuda.synchronize()
            conv_alloc_ms.append((time.perf_counter() - t0) * 1e3)
            B.csr5_free(h2)
            del c2, v2
    status = B.csr5_status(h)
    info = B.csr5_get_info(h)
    assert status & 3 == 0, status

    # ---------------------------------------------------------------- correctness of this configuration
    import oracle
    spmv_ex(h, x, y)
    torch.cuda.synchronize()
    if wide:
        # the oracle on a sample of rows (random ones, the longest ones, the first and the last)
        rng = np.random.default_rng(11)
        rows_s = np.unique(np.concatenate([rng.integers(0, m, 400), np.argsort(lens)[-8:], [0, m - 1]]))
        cs = np.concatenate([col0[row_ptr_h[r]:row_ptr_h[r + 1]].cpu().numpy() for r in rows_s])
        vs = np.concatenate([val0[row_ptr_h[r]:row_ptr_h[r + 1]].cpu().numpy() for r in rows_s])
        rp_s = np.concatenate([[0], np.cumsum(lens[rows_s])]).astype(np.int32)
        y_ref, s_abs = oracle.csr_spmv(len(rows_s), rp_s, cs, vs, x.cpu().numpy())
        err = np.abs(y[torch.from_numpy(rows_s).to(dev)].cpu().numpy() - y_ref)
    else:
        y_ref, s_abs = oracle.csr_spmv(m, a.row_ptr, a.col_idx, a.val.astype(np.float64), a.x.astype(np.float64))
        err = np.abs(y.cpu().numpy().astype(np.float64) - y_ref)
    parity_ok = bool(np.all(err <= (1e-5 if f32 else 1e-12) * s_abs + (1e-30 if f32 else 1e-300)))

    # ---------------------------------------------------------------- timed region: exactly K steps
    for _ in range(args.warmup):
        spmv_ex(h, x, y)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0, e1 = ev(), ev()
    e0.record()
    for _ in range(args.steps):
        spmv_ex(h, x, y)
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    ms_per_step = e0.elapsed_time(e1) / args.steps
    gflops = 2.0 * nnz / (ms_per_step * 1e-3) / 1e9
    B_model = bytes_model(m, nnz, info, n_ref, vb, 8 if wide else 4)
    B_gather = B_model - vb * n_ref + vb * nnz

    extras = {}
    if not args.quick:
        # the paper's protocol (Section 5.1) scaled down: best of 10 batches of 100 runs
        best = 1e30
        for _ in range(10):
            e0, e1 = ev(), ev()
            e0.record()
            for _ in range(100):
                spmv_ex(h, x, y)
            e1.record()
            torch.cuda.synchronize()
            best = min(best, e0.elapsed_time(e1) / 100)
        extras["ms_best_of_10x100"] = round(best, 5)
        # cache-cold: stream 1 GiB through the caches before every launch
        flush = torch.empty(1 << 27, dtype=torch.float64, device=dev)
        cold = []
        for _ in range(10):
            flush.add_(1.0)
            e0, e1 = ev(), ev()
            e0.record()
            spmv_ex(h, x, y)
            e1.record()
            torch.cuda.synchronize()
            cold.append(e0.elapsed_time(e1))
        del flush
        extras["ms_cold_median"] = round(float(np.median(cold)), 5)

    # ---------------------------------------------------------------- dominant kernel, HIP events inside the library
    ms_tiles, ms_fixup = spmv_profile(h, x, y, reps=min(max(args.steps, 50), 2000))
    achieved = B_model / (ms_tiles * 1e-3) / 1e9

    conv = float(np.median(conv_ms))
    out = {
        "metric": "SpMV GFLOP/s & achieved HBM GB/s (% of peak), fp64; convert time in SpMVs",
        "value": round(gflops, 2),
        "unit": "GFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": args.dtype,
        "data": "synthetic",
        "config": {
            "workload": (f"configs[{args.workload - 1}]" if args.workload <= 5 else f"extra workload {args.workload}")
                        + f" {name}: {m}x{n}, nnz={nnz}, "
                        f"nnz/row min/avg/max={st['row_len_min']}/{st['row_len_avg']:.2f}/{st['row_len_max']}, "
                        f"empty rows={st['empty_rows']}",
            "omega": 64, "sigma": info["sigma"], "tiles": info["p"], "index_bits": 64 if wide else 32,
            "desc_words_per_lane": info["desc_words_per_lane"],
            "empty_offset_len": info["empty_offset_len"],
        },
        "parity_ok": parity_ok,
        "spmv": {
            "gflops": round(gflops, 2),
            "bytes_model": B_model,
            "gbs_model": round(B_model / (ms_per_step * 1e-3) / 1e9, 1),
            "pct_hbm_peak_model": round(100 * B_model / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 2),
            "gbs_if_every_gather_missed": round(B_gather / (ms_per_step * 1e-3) / 1e9, 1),
            "wall_ms_per_step": round(wall_ms / args.steps, 5),
            **extras,
        },
        "convert": {
            "ms_workspace_no_host_check": round(conv, 4),
            "in_spmvs": round(conv / ms_per_step, 2),
            "ms_with_hipmalloc_and_host_check": round(float(np.median(conv_alloc_ms)), 4) if conv_alloc_ms else None,
            "in_spmvs_with_hipmalloc": round(float(np.median(conv_alloc_ms)) / ms_per_step, 2) if conv_alloc_ms else None,
        },
        "roofline": {
            "kernel": f"k_spmv<{info['sigma']}>",
            "bound": "hbm",
            "achieved": round(achieved, 1),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBS, 4),
            "traffic": None if f32 else MEASURED_TRAFFIC.get((args.workload, info["sigma"])),
            "kernel_ms": round(ms_tiles, 5),
            "fixup_kernel_ms": round(ms_fixup, 5),
            "bytes_per_launch": B_model,
        },
    }

    if not args.no_cpu_baseline:
        # the oracle as it stands (sequential Algorithm 1, one core), repeated on the
        # same matrix until about cpu_seconds of work
        if wide:      # a bounded part of the matrix: its first rows, about 3e7 nonzeros
            m_s = int(np.searchsorted(row_ptr_h, 30_000_000))
            nnz_s = int(row_ptr_h[m_s])
            o_args = (m_s, row_ptr_h[:m_s + 1].astype(np.int32), col0[:nnz_s].cpu().numpy(),
                      val0[:nnz_s].cpu().numpy(), x.cpu().numpy())
            what = f"SpMVs of the first {m_s} rows ({nnz_s} nonzeros) of the same matrix"
        else:
            nnz_s = nnz
            o_args = (m, a.row_ptr, a.col_idx, a.val, a.x)             # the oracle computes in fp64
            what = "full SpMVs of the same matrix"
        reps, t_acc = 0, 0.0
        while t_acc < args.cpu_seconds and reps < 2000:
            t0 = time.perf_counter()
            oracle.csr_spmv(*o_args)
            t_acc += time.perf_counter() - t0
            reps += 1
        out["cpu_baseline"] = {
            "value": round(2.0 * nnz_s * reps / t_acc / 1e9, 3),
            "unit": "GFLOP/s",
            "cores": 1,
            "kind": "oracle",
            "sample": f"{reps} {what} (sequential Algorithm 1, gcc -O2), "
                      f"{t_acc:.1f} s of CPU time; host has {os.cpu_count()} logical CPUs",
        }
        # the same oracle loop with the rows shared among all host cores (extra figure)
        reps2, t_acc2, threads = 0, 0.0, 1
        while t_acc2 < args.cpu_seconds / 2 and reps2 < 4000:
            t0 = time.perf_counter()
            threads = oracle.csr_spmv_all_cores(*o_args)[2]
            t_acc2 += time.perf_counter() - t0
            reps2 += 1
        out["cpu_baseline_all_cores"] = {
            "value": round(2.0 * nnz_s * reps2 / t_acc2 / 1e9, 3),
            "unit": "GFLOP/s",
            "cores": threads,
            "kind": "oracle",
            "sample": f"{reps2} {what} (Algorithm 1, rows shared among {threads} OpenMP threads), "
                      f"{t_acc2:.1f} s of wall time",
        }

    B.csr5_free(h)
    print(json.dumps(out))


# HBM traffic (bytes) of one k_spmv launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs,
# scaled by what the same counters read for a plain copy of known size (2.000 and 1.000),
# keyed by (workload, sigma).  profiles/k_spmv_hbm_traffic_pmc.md and
# profiles/k_spmv_huge_mixed_kernel_trace_and_traffic.md have the runs.
MEASURED_TRAFFIC: dict = {
    (2, 16): int((2.000 * 164523.1 + 8014.9) * 1024),     # stencil: 336.9 MB read + 8.2 MB written
    (3, 16): int((2.000 * 176192.6 + 15956.8) * 1024),    # power-law: 360.8 MB read + 16.3 MB written
    (7, 16): int((2.000 * 13661631.8 + 67157.0) * 1024),  # huge_mixed: 27.98 GB read + 68.8 MB written
}


if __name__ == "__main__":
    main()
