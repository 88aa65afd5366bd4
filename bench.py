#!/usr/bin/env python3
"""Benchmark of libcsr5 on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 2] [--sigma 0]
                    [--also 1,3,4,5] [--scale S] [--protocol warm|rotate]

One "step" is one y = A*x on the CSR5 form of the workload (one csr5_spmv_ex
call: the tile kernel plus whatever follows it) with every input resident in
HBM.  The CSR -> CSR5 conversion is timed in the same run and reported in units
of one SpMV.  Prints ONE JSON line.  The headline value is SpMV GFLOP/s =
2*nnz / t of --workload (default: the 27-point stencil, configs[1]); the
`workloads` array of the same line carries the same measurements, shorter, for
the configurations listed in --also (regular and irregular matrices, Section 5.2).

Two timing protocols, both reported for every workload:
  warm    back-to-back SpMVs on one matrix (the paper's protocol, Section 5.1).
          A matrix of up to a few hundred MB is then partly served by the
          256 MB Infinity Cache that sits in front of HBM.
  rotate  back-to-back SpMVs that cycle over k separate device copies of the
          whole problem (matrix, descriptors, x, y), k chosen so that more than
          1.3 GB streams between two uses of the same copy: every byte comes
          from HBM.  No flush kernel and no host synchronisation inside the
          timed region.

Order inside a workload: conversion, correctness check (host), then the
per-kernel series and the paper's best-of-batches protocol, and only then the
timed region proper (W warm-up steps, a device synchronisation, exactly K steps
between two events on the stream the SpMVs run on, a synchronisation).  The
host-side check leaves the GPU idle, and the chip needs some milliseconds of
work to return to its working clocks; the series in between provide them.

The CPU oracle is used for two things only: a correctness check of every timed
configuration, and the `cpu_baseline` figure (the oracle timed as it stands).
"""
from __future__ import annotations

import argparse
import json
import math
import os
import subprocess
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published peak
ROTATE_BYTES = 1.3e9           # streamed between two uses of one copy in the rotating protocol
ROTATE_MAX_COPIES = 8
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "k_spmv_hbm_traffic.txt")


def bytes_model(m, nnz, info, n_ref, vb=8, ib=4):
    """Algorithmic bytes of one SpMV: val + col_idx (vb + 4 B per nonzero), packed
    descriptors, tile_ptr, empty_offset and its per-tile starts, every
    referenced x entry once, y written once.  vb = bytes per value (8 or 4),
    ib = bytes per tile_ptr / empty_offset_ptr entry (8 in the 64-bit index variant)."""
    W, p, pc, E = info["desc_words_per_lane"], info["p"], info["p_complete"], info["empty_offset_len"]
    return ((vb + 4) * nnz + 4 * W * 64 * pc + ib * (p + 1) + ib * (pc + 1) + 4 * E + vb * n_ref + vb * m)


def measured_traffic(workload, sigma, dtype, scale):
    """HBM traffic of one tile-kernel launch from the tracked rocprofv3 --pmc summary
    (offline runs; the file names the commit each line was measured at)."""
    if scale != 1.0 or not os.path.exists(TRAFFIC_FILE):
        return None
    for line in open(TRAFFIC_FILE):
        f = line.split()
        if len(f) >= 7 and not line.startswith("#") and f[0] == str(workload) and f[1] == str(sigma) and f[2] == dtype:
            # FETCH_SIZE reads half of a known copy on gfx950, WRITE_SIZE reads it exactly
            fetch_kib, write_kib = float(f[3]), float(f[4])
            return {"bytes": int((2.0 * fetch_kib + write_kib) * 1024), "read_bytes": int(2.0 * fetch_kib * 1024),
                    "write_bytes": int(write_kib * 1024), "measured_at_commit": f[5], "kernel": f[6]}
    return None


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown CPU"


def git_head():
    try:
        return subprocess.check_output(["git", "-C", ROOT, "rev-parse", "--short", "HEAD"],
                                       stderr=subprocess.DEVNULL).decode().strip()
    except Exception:
        return None


class Problem:
    """One workload on the device: pristine CSR arrays plus working copies."""

    def __init__(self, workload, dtype, scale, dev, zero_columns=False):
        import torch
        from paper_1503_05032_amd import binding as B
        from paper_1503_05032_amd import workloads as wl
        self.workload, self.dtype, self.dev = workload, dtype, dev
        self.f32 = dtype == "f32"
        self.tdt = torch.float32 if self.f32 else torch.float64
        self.vb = 4 if self.f32 else 8
        self.wide = workload == 7
        self.convert_ex = B.csr5s_convert_ex if self.f32 else B.csr5_convert_ex
        self.spmv_ex = B.csr5s_spmv_ex if self.f32 else B.csr5_spmv_ex
        self.spmv_profile = B.csr5s_spmv_profile if self.f32 else B.csr5_spmv_profile
        self.workspace_bytes = B.csr5_workspace_bytes
        if self.wide:
            if self.f32:
                raise SystemExit("bench.py: the 64-bit index variant is double precision only")
            from paper_1503_05032_amd import workloads_device as wd
            A = wd.huge_mixed(dev)
            self.a = None
            self.m, self.n, self.nnz, self.name = A["m"], A["n"], A["nnz"], A["name"]
            self.row_ptr, self.col0, self.val0, self.x = A["row_ptr"], A["col_idx"], A["val"], A["x"]
            self.row_ptr_h = self.row_ptr.cpu().numpy()
            lens = np.diff(self.row_ptr_h)
            self.lens = lens
            self.st = {"row_len_min": int(lens.min()), "row_len_avg": float(lens.mean()),
                       "row_len_max": int(lens.max()), "empty_rows": int((lens == 0).sum())}
            seen = torch.zeros(self.n, dtype=torch.bool, device=dev)
            for e0 in range(0, self.nnz, 1 << 28):
                seen[self.col0[e0:e0 + (1 << 28)].long()] = True
            self.n_ref = int(seen.sum().item())
            del seen
            self.convert_ex, self.workspace_bytes = B.csr5l_convert_ex, B.csr5l_workspace_bytes
        else:
            a = wl.config(workload, scale=scale)
            if zero_columns:          # every gather hits x[0]: what is left of the traffic is not x
                a.col_idx[:] = 0
                a.name += "_all_columns_0"
            if self.f32:
                a.val = a.val.astype(np.float32)
                a.x = a.x.astype(np.float32)
            self.a = a
            self.m, self.n, self.nnz, self.name = a.m, a.n, a.nnz, a.name
            self.st = a.stats()
            self.n_ref = int(np.unique(a.col_idx).size)
            self.row_ptr = torch.from_numpy(a.row_ptr).to(dev)
            self.col0 = torch.from_numpy(a.col_idx).to(dev)        # pristine CSR copies
            self.val0 = torch.from_numpy(a.val).to(dev)
            self.x = torch.from_numpy(a.x).to(dev)

    def describe(self):
        st = self.st
        tag = f"configs[{self.workload - 1}]" if self.workload <= 5 else f"extra workload {self.workload}"
        return (f"{tag} {self.name}: {self.m}x{self.n}, nnz={self.nnz}, "
                f"nnz/row min/avg/max={st['row_len_min']}/{st['row_len_avg']:.2f}/{st['row_len_max']}, "
                f"empty rows={st['empty_rows']}")


def ev():
    import torch
    return torch.cuda.Event(enable_timing=True)


def timed_loop(calls, steps):
    """steps launches back to back, cycling over `calls`; events around the whole series."""
    import torch
    k = len(calls)
    e0, e1 = ev(), ev()
    e0.record()
    for i in range(steps):
        calls[i % k]()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps


def measure(P, sigma_arg, steps, warmup, headline, quick):
    """All measurements of one workload, on a stream of their own: launches on the
    legacy default stream carry its implicit synchronisation with every other
    stream, 1.2 us per SpMV here."""
    import torch
    S = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(S):
        return measure_on(P, sigma_arg, steps, warmup, headline, quick, S.cuda_stream)


def measure_on(P, sigma_arg, steps, warmup, headline, quick, stream):
    """Everything below enqueues on `stream`, torch's current stream (events included)."""
    import torch
    import oracle
    from paper_1503_05032_amd import binding as B
    dev = P.dev
    m, n, nnz = P.m, P.n, P.nnz
    sigma = sigma_arg or B.csr5_sigma_auto(nnz, m)
    wsb = P.workspace_bytes(m, nnz, sigma)
    col, val = P.col0.clone(), P.val0.clone()
    y = torch.empty(m, dtype=P.tdt, device=dev)
    ws = torch.empty(wsb, dtype=torch.uint8, device=dev)

    # ---------------------------------------------------------------- conversion
    conv_ms, conv_alloc_ms = [], []
    h = None
    for it in range(1 if quick else (7 if headline else 5)):
        if h is not None:
            B.csr5_free(h)
        col.copy_(P.col0)
        val.copy_(P.val0)
        torch.cuda.synchronize()
        e0, e1 = ev(), ev()
        e0.record()
        h = P.convert_ex(m, n, nnz, P.row_ptr, col, val, sigma=sigma, workspace=ws, stream=stream,
                         flags=B.CSR5_FLAG_NO_HOST_CHECK)
        e1.record()
        torch.cuda.synchronize()
        conv_ms.append(e0.elapsed_time(e1))
    if not quick:
        for it in range(5 if headline else 3):     # the plain entry point: hipMalloc + host check inside
            c2, v2 = P.col0.clone(), P.val0.clone()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            h2 = P.convert_ex(m, n, nnz, P.row_ptr, c2, v2, sigma=sigma, stream=stream)
            torch.cuda.synchronize()
            conv_alloc_ms.append((time.perf_counter() - t0) * 1e3)
            B.csr5_free(h2)
            del c2, v2
    status = B.csr5_status(h)
    info = B.csr5_get_info(h)
    assert status & 3 == 0, status

    # ---------------------------------------------------------------- correctness of this configuration
    P.spmv_ex(h, P.x, y, stream=stream)
    torch.cuda.synchronize()
    if P.wide:
        # the oracle on a sample of rows (random ones, the longest ones, the first and the last)
        rng = np.random.default_rng(11)
        rp = P.row_ptr_h
        rows_s = np.unique(np.concatenate([rng.integers(0, m, 400), np.argsort(P.lens)[-8:], [0, m - 1]]))
        cs = np.concatenate([P.col0[rp[r]:rp[r + 1]].cpu().numpy() for r in rows_s])
        vs = np.concatenate([P.val0[rp[r]:rp[r + 1]].cpu().numpy() for r in rows_s])
        rp_s = np.concatenate([[0], np.cumsum(P.lens[rows_s])]).astype(np.int32)
        y_ref, s_abs = oracle.csr_spmv(len(rows_s), rp_s, cs, vs, P.x.cpu().numpy())
        rows_dev = torch.from_numpy(rows_s).to(dev)
        parity_scope = f"{len(rows_s)} sampled rows"
    else:
        a = P.a
        y_ref, s_abs = oracle.csr_spmv(m, a.row_ptr, a.col_idx, a.val.astype(np.float64), a.x.astype(np.float64))
        rows_dev = None
        parity_scope = "every row"

    def agrees(y_dev):
        """The benchmark spec's bar, per row: |y - y_ref| <= 1e-12 * sum_j |a_ij x_j| + 1e-300 (1e-5 / 1e-30 in single precision)."""
        got = (y_dev if rows_dev is None else y_dev[rows_dev]).cpu().numpy().astype(np.float64)
        return bool(np.all(np.abs(got - y_ref) <= (1e-5 if P.f32 else 1e-12) * s_abs + (1e-30 if P.f32 else 1e-300)))

    parity_ok = agrees(y)

    B_model = bytes_model(m, nnz, info, P.n_ref, P.vb, 8 if P.wide else 4)
    B_gather = B_model - P.vb * P.n_ref + P.vb * nnz

    # ---------------------------------------------------------------- rotating copies (every byte from HBM)
    copies = int(min(ROTATE_MAX_COPIES, max(1, math.ceil(ROTATE_BYTES / B_model))))
    rot = [(h, P.x, y)]
    keep = []
    for c in range(1, copies):
        rp_c, col_c, val_c, x_c = P.row_ptr.clone(), P.col0.clone(), P.val0.clone(), P.x.clone()
        y_c = torch.empty_like(y)
        ws_c = torch.empty(wsb, dtype=torch.uint8, device=dev)
        h_c = P.convert_ex(m, n, nnz, rp_c, col_c, val_c, sigma=sigma, workspace=ws_c, stream=stream,
                           flags=B.CSR5_FLAG_NO_HOST_CHECK)
        assert B.csr5_status(h_c) & 3 == 0      # also lets the handle learn which launches the matrix needs
        keep.append((rp_c, col_c, val_c, ws_c))
        rot.append((h_c, x_c, y_c))
    torch.cuda.synchronize()
    # (arguments checked and marshalled once: the loops below only make the C call)
    warm_calls = [B.csr5_spmv_bound(h, P.x, y, stream=stream)]
    rot_calls = [B.csr5_spmv_bound(t[0], t[1], t[2], stream=stream) for t in rot]

    # ---------------------------------------------------------------- dominant kernel, HIP events inside the library
    # These series come first on purpose.  After even a short idle spell the chip
    # needs some milliseconds of work to be back at its working clocks (series of 20
    # SpMVs separated by waits: 65-68 us per SpMV; series of 300: 63.5 us from the
    # second series on), and the host-side parity check above is such a spell.  The
    # contract's region below (W warm-up steps, then exactly K timed ones) may be far
    # shorter than that ramp, so it is entered with the GPU already at work.
    reps = min(max(steps, 200), 2000)
    P.spmv_profile(h, P.x, y, reps=reps, stream=stream)      # brings the chip to its working clocks; figures dropped
    ms_tiles, ms_fixup = P.spmv_profile(h, P.x, y, reps=reps, stream=stream)
    # what the memory system alone charges for the tile kernel's streams: a bare read
    # of col_idx, val and the descriptors, without and with the rows of y written
    try:
        floor = B.csr5_stream_floor(h, torch.empty_like(y), reps=reps, stream=stream)
    except B.Csr5Error:
        floor = None        # no complete tile
    P.spmv_ex(h, P.x, y, stream=stream)     # y holds A*x again

    extras = {}
    if not quick:
        # the paper's protocol (Section 5.1) scaled down: best of 10 batches of 100 runs (3 batches
        # for the workloads of the `workloads` array)
        batches = 10 if headline else 3
        best = min(timed_loop(warm_calls, 100) for _ in range(batches))
        extras[f"ms_best_of_{batches}x100"] = round(best, 5)

    # ---------------------------------------------------------------- timed region: exactly `steps` steps
    def run(calls):
        for i in range(warmup):
            calls[i % len(calls)]()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ms = timed_loop(calls, steps)
        return ms, (time.perf_counter() - t0) * 1e3 / steps

    ms_warm, wall_warm = run(warm_calls)
    ms_rot, wall_rot = run(rot_calls) if copies > 1 else (ms_warm, wall_warm)
    if copies > 1:      # every copy's y against the oracle too
        parity_ok = parity_ok and all(agrees(t[2]) for t in rot[1:])

    conv = float(np.median(conv_ms))
    res = {
        "P": P, "h": h, "info": info, "sigma": info["sigma"], "parity_ok": parity_ok, "parity_scope": parity_scope,
        "B_model": B_model, "B_gather": B_gather, "copies": copies,
        "ms_warm": ms_warm, "ms_rot": ms_rot, "wall_warm": wall_warm, "wall_rot": wall_rot,
        "ms_tiles": ms_tiles, "ms_fixup": ms_fixup, "floor": floor, "conv_ms": conv,
        "conv_alloc_ms": float(np.median(conv_alloc_ms)) if conv_alloc_ms else None,
        "extras": extras,
    }
    for t in rot[1:]:
        B.csr5_free(t[0])
    del keep, rot
    return res


def gbs(nbytes, ms):
    return nbytes / (ms * 1e-3) / 1e9


def short_entry(r):
    """One element of the `workloads` array."""
    P = r["P"]
    t = r["ms_warm"]
    traffic = measured_traffic(P.workload, r["sigma"], P.dtype, P.scale)
    e = {
        "workload": P.describe(),
        "nnz": P.nnz, "sigma": r["sigma"], "tiles": r["info"]["p"],
        "parity_ok": r["parity_ok"], "parity_scope": r["parity_scope"] + " against the oracle's Algorithm 1",
        "ms_per_step": round(t, 5),
        "gflops": round(2.0 * P.nnz / (t * 1e-3) / 1e9, 2),
        "bytes_model": r["B_model"],
        "gbs_model": round(gbs(r["B_model"], t), 1),
        "pct_hbm_peak_model": round(100 * gbs(r["B_model"], t) / HBM_PEAK_GBS, 2),
        "rotating": {"copies": r["copies"], "ms_per_step": round(r["ms_rot"], 5),
                     "pct_hbm_peak_model": round(100 * gbs(r["B_model"], r["ms_rot"]) / HBM_PEAK_GBS, 2)},
        "tile_kernel": {"kernel": f"k_spmv<{r['sigma']}>", "ms": round(r["ms_tiles"], 5),
                        "frac": round(gbs(r["B_model"], r["ms_tiles"]) / HBM_PEAK_GBS, 4),
                        "second_kernel_ms": round(r["ms_fixup"], 5)},
        "convert": {"ms": round(r["conv_ms"], 4), "in_spmvs": round(r["conv_ms"] / t, 2),
                    "in_spmvs_with_hipmalloc": round(r["conv_alloc_ms"] / t, 2) if r["conv_alloc_ms"] else None},
    }
    for k, v in r["extras"].items():
        e[k] = v
    if r["floor"]:
        e["tile_kernel"]["stream_floor_ms"] = {"read": round(r["floor"][0], 5), "read_and_y": round(r["floor"][1], 5)}
        e["tile_kernel"]["kernel_over_floor"] = round(r["ms_tiles"] / r["floor"][1], 3)
    if traffic:
        e["tile_kernel"]["traffic"] = traffic["bytes"]
        e["tile_kernel"]["frac_of_peak_on_measured_traffic"] = round(gbs(traffic["bytes"], r["ms_tiles"]) / HBM_PEAK_GBS, 4)
        e["tile_kernel"]["traffic_measured_at_commit"] = traffic["measured_at_commit"]
    return e


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--workload", type=int, default=2,
                    help="1..5 = the five configurations (default 2: the 27-point stencil); 6 = the paper's dense "
                         "2000x2000 matrix; 7 = the 2.2e9-nonzero matrix of the 64-bit index variant, generated "
                         "in GPU memory; 8 = configuration 4 with fewer dense rows (12 M nonzeros)")
    ap.add_argument("--also", default="1,3,4,5",
                    help="further workloads measured after the headline one and reported in the `workloads` "
                         "array of the same line ('' = none)")
    ap.add_argument("--scale", type=float, default=1.0,
                    help="size of --workload relative to its configuration (rows; the stencil's grid edge is "
                         "100*scale^(1/3)); anything but 1 is a size sweep, not the headline")
    ap.add_argument("--sigma", type=int, default=0, help="tile height, 0 = the library's rule")
    ap.add_argument("--dtype", choices=["f64", "f32"], default="f64",
                    help="f64 is the headline; f32 runs the single-precision instantiation")
    ap.add_argument("--protocol", choices=["warm", "rotate"], default="warm",
                    help="which of the two timings is `value` / `ms_per_step` (both are always reported)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=10.0)
    ap.add_argument("--quick", action="store_true", help="one conversion, no extras, no further workloads")
    ap.add_argument("--zero-columns", action="store_true",
                    help="traffic probe: the same matrix with every column index set to 0, so that x costs no "
                         "memory traffic (the difference to the real matrix under rocprofv3 --pmc FETCH_SIZE is "
                         "what the x gathers fetch)")
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

    P = Problem(args.workload, args.dtype, args.scale, dev, zero_columns=args.zero_columns)
    P.scale = args.scale if not args.zero_columns else 0.0      # a probe matrix has no stored traffic figure
    r = measure(P, args.sigma, args.steps, args.warmup, headline=True, quick=args.quick)
    info, h = r["info"], r["h"]
    nnz = P.nnz
    rotate = args.protocol == "rotate"
    ms_per_step = r["ms_rot"] if rotate else r["ms_warm"]
    wall = r["wall_rot"] if rotate else r["wall_warm"]
    gflops = 2.0 * nnz / (ms_per_step * 1e-3) / 1e9
    B_model = r["B_model"]
    achieved = gbs(B_model, r["ms_tiles"])
    traffic = None if P.f32 else measured_traffic(args.workload, info["sigma"], args.dtype, P.scale)

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
            "workload": P.describe(),
            "omega": 64, "sigma": info["sigma"], "tiles": info["p"], "index_bits": 64 if P.wide else 32,
            "desc_words_per_lane": info["desc_words_per_lane"],
            "empty_offset_len": info["empty_offset_len"],
            "protocol": ("rotating over %d device copies of the problem (every byte from HBM)" % r["copies"]) if rotate
                        else "warm: back-to-back SpMVs on one matrix (Section 5.1)",
            "scale": args.scale,
        },
        "parity_ok": r["parity_ok"],
        "spmv": {
            "gflops": round(gflops, 2),
            "bytes_model": B_model,
            "gbs_model": round(gbs(B_model, ms_per_step), 1),
            "pct_hbm_peak_model": round(100 * gbs(B_model, ms_per_step) / HBM_PEAK_GBS, 2),
            "gbs_if_every_gather_missed": round(gbs(r["B_gather"], ms_per_step), 1),
            "wall_ms_per_step": round(wall, 5),
            "warm": {"ms_per_step": round(r["ms_warm"], 5),
                     "pct_hbm_peak_model": round(100 * gbs(B_model, r["ms_warm"]) / HBM_PEAK_GBS, 2)},
            "rotating": {"copies": r["copies"], "ms_per_step": round(r["ms_rot"], 5),
                         "pct_hbm_peak_model": round(100 * gbs(B_model, r["ms_rot"]) / HBM_PEAK_GBS, 2)},
            **r["extras"],
        },
        "convert": {
            "ms_workspace_no_host_check": round(r["conv_ms"], 4),
            "in_spmvs": round(r["conv_ms"] / ms_per_step, 2),
            "ms_with_hipmalloc_and_host_check": round(r["conv_alloc_ms"], 4) if r["conv_alloc_ms"] else None,
            "in_spmvs_with_hipmalloc": round(r["conv_alloc_ms"] / ms_per_step, 2) if r["conv_alloc_ms"] else None,
        },
        "roofline": {
            "kernel": f"k_spmv<{info['sigma']}>",
            "bound": "hbm",
            "achieved": round(achieved, 1),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBS, 4),
            "traffic": traffic["bytes"] if traffic else None,
            "traffic_source": ("offline rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command, "
                               "profiles/k_spmv_hbm_traffic.txt, measured at commit " + traffic["measured_at_commit"])
                              if traffic else None,
            "frac_on_measured_traffic": round(gbs(traffic["bytes"], r["ms_tiles"]) / HBM_PEAK_GBS, 4) if traffic else None,
            "kernel_ms": round(r["ms_tiles"], 5),
            "second_kernel_ms": round(r["ms_fixup"], 5),
            "bytes_per_launch": B_model,
            "stream_floor_ms": ({"read": round(r["floor"][0], 5), "read_and_y": round(r["floor"][1], 5),
                                 "what": "bare read of the same col_idx, val and descriptors by one wavefront per tile "
                                         "(csr5_stream_floor), without and with the rows of y written"}
                                if r["floor"] else None),
            "kernel_over_floor": round(r["ms_tiles"] / r["floor"][1], 3) if r["floor"] else None,
            "timing": "HIP events inside the library around a series of launches of this kernel on one matrix (warm)",
        },
        "commit": git_head(),
    }

    if not args.no_cpu_baseline:
        import oracle
        # the oracle as it stands (sequential Algorithm 1, one core), repeated on the
        # same matrix until about cpu_seconds of work
        if P.wide:      # a bounded part of the matrix: its first rows, about 3e7 nonzeros
            rp = P.row_ptr_h
            m_s = int(np.searchsorted(rp, 30_000_000))
            nnz_s = int(rp[m_s])
            o_args = (m_s, rp[:m_s + 1].astype(np.int32), P.col0[:nnz_s].cpu().numpy(),
                      P.val0[:nnz_s].cpu().numpy(), P.x.cpu().numpy())
            what = f"SpMVs of the first {m_s} rows ({nnz_s} nonzeros) of the same matrix"
        else:
            a = P.a
            nnz_s = nnz
            o_args = (P.m, a.row_ptr, a.col_idx, a.val, a.x)             # the oracle computes in fp64
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
                      f"{t_acc:.1f} s of CPU time; host has {os.cpu_count()} logical CPUs ({cpu_model()})",
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
    entries = [short_entry(r)]
    del r, P
    torch.cuda.empty_cache()

    # ---------------------------------------------------------------- the other configurations, same measurements
    also = [] if args.quick else [int(k) for k in args.also.split(",") if k.strip()]
    for k in also:
        if k == args.workload and args.scale == 1.0:
            continue
        Pk = Problem(k, args.dtype, 1.0, dev)
        Pk.scale = 1.0
        rk = measure(Pk, 0, min(args.steps, 200), min(args.warmup, 20), headline=False, quick=False)
        B.csr5_free(rk["h"])
        entries.append(short_entry(rk))
        del rk, Pk
        torch.cuda.empty_cache()
    entries.sort(key=lambda e: e["workload"])
    out["workloads"] = entries
    out["targets"] = {
        "note": "north-star targets read off the `workloads` array (warm protocol, whole SpMV, bytes model)",
        "stencil_pct_hbm_peak": next((e["pct_hbm_peak_model"] for e in entries if e["workload"].startswith("configs[1]")), None),
        "powerlaw_pct_hbm_peak": next((e["pct_hbm_peak_model"] for e in entries if e["workload"].startswith("configs[2]")), None),
        "max_convert_in_spmvs": max([e["convert"]["in_spmvs"] for e in entries if not e["workload"].startswith("configs[0]")],
                                    default=None),
        "all_parity_ok": all(e["parity_ok"] for e in entries),
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
