#!/usr/bin/env python3
"""Benchmark of the sparse x dense hot path on one MI355X.

Default workload (the one the headline metric is quoted on): f64 CSR SpMV on the 1M x 1M matrix
with lognormal row lengths (~16.8M stored entries), 32-bit pos/crd.  One step = one sp_matmul
through the C ABI.  A, B and C are resident in HBM before the timed region; the steps rotate over
several independent copies so that no step finds its operands in the 256 MB last-level cache
("cold"); the same-buffers ("warm") figure is reported next to it.  Prints one JSON line: effective
GB/s on the algorithmic bytes, the roofline of the dominant kernel (timed with HIP events that the
library records around it), and the CPU checker timed on the host.

Other workloads (--workload cfg1|cfg3|cfg4|cfg5|rowband|sddmm|mttkrp) print the same line for the other configurations.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0

REPS = 5          # timed blocks of `steps` products each: the line carries their median and their minimum


def measured_traffic(workload, width, kernel):
    """HBM bytes per product from the counter runs: the table in profiles/hbm_traffic_per_product.md (one row per workload,
    width and kernel, with the commit it was measured at).  None when there is no row."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic_per_product.md")
    try:
        rows = [[c.strip() for c in l.strip().strip("|").split("|")] for l in open(path) if l.startswith("|")]
    except OSError:
        return None, None
    for r in rows[2:]:
        if len(r) >= 6 and r[0] == workload and r[1] == str(width) and r[2] == str(kernel):
            return float(r[3]), {"commit": r[4], "summary": r[5]}
    return None, None


def timed_blocks(torch, run, steps, reps=REPS):
    """`reps` blocks of exactly `steps` steps, each between its own pair of events: ms per step of every block."""
    out = []
    for _ in range(reps):
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        run(steps)
        e1.record()
        torch.cuda.synchronize()
        out.append(e0.elapsed_time(e1) / steps)
    return out


def median(v):
    v = sorted(v)
    return v[len(v) // 2]


def make_workload(name, small):
    from gen import workloads as W
    if name == "cfg1":
        return W.cfg1_uniform_csr()
    if name == "cfg2":
        return W.cfg2_powerlaw_csr(1 << 16, 1 << 16) if small else W.cfg2_powerlaw_csr()
    if name == "cfg3":
        return W.cfg3_powerlaw_csr_spmm(1 << 16, 1 << 16) if small else W.cfg3_powerlaw_csr_spmm()
    if name == "cfg4":
        return W.cfg4_hypersparse_dcsr(1 << 19, 1 << 19) if small else W.cfg4_hypersparse_dcsr()
    if name == "cfg5":
        return W.cfg5_zipf_csc_spmm(1 << 17, 1 << 17) if small else W.cfg5_zipf_csc_spmm()
    if name == "sddmm":
        w = W.cfg2_powerlaw_csr(1 << 16, 1 << 16) if small else W.cfg2_powerlaw_csr()
        w.N = 64
        w.name = "sddmm"
        return w
    if name == "rowband":
        return W.row_band(1024 if small else 65536, 100 if small else 1000)
    raise SystemExit("unknown workload " + name)


DESCRIPTIONS = {
    "cfg1": "cfg1: CSR SpMV y=A.x, A %(m)dx%(n)d f64, exactly 8 stored entries per row, %(nnz)d stored entries",
    "cfg2": "cfg2: CSR SpMV y=A.x, A %(m)dx%(n)d f64, lognormal row lengths (mean 16, sigma 1.5, clip [1,20000]), %(nnz)d stored entries",
    "cfg3": "cfg3: CSR SpMM C=A.B, A as cfg2 (%(m)dx%(n)d f64, %(nnz)d stored entries), B %(n)dx%(N)d f64 row-major",
    "cfg4": "cfg4: DCSR SpMV y=A.x, A %(m)dx%(n)d f64, 1%% of rows stored, 32 entries each, %(nnz)d stored entries",
    "rowband": "row band (the shape of the paper's SpMV experiment, Section 6.2): SpMV y=A.x, A %(m)dx%(n)d f64, the first rows full, the rest empty, %(nnz)d stored entries",
    "sddmm": "SDDMM X=S.*(A.B) (Section 6.2), S = the cfg2 matrix (%(m)dx%(n)d f64 CSR, %(nnz)d stored entries), A %(m)dx%(N)d, B %(N)dx%(n)d f64 row-major (transposed inside every call)",
    "cfg5": "cfg5: CSC SpMM C=A.B, A %(m)dx%(n)d f32, rank-size Zipf(1.2) column lengths capped at 50000, %(nnz)d stored entries, B %(n)dx%(N)d f32",
}


def algorithmic_bytes(name, w, info, N, vbytes):
    """Compulsory bytes of one product: the storage arrays once, B (x) once, C (y) once."""
    m, n = w.shape
    a = int(info.storageBytes)
    if name == "sddmm":
        return a + m * N * vbytes + n * N * vbytes + w.nnz * vbytes      # S, A, B once, X once
    if name == "cfg4":
        # x: only the touched elements; y: the whole vector is written in overwrite mode
        return a + w.nnz * vbytes + m * vbytes
    return a + n * N * vbytes + m * N * vbytes


def copy_yardstick(torch, sp, dev):
    """GB/s of the library's plain copy kernel on 1 GiB (read + write = 2 GiB of traffic)."""
    nbytes = 1 << 30
    src = torch.empty(nbytes, dtype=torch.uint8, device=dev).fill_(1)
    dst = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    for _ in range(3):
        sp.sp_stream_copy(dst, src)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(10):
        sp.sp_stream_copy(dst, src)
    e1.record()
    torch.cuda.synchronize()
    return 2.0 * nbytes * 10 / (e0.elapsed_time(e1) * 1e-3) / 1e9


def read_yardstick(torch, sp, dev):
    """GB/s of the library's plain read-only streaming kernel on 1 GiB."""
    nbytes = 1 << 30
    src = torch.empty(nbytes, dtype=torch.uint8, device=dev).fill_(1)
    sink = torch.zeros(4, dtype=torch.uint8, device=dev)
    for _ in range(3):
        sp.sp_stream_read(src, sink)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(10):
        sp.sp_stream_read(src, sink)
    e1.record()
    torch.cuda.synchronize()
    return 1.0 * nbytes * 10 / (e0.elapsed_time(e1) * 1e-3) / 1e9


def bench_mttkrp(args, torch, sp, dev):
    """A[i,j] = B[i,k,l] * D[l,j] * C[k,j] (Section 6.3) on a synthetic tensor with the shape, entry count and output
    width of the paper's experiment; one step = one sp_mttkrp."""
    from gen import workloads as W
    t0 = time.time()
    w = (W.tensor3_slices(I=1200, K=900, L=2800, nnz=760_000, k_mean=120, l_mean=300) if args.small else W.tensor3_slices())
    gen_s = time.time() - t0
    fmt = args.format or "dss"
    lt = (0, 1, 1) if fmt.startswith("dss") else (1, 1, 1)
    order = (0, 2, 1) if fmt.endswith("-alt") else (0, 1, 2)
    I, K, L = w.shape
    J, nnz = w.J, w.nnz
    steps = args.steps or 20
    warmup = args.warmup or 3
    ncopies = args.copies or 2
    C_host, D_host = w.factors()
    coords = [torch.from_numpy(c).to(dev) for c in (w.ci, w.ck, w.cl)]
    vals_d = torch.from_numpy(w.vals).to(dev)
    enc = sp.sp_encode(lt, order, args.width, args.width)
    copies, pack_ms = [], []
    for c in range(ncopies):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        B = sp.sp_pack(enc, w.shape, coords, vals_d)
        e1.record()
        torch.cuda.synchronize()
        pack_ms.append(e0.elapsed_time(e1))
        copies.append((B, torch.from_numpy(C_host).to(dev), torch.from_numpy(D_host).to(dev),
                       torch.zeros((I, J), dtype=torch.float64, device=dev)))
    del coords, vals_d
    info = sp.sp_tensor_info(copies[0][0])
    nfib = int(sp.sp_crd(copies[0][0], 1).shape[0])
    abytes = int(info.storageBytes) + (K + L + I) * J * 8          # the storage, C, D and A once each
    flops = 2.0 * J * (nnz + nfib)                                 # a multiply-add per entry and per fibre and column
    acc = bool(args.accumulate)

    def run_steps(k, rotate=True):
        for i in range(k):
            B, Cd, Dd, Ad = copies[i % len(copies)] if rotate else copies[0]
            sp.sp_mttkrp(B, Cd, Dd, Ad, accumulate=acc)

    run_steps(len(copies))             # the first product of a tensor builds its tables and scratch: every copy, whatever --warmup says
    run_steps(warmup)
    cold = timed_blocks(torch, run_steps, steps)
    ms_cold = median(cold)
    run_steps(warmup, rotate=False)
    ms_warm = median(timed_blocks(torch, lambda k: run_steps(k, rotate=False), steps))
    for c in copies:
        sp.sp_tensor_tune(c[0], sp.SP_TUNE_PROFILE, 1)
    run_steps(steps)
    torch.cuda.synchronize()
    tot_ms, launches = 0.0, 0
    for c in copies:
        a, b = sp.sp_profile_read(c[0])
        tot_ms += a
        launches += b
        sp.sp_tensor_tune(c[0], sp.SP_TUNE_PROFILE, 0)
    kernel_ms = tot_ms / max(launches, 1)
    copies[0][3].zero_()
    sp.sp_mttkrp(*copies[0], accumulate=False)
    torch.cuda.synchronize()
    copy_gbs = copy_yardstick(torch, sp, dev)

    cpu, parity = None, None
    if not args.no_cpu:
        import oracle
        t0 = time.time()
        ref, mag = oracle.mttkrp_coo(w.shape, w.ci, w.ck, w.cl, w.vals, C_host, D_host)
        cpu_s = time.time() - t0
        parity = bool(np.all(np.abs(copies[0][3].cpu().numpy() - ref) <= 1e-12 * mag))
        cpu = {"value": abytes / cpu_s / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
               "sample": "the whole workload (%d stored entries x %d columns, one product), one run, %.3f s" % (nnz, J, cpu_s),
               "gflops": flops / cpu_s / 1e9}
    achieved = abytes / (kernel_ms * 1e-3) / 1e9
    kernel_name = "mttkrp_windows_kernel (+ fix-up)"
    out = {
        "metric": "effective HBM GB/s (algorithmic bytes / time per product)",
        "value": abytes / (ms_cold * 1e-3) / 1e9, "unit": "GB/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": ms_cold, "ms_per_step_min": min(cold), "ms_per_step_blocks": cold,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "config": {"workload": "MTTKRP A[i,j]=B[i,k,l]*D[l,j]*C[k,j] (Section 6.3), B %dx%dx%d f64 synthetic with %d stored entries "
                               "(shape, entry count and J=%d of the paper's experiment), stored as %s, pos/crd %d-bit" % (
                                   I, K, L, nnz, J, fmt, args.width),
                   "regime": "cold: rotating over %d copies (%.2f GB)" % (ncopies, ncopies * abytes / 1e9), "kernel": kernel_name,
                   "accumulate": acc, "small": bool(args.small)},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": None if args.small else measured_traffic("mttkrp", args.width, fmt)[0],
                     "traffic_source": None if args.small else measured_traffic("mttkrp", args.width, fmt)[1], "kernel": kernel_name, "kernel_us": kernel_ms * 1e3, "algorithmic_bytes": abytes},
        "cpu_baseline": cpu,
        "gflops": flops / (ms_cold * 1e-3) / 1e9,
        "frac_of_peak": abytes / (ms_cold * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "warm": {"ms_per_step": ms_warm, "value": abytes / (ms_warm * 1e-3) / 1e9},
        "copy_kernel_gbs": copy_gbs,
        "pack": {"ms": sorted(pack_ms)[len(pack_ms) // 2], "mnnz_per_s": nnz / (sorted(pack_ms)[len(pack_ms) // 2] * 1e-3) / 1e6},
        "tensor": dict(w.stats, storage_bytes=int(info.storageBytes), fibres=nfib),
        "parity_ok": parity,
        "gen_s": gen_s,
        "paper_ms": {"note": "the paper's table for its tensor on one Xeon W2135 core, for context only",
                     "DSS": 2340.82, "DSS-alt": 1754.98, "DSS-vec": 1299.97},
    }
    print(json.dumps(out))


def bench_pack(args, torch, sp, dev):
    """The storage builder alone (Section 6.1 measures reading and packing tensors into an all-compressed format): four
    synthetic tensors with the rank and entry count of the paper's table, uniform random distinct coordinates in a
    seeded shuffled order, packed with every level compressed.  The paper prints no shapes except the rank-3 one;
    the others are this benchmark's own choice.  One step = one sp_pack (it synchronises)."""
    from gen import workloads as W, prng
    cases = [("rank 2", (16384, 16384), 1_091_362, 136.0), ("rank 3", (12092, 9184, 28818), 76_879_419, 2055.0),
             ("rank 4", (256, 32, 1024, 2048), 3_309_490, 107.0), ("rank 5", (131072, 8192, 2, 128, 64), 26_021_945, 1728.0)]
    if args.small:
        cases = [(n, s, z // 64, p) for n, s, z, p in cases]
    steps = args.steps or 5
    warmup = args.warmup or 1
    table, t0 = [], time.time()
    cpu, parity = None, None
    for ci, (label, shape, nnz, paper_ms) in enumerate(cases):
        rank = len(shape)
        cells = int(np.prod([int(x) for x in shape]))
        _, lin = W.distinct_sorted_per_segment(W.BASE_SEED + 800 + ci, 1, np.array([nnz], dtype=np.int64), cells)
        lin = lin[prng.permutation(W.BASE_SEED + 800 + ci, 2, nnz)]
        coords, rest = [], lin
        for d in range(rank - 1, -1, -1):
            coords.insert(0, np.ascontiguousarray(rest % shape[d]))
            rest = rest // shape[d]
        vals = prng.uniform_pm1(W.BASE_SEED + 800 + ci, 3, nnz)
        enc = sp.sp_encode((1,) * rank, tuple(range(rank)), args.width, args.width)
        cd = [torch.from_numpy(c).to(dev) for c in coords]
        vd = torch.from_numpy(vals).to(dev)
        for _ in range(warmup):
            sp.sp_pack(enc, shape, cd, vd).free()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            sp.sp_pack(enc, shape, cd, vd).free()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / steps
        T = sp.sp_pack(enc, shape, cd, vd)
        info = sp.sp_tensor_info(T)
        in_bytes = nnz * (8 * rank + 8)
        row = {"tensor": label, "shape": list(shape), "nnz": nnz, "ms": ms, "mnnz_per_s": nnz / ms / 1e3,
               "bytes": int(in_bytes + info.storageBytes), "paper_pack_ms": paper_ms}
        if not args.no_cpu and nnz <= 4_000_000:
            import oracle
            t1 = time.time()
            ref = oracle.pack((1,) * rank, tuple(range(rank)), shape, coords, vals, args.width, args.width)
            row["oracle_ms"] = (time.time() - t1) * 1e3
            ok = all(np.array_equal(sp.sp_pos(T, l).cpu().numpy(), ref.pos[l]) and np.array_equal(sp.sp_crd(T, l).cpu().numpy(), ref.crd[l])
                     for l in range(rank)) and sp.sp_values(T).cpu().numpy().tobytes() == ref.values.tobytes()
            parity = ok if parity is None else (parity and ok)
            cpu = {"value": row["bytes"] / (row["oracle_ms"] * 1e-3) / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
                   "sample": "the %s tensor (%d entries), one run, %.3f s" % (label, nnz, row["oracle_ms"] * 1e-3)}
        table.append(row)
        T.free()
        del cd, vd
    gen_s = time.time() - t0
    top = max(table, key=lambda r: r["nnz"])
    achieved = top["bytes"] / (top["ms"] * 1e-3) / 1e9
    out = {
        "metric": "effective HBM GB/s (algorithmic bytes / time per pack)",
        "value": achieved, "unit": "GB/s", "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": top["ms"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u64", "data": "synthetic",
        "config": {"workload": "sp_pack to an all-compressed format (Section 6.1): %s, %s, %d entries (coordinates int64 per dimension + f64 "
                               "values in, pos/crd %d-bit + values out)" % (top["tensor"], "x".join(str(x) for x in top["shape"]), top["nnz"], args.width),
                   "kernel": "make_keys + radix sort passes + level sweep", "small": bool(args.small)},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": None,
                     "kernel": "whole sp_pack call (allocation and host synchronisations included)", "kernel_us": top["ms"] * 1e3,
                     "algorithmic_bytes": top["bytes"]},
        "cpu_baseline": cpu, "table": table, "parity_ok": parity, "gen_s": gen_s,
        "paper_note": "paper_pack_ms: the pack column of the paper's input table (its real tensors, one Xeon W2135 core), context only",
    }
    print(json.dumps(out))


def bench_spmspm(args, torch, sp, dev):
    """C = A.B with sparse A, B and C, all CSR (Sections 4.4 and 6.2): n x n uniform random operands of density 0.01, the
    sizes of the paper's table; the headline line is the largest one.  One step = one sp_spgemm (it allocates and
    builds C, and synchronises)."""
    from gen import workloads as W
    sizes = [256, 512] if args.small else [1024, 2048, 4096, 8192]
    steps = args.steps or 10
    warmup = args.warmup or 2
    enc = sp.sp_encode((0, 1), (0, 1), args.width, args.width)
    table = []
    t0 = time.time()
    for n in sizes:
        nnz = int(round(0.01 * n * n))
        a = W.uniform_random(n, n, nnz, seed=W.BASE_SEED + 500 + n)
        b = W.uniform_random(n, n, nnz, seed=W.BASE_SEED + 600 + n)
        A = sp.sp_pack(enc, a.shape, [torch.from_numpy(a.rows).to(dev), torch.from_numpy(a.cols).to(dev)], torch.from_numpy(a.vals).to(dev))
        B = sp.sp_pack(enc, b.shape, [torch.from_numpy(b.rows).to(dev), torch.from_numpy(b.cols).to(dev)], torch.from_numpy(b.vals).to(dev))
        sp.sp_tensor_tune(A, sp.SP_TUNE_SPGEMM_KERNEL, args.spgemm_kernel)
        for _ in range(warmup):
            sp.sp_spgemm(A, B, enc).free()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            sp.sp_spgemm(A, B, enc).free()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / steps
        C = sp.sp_spgemm(A, B, enc)
        ia, ib, ic = sp.sp_tensor_info(A), sp.sp_tensor_info(B), sp.sp_tensor_info(C)
        pairs = int((torch.bincount(sp.sp_crd(A, 1).long(), minlength=n) * (sp.sp_pos(B, 1)[1:] - sp.sp_pos(B, 1)[:-1]).long()).sum())
        table.append({"n": n, "ms": ms, "density_c": ic.nvalues / float(n * n), "pairs": pairs, "entries_c": int(ic.nvalues),
                      "bytes": int(ia.storageBytes + ib.storageBytes + ic.storageBytes)})
        last = (a, b, C, n)
    gen_s = time.time() - t0
    a, b, C, n = last
    top = table[-1]
    cpu, parity = None, None
    if not args.no_cpu:
        import oracle
        t0 = time.time()
        ci, cj, cv, mag = oracle.spgemm_coo(a.shape, a.rows, a.cols, a.vals, b.shape, b.rows, b.cols, b.vals)
        cpu_s = time.time() - t0
        P = oracle.pack((0, 1), (0, 1), (n, n), [ci, cj], cv, args.width, args.width)
        M = oracle.pack((0, 1), (0, 1), (n, n), [ci, cj], mag, args.width, args.width)
        parity = bool(np.array_equal(sp.sp_pos(C, 1).cpu().numpy(), P.pos[1]) and np.array_equal(sp.sp_crd(C, 1).cpu().numpy(), P.crd[1])
                      and np.all(np.abs(sp.sp_values(C).cpu().numpy() - P.values) <= 1e-12 * M.values))
        cpu = {"value": top["bytes"] / cpu_s / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
               "sample": "the whole n = %d product (%d pairs), one run, %.3f s" % (n, top["pairs"], cpu_s), "ms": cpu_s * 1e3}
    paper = {1024: 3.7, 2048: 27.0, 4096: 224.4, 8192: 1775.1}
    for r in table:
        r["paper_ms"] = paper.get(r["n"])
    achieved = top["bytes"] / (top["ms"] * 1e-3) / 1e9
    out = {
        "metric": "effective HBM GB/s (algorithmic bytes / time per product)",
        "value": achieved, "unit": "GB/s", "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": top["ms"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "config": {"workload": "SpMSpM C=A.B, all CSR f64 (Sections 4.4, 6.2): n x n uniform random A and B of density 0.01, n = %d, "
                               "%d pairs -> %d stored entries of C, pos/crd %d-bit" % (n, top["pairs"], top["entries_c"], args.width),
                   "kernel": {1: "spgemm_expand_kernel + radix sort + sum_runs_kernel + level build",
                              2: "spgemm_ws_count_kernel + scan + spgemm_ws_numeric_panels_kernel (4 waves per row)",
                              3: "spgemm_ws_count_kernel + scan + spgemm_ws_numeric_kernel (1 wave per row)",
                              5: "spgemm_ws_count_kernel + scan + spgemm_ws_numeric_entries_kernel (16 waves per row, order of the additions not fixed)",
                              }.get(args.spgemm_kernel, "spgemm_ws_count_kernel + scan + spgemm_ws_numeric_wide_kernel (16 waves per row; 4 below 8192 columns)"),
                   "small": bool(args.small)},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": None, "kernel": "whole sp_spgemm call (allocation and host synchronisations included)",
                     "kernel_us": top["ms"] * 1e3, "algorithmic_bytes": top["bytes"]},
        "cpu_baseline": cpu,
        "table": table,
        "parity_ok": parity,
        "gen_s": gen_s,
        "paper_note": "paper_ms: the paper's table on one Xeon W2135 core, for context only",
    }
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="timed products (default: 300 for SpMV, 20 for SpMM)")
    ap.add_argument("--warmup", type=int, default=0)
    ap.add_argument("--workload", default="cfg2", choices=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5", "rowband", "sddmm", "mttkrp", "spmspm", "pack"])
    ap.add_argument("--format", default="", choices=["", "csr", "dcsr", "cdr", "dense", "dss", "dss-alt", "sss", "sss-alt"],
                    help="store the workload's matrix under another row-major encoding (rowband: csr, dcsr or cdr as in the paper's table); "
                         "mttkrp: dss (default) / dss-alt as in the paper's table, sss / sss-alt with a compressed outer level")
    ap.add_argument("--copies", type=int, default=0, help="independent copies of A, B, C rotated through (cold regime)")
    ap.add_argument("--width", type=int, default=32, choices=[32, 64], help="pos/crd bit width")
    ap.add_argument("--kernel", type=int, default=0, help="SpMV kernel: 0 auto, 1 lanes-per-row, 2 streaming, 3 column-segmented streaming, 4 binned by column panel and row block")
    ap.add_argument("--csc-mode", type=int, default=0, help="column-major tensors: 0 auto, 1 scatter with atomics, 2 cached transpose")
    ap.add_argument("--spmm-kernel", type=int, default=0, help="SpMM kernel: 0 auto, 1 one column per lane, 2 16-byte loads with a wave per row, 3 16-byte loads cut by entries")
    ap.add_argument("--spgemm-kernel", type=int, default=0, help="SpMSpM: 0 auto, 1 pairs through the storage builder, 2 / 3 / 4 LDS workspace per row with 4 / 1 / 16 waves, 5 = 16 waves dealing out the entries (fastest, not bit-reproducible)")
    ap.add_argument("--accumulate", action="store_true", help="C += A.B instead of C = A.B")
    ap.add_argument("--small", action="store_true", help="scaled-down matrix (for quick checks)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU baseline leg")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU; --gpus %d is not supported "
              "(no collectives or sharding are part of it)" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2202_04305_amd as sp

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    name = args.workload
    if name == "mttkrp":
        return bench_mttkrp(args, torch, sp, dev)
    if name == "spmspm":
        return bench_spmspm(args, torch, sp, dev)
    if name == "pack":
        return bench_pack(args, torch, sp, dev)
    t0 = time.time()
    w = make_workload(name, args.small)
    gen_s = time.time() - t0
    out = bench_matmul(args, torch, sp, dev, name, w, args.width, full=True)
    out["gen_s"] = gen_s
    # the paper's default widths are 64 bits (width 0 = native), its best strategies use 32: both are measured on the headline workload
    if name == "cfg2" and args.width == 32 and not args.kernel and not args.format:
        o = bench_matmul(args, torch, sp, dev, name, w, 64, full=False)
        out["w64"] = {"ms_per_step": o["ms_per_step"], "ms_per_step_min": o["ms_per_step_min"], "value": o["value"], "unit": "GB/s",
                      "frac": o["roofline"]["frac"], "kernel_us": o["roofline"]["kernel_us"], "algorithmic_bytes": o["roofline"]["algorithmic_bytes"],
                      "kernel": o["roofline"]["kernel"], "storage_multiplier": o["storage_multiplier"], "inspector_ms": o["inspector_ms"],
                      "note": "the same workload with 64-bit pos/crd (the paper's native width)"}
    print(json.dumps(out))


SPMV_KERNELS = {1: "spmv_rows_kernel", 2: "spmv_stream_kernel (+ fix-up)",
                3: "column-segmented SpMV: spmv_stream_kernel on the panel copy + fix-up + spmv_panel_sum_kernel",
                4: "binned SpMV: spmv_bins_multiply_kernel + spmv_bins_reduce_kernel"}


def bench_matmul(args, torch, sp, dev, name, w, wbits, full):
    """One workload at one pos/crd width: pack the copies, run the inspector on every one of them (sp_prepare), then time
    REPS blocks of `steps` products.  full = False leaves out the extras (warm regime, graph replay, CPU leg)."""
    m, n = w.shape
    nnz, N = w.nnz, w.N
    tdtype = torch.float64 if w.dtype == np.float64 else torch.float32
    vbytes = 8 if w.dtype == np.float64 else 4
    sddmm = name == "sddmm"
    B_host = w.dense_operand(N)              # n x N; for SDDMM its transpose is the K x n operand B
    spmv = N == 1
    steps = args.steps or (300 if spmv else 20)
    warmup = args.warmup or (30 if spmv else 3)
    ncopies = args.copies or (6 if spmv else 2)

    rows_d = torch.from_numpy(w.rows).to(dev)
    cols_d = torch.from_numpy(w.cols).to(dev)
    vals_d = torch.from_numpy(w.vals).to(dev)
    lt, order = w.level_types, w.dim_ordering
    if args.format:
        lt, order = {"csr": (0, 1), "dcsr": (1, 1), "cdr": (1, 0), "dense": (0, 0)}[args.format], (0, 1)
    enc = sp.sp_encode(lt, order, wbits, wbits)
    copies = []
    pack_ms, inspector_ms = [], []
    for c in range(ncopies):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        A = sp.sp_pack(enc, w.shape, [rows_d, cols_d], vals_d)
        e1.record()
        torch.cuda.synchronize()
        pack_ms.append(e0.elapsed_time(e1))
        sp.sp_tensor_tune(A, sp.SP_TUNE_SPMV_KERNEL, args.kernel)
        sp.sp_tensor_tune(A, sp.SP_TUNE_CSC_MODE, args.csc_mode)
        sp.sp_tensor_tune(A, sp.SP_TUNE_SPMM_KERNEL, args.spmm_kernel)
        if not sddmm:
            # the inspector: kernel choice, regrouped copies, scratch.  Once per tensor, outside every timed region, timed on its own.
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            sp.sp_prepare(A, N)
            e1.record()
            torch.cuda.synchronize()
            inspector_ms.append(e0.elapsed_time(e1))
        if sddmm:
            from gen import prng
            A_host = prng.uniform_pm1(w.seed, 8, m * N, dtype=w.dtype).reshape(m, N)
            Bd = (torch.from_numpy(A_host).to(dev), torch.from_numpy(np.ascontiguousarray(B_host.T)).to(dev))
            Cd = torch.zeros(nnz, dtype=tdtype, device=dev)
        else:
            Bd = torch.from_numpy(B_host[:, 0].copy() if spmv else B_host).to(dev)
            Cd = torch.zeros(m if spmv else (m, N), dtype=tdtype, device=dev)
        copies.append((A, Bd, Cd))
    del rows_d, cols_d, vals_d
    info = sp.sp_tensor_info(copies[0][0])
    abytes = algorithmic_bytes(name, w, info, N, vbytes)
    flops = 2.0 * nnz * N
    acc = bool(args.accumulate)

    def run_steps(k, rotate=True):
        for i in range(k):
            A, Bd, Cd = copies[i % len(copies)] if rotate else copies[0]
            if sddmm:
                sp.sp_sddmm(A, Bd[0], Bd[1], Cd)
            else:
                sp.sp_matmul(A, Bd, Cd, accumulate=acc)

    run_steps(len(copies))     # one product on every copy whatever --warmup says (SDDMM has no inspector call: its first call allocates)
    run_steps(warmup)
    cold = timed_blocks(torch, run_steps, steps)
    ms_cold = median(cold)
    lazy = sum(sp.sp_tensor_info(A).lazyPrepares for A, _, _ in copies)
    ms_warm, graph_ms = None, None
    if full:
        run_steps(warmup, rotate=False)
        ms_warm = median(timed_blocks(torch, lambda k: run_steps(k, rotate=False), steps))
        # the same rotation recorded once into a HIP graph and replayed: what a caller with a launch-bound loop would do
        if not sddmm:
            g = torch.cuda.CUDAGraph()
            per_graph = min(steps, 100)
            with torch.cuda.graph(g):
                run_steps(per_graph)
            g.replay()
            graph_ms = median(timed_blocks(torch, lambda k: [g.replay() for _ in range(k)], max(1, steps // per_graph))) / per_graph
            del g

    # the kernels that stream A, timed by the library's own event pairs around them on the stream they run on (separate pass)
    for A, _, _ in copies:
        sp.sp_tensor_tune(A, sp.SP_TUNE_PROFILE, 1)
    run_steps(steps)
    torch.cuda.synchronize()
    tot_ms, launches = 0.0, 0
    for A, _, _ in copies:
        a, b = sp.sp_profile_read(A)
        tot_ms += a
        launches += b
        sp.sp_tensor_tune(A, sp.SP_TUNE_PROFILE, 0)
    kernel_ms = tot_ms / max(launches, 1)

    # one clean product on copy 0 for the parity check below
    if acc:
        copies[0][2].zero_()
    if not sddmm:
        sp.sp_matmul(copies[0][0], copies[0][1], copies[0][2], accumulate=False)
    torch.cuda.synchronize()

    copy_gbs = copy_yardstick(torch, sp, dev)
    read_gbs = read_yardstick(torch, sp, dev)

    # CPU checker on the same input, one host core; also the parity check of this very run
    cpu = None
    parity = None
    if full and not args.no_cpu:
        import oracle
        reps = 3 if spmv else 1
        times = []
        for _ in range(reps):
            t0 = time.time()
            if sddmm:
                xref, xmag = oracle.sddmm_coo(w.shape, w.rows, w.cols, w.vals, A_host, np.ascontiguousarray(B_host.T))
            else:
                Cref, mag = oracle.matmul_coo(w.shape, w.rows, w.cols, w.vals, B_host)
            times.append(time.time() - t0)
        cpu_s = sorted(times)[len(times) // 2]
        if sddmm:     # per-triple results into storage order: the checker packs them under the same encoding
            Cref = oracle.pack(w.level_types, w.dim_ordering, w.shape, [w.rows, w.cols], xref, wbits, wbits).values.reshape(-1, 1)
            mag = oracle.pack(w.level_types, w.dim_ordering, w.shape, [w.rows, w.cols], xmag, wbits, wbits).values.reshape(-1, 1)
            Cg = copies[0][2].cpu().numpy().reshape(-1, 1).astype(np.float64)
        else:
            Cg = copies[0][2].cpu().numpy().reshape(m, N).astype(np.float64)
        tol = 1e-12 if vbytes == 8 else 1e-5
        parity = bool(np.all(np.abs(Cg - Cref) <= tol * mag))
        cpu = {"value": abytes / cpu_s / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
               "sample": "the whole workload (%d stored entries x %d columns, one product), median of %d, %.3f s per product" % (
                   nnz, N, reps, cpu_s),
               "gflops": flops / cpu_s / 1e9}

    # which kernel ran: the library's own answer for SpMV (sp_tensor_info), the dispatch rule for the rest
    kk = 0
    if spmv:
        kk = int(info.spmvKernel)
        kernel_name = SPMV_KERNELS.get(kk, "spmv kernel %d" % kk)
        if lt[1] == 0:
            kernel_name = "dense_rows_kernel"
    else:
        kernel_name = "sddmm_rows_vec_kernel" if sddmm else "spmm_scatter_kernel" if (name == "cfg5" and args.csc_mode == 1) else (
            "spmm_rows_kernel" if args.spmm_kernel == 1 else "spmm_rows_vec_kernel" if args.spmm_kernel == 2 else "spmm_windows_vec_kernel (+ fix-up)")
    achieved = abytes / (kernel_ms * 1e-3) / 1e9
    traffic, traffic_source = (None, None) if args.small else measured_traffic(name, wbits, kk if spmv else 0)
    # what the kernel's own design has to move (the binned SpMV streams 28 bytes per stored entry instead of CSR's 12), priced at
    # the rate of the plain read-only streaming kernel of this run (optimistic for the part that is written): how close the
    # kernel is to the floor of its design, next to `frac`
    design_bytes = abytes
    if spmv and kk == 4:
        design_bytes = nnz * (2 * vbytes + 2 * 2 + vbytes) + n * vbytes + m * vbytes
    floor_us = design_bytes / read_gbs * 1e-3
    wl = DESCRIPTIONS[name] % dict(m=m, n=n, nnz=nnz, N=N) + ", pos/crd %d-bit" % wbits
    if args.format:
        wl += ", stored as " + args.format
    out = {
        "metric": "effective HBM GB/s (+GFLOP/s) for f64 CSR SpMV/SpMM, fraction of peak",
        "metric_note": "value = algorithmic bytes / time per product (median of %d blocks of `steps` products); GFLOP/s in gflops, fraction of the 8 TB/s peak in frac_of_peak" % REPS,
        "value": abytes / (ms_cold * 1e-3) / 1e9,
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": ms_cold,
        "ms_per_step_min": min(cold),
        "ms_per_step_blocks": cold,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f64" if vbytes == 8 else "f32",
        "data": "synthetic",
        "config": {"workload": wl, "regime": "cold: rotating over %d copies of A, B, C (%.2f GB)" % (
            ncopies, ncopies * abytes / 1e9), "kernel": kernel_name, "accumulate": acc, "small": bool(args.small)},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_source,
                     "kernel": kernel_name, "kernel_us": kernel_ms * 1e3, "algorithmic_bytes": abytes,
                     "design_bytes": design_bytes, "floor_us": floor_us, "frac_of_floor": floor_us / (kernel_ms * 1e3),
                     "floor_note": "design_bytes = what the kernel's data layout streams per product; floor_us = that at the plain read-only streaming kernel's rate of this run (read_kernel_gbs)"},
        "cpu_baseline": cpu,
        "gflops": flops / (ms_cold * 1e-3) / 1e9,
        "frac_of_peak": abytes / (ms_cold * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "inspector_ms": None if not inspector_ms else median(inspector_ms),
        "inspector_note": "sp_prepare per tensor (kernel choice, regrouped copy, scratch), outside the timed region; break-even after inspector_ms / ms_per_step products",
        "lazy_prepares": lazy,      # products that had to build something first (sp_tensor_info): none after sp_prepare
        "storage_multiplier": (info.storageBytes + info.derivedBytes) / float(info.storageBytes),
        "storage_bytes": int(info.storageBytes), "derived_bytes": int(info.derivedBytes),
        "warm": None if ms_warm is None else {"ms_per_step": ms_warm, "value": abytes / (ms_warm * 1e-3) / 1e9,
                                               "note": "same buffers every step: part of the working set stays in the last-level cache"},
        "graph_replay": None if graph_ms is None else {"ms_per_step": graph_ms, "value": abytes / (graph_ms * 1e-3) / 1e9,
                                                       "note": "the same products recorded once into a HIP graph and replayed (cold rotation)"},
        "copy_kernel_gbs": copy_gbs,
        "read_kernel_gbs": read_gbs,
        "frac_of_copy": abytes / (ms_cold * 1e-3) / 1e9 / copy_gbs,
        "pack": {"ms": median(pack_ms), "mnnz_per_s": nnz / (median(pack_ms) * 1e-3) / 1e6},
        "matrix": dict(w.stats, storage_bytes=int(info.storageBytes)),
        "parity_ok": parity,
    }
    for A, _, _ in copies:
        A.free()
    return out


if __name__ == "__main__":
    main()
