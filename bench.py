#!/usr/bin/env python3
"""Benchmark of the position-space sparse x dense path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--tile T]

A step is one complete product through the C ABI: position cut, tile kernel, carry fix-up.  Inputs
are synthetic, seeded, resident in HBM before the timed region.  One JSON line is printed:
whole-job throughput (`value`, GFLOP/s = 2*nnz*k / time), the roofline record of the dominant
kernel (algorithmic bytes / its own event-timed duration, against 8 TB/s) and the CPU oracle timed
on the host cores of the same machine.

Workloads (names of the evaluated configurations):
  powerlaw (default)  CSR SpMV, 2M x 2M, truncated Zipf(1.8) row lengths in [1, 200000]
  stencil             CSR SpMV, 27-point stencil on 160^3
  uniform10           CSR SpMV, 1024 x 1024, 10 per row (launch-latency bound)
  spmm                CSR SpMM, 1M x 1M with 16 per row, B 1M x 128
  bcsr_spmv           BCSR 4x4 SpMV, 250k x 250k blocks, 8 blocks per block row
  bcsr_spmm           BCSR 4x4 SpMM with 64 dense columns
  uniform28           CSR SpMV, 2M x 2M, exactly 28 per row at uniform random columns (the uniform
                      matrix of the power-law matrix's size class, for the per-nnz comparison)
  spmm_dense32        CSR SpMM, 100k x 100k with 1000 random nonzeros per row times a dense 100k x 32 operand (the
                      shape of the paper's locality experiment, Section 8.6)
  mttkrp              MTTKRP A(i,j) = B(i,k,l) C(k,j) D(l,j): B 500k x 100k x 100k in three compressed levels,
                      ~4M fibers, ~46M nonzeros (Zipf leaves per fiber), j = 64 (the paper's third kernel;
                      synthetic stand-in for the FROSTT tensors it uses)
  dcsr                SpMV on a hypersparse DCSR operand: 2^26 rows of which 10^6 are stored, Zipf row lengths
                      (alpha 1.8, <= 50 000), 2^21 columns, ~21 M nonzeros; --cut positions|rows
  fewlong             CSR SpMV, 100 x 100000 with 10000 per row (Section 8.5: too few rows for a
                      row-split kernel to fill the GPU)
  expskew             CSR SpMV, 65536 x 1M, 4M nonzeros, row lengths ~ base**rank shuffled
                      (Section 8.4; --skew-base, default 1.00256)
  copy                not a product: a plain device copy of 1 GiB, the calibration kernel for the
                      rocprofv3 FETCH_SIZE / WRITE_SIZE counters and the practical HBM ceiling
  stream_read         not a product: 1 GiB read once with 16-byte non-temporal loads (the read-only ceiling)
  gather              not a product: 2^26 gathers of 4-byte words at seeded uniform random indices from a table
                      of --table-mb MB (default 8) in global memory: the cost of one gather of x
  gather_lds          not a product: the same gathers from a table of 32736 floats that each workgroup holds
                      in on-chip memory (the column-slab kernel's way of reading x)
"""
import argparse
import json
import os
import statistics
import sys
import time

import numpy as np

HBM_PEAK_GBS = 8000.0

def profile_traffic(workload, tile, col_passes, path="csr"):
    """HBM-side bytes per product of the timed kernels, read from the rocprofv3 summaries under profiles/
    (two --pmc runs, FETCH_SIZE and WRITE_SIZE, scaled by the copy-kernel calibration).  A summary carries a line
        bench-key: workload=W path=P tile=T col_passes=Q traffic_bytes=N
    for the configuration it was measured on.  Returns (bytes, file name) or (None, note) when no summary
    matches the configuration that is being run."""
    import glob
    import re

    here = os.path.dirname(os.path.abspath(__file__))
    want = {"workload": workload, "path": path, "tile": str(tile), "col_passes": str(col_passes)}
    for f in sorted(glob.glob(os.path.join(here, "profiles", "*.txt"))):
        for line in open(f, errors="replace"):
            if not line.startswith("bench-key:"):
                continue
            kv = dict(re.findall(r"(\w+)=(\S+)", line))
            if all(kv.get(k) == v for k, v in want.items()) and "traffic_bytes" in kv:
                return int(kv["traffic_bytes"]), os.path.basename(f)
    return None, "no rocprofv3 summary under profiles/ for workload=%s path=%s tile=%s col_passes=%s" % (
        workload, path, tile, col_passes)



WORKLOADS = {
    "uniform10": (1, "csr_spmv"),
    "powerlaw": (2, "csr_spmv"),
    "stencil": (3, "csr_spmv"),
    "spmm": (4, "csr_spmm"),
    "bcsr_spmv": (5, "bcsr_spmv"),
    "bcsr_spmm": (5, "bcsr_spmm"),
    "uniform28": (0, "csr_spmv"),
    "spmm_dense32": (0, "csr_spmm"),
    "mttkrp": (0, "mttkrp"),
    "dcsr": (0, "dcsr"),
    "fewlong": (0, "csr_spmv"),
    "expskew": (0, "csr_spmv"),
    "copy": (0, "copy"),
    "stream_read": (0, "calibration"),
    "gather": (0, "calibration"),
    "gather_lds": (0, "calibration"),
}


def algorithmic_bytes(kind, A, k):
    """Bytes the method must move once: the sparse operand, the dense operand once, the output once.
    For SpMM / BCSR SpMM the second figure charges one dense row per stored position (no reuse)."""
    rows, cols, nnz = A.rows, A.cols, A.nnz
    if kind == "csr_spmv":
        b = 8 * nnz + 4 * (rows + 1) + 4 * cols + 4 * rows
        return b, b
    if kind == "csr_spmm":
        a = 8 * nnz + 4 * (rows + 1)
        return a + 4 * k * cols + 4 * k * rows, a + 4 * k * nnz + 4 * k * rows
    if kind == "bcsr_spmv":
        b = (4 * A.bs * A.bs + 4) * nnz + 4 * (rows + 1) + 4 * A.bs * cols + 4 * A.bs * rows
        return b, b
    if kind == "bcsr_spmm":
        a = (4 * A.bs * A.bs + 4) * nnz + 4 * (rows + 1)
        w = 4 * A.bs * k
        return a + w * cols + w * rows, a + w * nnz + w * rows
    raise ValueError(kind)


def input_hash(*arrays):
    """Hash of the generated operands: the same seed must give the same bytes on every machine."""
    import hashlib

    h = hashlib.blake2b(digest_size=8)
    for a in arrays:
        h.update(np.ascontiguousarray(a).view(np.uint8).reshape(-1).data)
    return h.hexdigest()


def time_cpu(fn, budget_s=10.0, max_runs=25):
    """One warm-up call, then repeated calls for about budget_s seconds of CPU work (3..max_runs calls);
    returns (median seconds, calls)."""
    t = time.perf_counter()
    fn()
    first = time.perf_counter() - t
    n = int(max(3, min(max_runs, budget_s / max(first, 1e-6))))
    ts = []
    for _ in range(n):
        t = time.perf_counter()
        fn()
        ts.append(time.perf_counter() - t)
    return statistics.median(ts), n


def flops(kind, A, k):
    per = 2 * (A.bs * A.bs)
    return per * A.nnz * (k if kind.endswith("spmm") else 1)


def bench_copy(args, torch):
    """Plain copy of 2^28 floats (1 GiB read + 1 GiB written per launch) with torch's copy kernel."""
    n = 1 << 28
    src = torch.ones(n, device="cuda:0")
    dst = torch.empty(n, device="cuda:0")
    stream = torch.cuda.current_stream()
    for _ in range(args.warmup):
        dst.copy_(src)
    torch.cuda.synchronize()
    ts = []
    for _ in range(args.steps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        dst.copy_(src)
        e1.record(stream)
        e1.synchronize()
        ts.append(e0.elapsed_time(e1))
    avg = sum(ts) / len(ts)
    print(json.dumps({"metric": "device copy GB/s (read + written bytes)", "value": round(8.0 * n / (avg * 1e-3) / 1e9, 2),
                      "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
                      "ms_per_step": round(avg, 6), "bytes_read": 4 * n, "bytes_written": 4 * n,
                      "config": {"workload": "copy: 2^28 fp32 elements, torch copy kernel"}}))


def cu_trace_report(args, torch, psk, A, s, tile, col_passes, path, stream):
    """Per-CU busy time from the instrumented build: every workgroup records start, end (100 MHz wall clock) and
    the compute unit it ran on; a CU's busy time is the length of the union of its workgroups' intervals."""
    SLAB_REC = 1024            # PSK_CU_TRACE_SLAB_RECORDS: the slab pair kernel's records come first
    nrec = SLAB_REC + max(A.rows // 4 + 8, A.nnz // 256 + 64, A.rows // 256 + 8)
    trace = torch.zeros(3 * nrec, dtype=torch.int64, device="cuda:0")
    psk.psk_cu_trace_set(trace)
    ws1 = psk.workspace(psk.PSK_OP_SPMV_CSR, A.rows, A.nnz, tile=2048, device="cuda:0")
    variants = [
        ("position cut, tile 2048, one pass (k_spmv_pos)",
         lambda ph: psk.psk_spmv_csr(A.rows, A.cols, A.nnz, s["pos"], s["crd"], s["vals"], s["dense"], s["out"], tile=2048,
                                     col_passes=1, phases=ph, ws=ws1, stream=stream)),
        ("row split, wave per row (k_spmv_wave_per_row)",
         lambda ph: psk.psk_spmv_csr_rowsplit(A.rows, A.cols, A.nnz, s["pos"], s["crd"], s["vals"], s["dense"], s["out"],
                                              variant=1, stream=stream)),
        ("row split, thread per row (k_spmv_thread_per_row)",
         lambda ph: psk.psk_spmv_csr_rowsplit(A.rows, A.cols, A.nnz, s["pos"], s["crd"], s["vals"], s["dense"], s["out"],
                                              variant=0, stream=stream)),
    ]
    if path == "slab":
        variants.insert(0, ("column-slab path, pair sums (k_slab_pairs) + row sums (k_spmv_pos, unit values)",
                            lambda ph: psk.psk_spmv_slab(s["slab"], s["dense"], s["out"], phases=ph, ws=s["slab_ws"], stream=stream)))
    out = []
    for name, fn in variants:
        fn(psk.PSK_PHASE_PARTITION | psk.PSK_PHASE_MAIN)           # warm-up, and the table for the traced launch
        torch.cuda.synchronize()
        trace.zero_()
        torch.cuda.synchronize()
        fn(psk.PSK_PHASE_MAIN)
        torch.cuda.synchronize()
        t = trace.cpu().numpy().reshape(-1, 3)
        if name.startswith("column-slab"):
            pair_part = t[:SLAB_REC]
            pair_part = pair_part[pair_part[:, 1] > 0]
            pair_span = float((pair_part[:, 1].max() - pair_part[:, 0].min()) * 0.01)
        t = t[t[:, 1] > 0]
        t0, t1, hw = t[:, 0], t[:, 1], t[:, 2]
        cu = ((hw >> 32) & 0xF) * 1024 + ((hw >> 13) & 7) * 32 + ((hw >> 12) & 1) * 16 + ((hw >> 8) & 0xF)
        busy = []
        for k in np.unique(cu):
            m = cu == k
            a, b = t0[m], t1[m]
            o = np.argsort(a)
            a, b = a[o], b[o]
            end = np.maximum.accumulate(b)
            gap = np.maximum(0, a[1:] - end[:-1])                  # idle time between consecutive intervals
            busy.append((end[-1] - a[0] - gap.sum()) * 0.01)       # ticks of 10 ns -> us
        busy = np.array(busy)
        dur = (t1 - t0) * 0.01
        out.append({"schedule": name, "workgroups": int(len(t)), "compute_units": int(len(busy)),
                    "span_us": round(float((t1.max() - t0.min()) * 0.01), 1),
                    "cu_busy_us": {"mean": round(float(busy.mean()), 1), "max": round(float(busy.max()), 1),
                                   "min": round(float(busy.min()), 1)},
                    "max_over_mean": round(float(busy.max() / busy.mean()), 3),
                    "workgroup_us": {"median": round(float(np.median(dur)), 2), "p99": round(float(np.percentile(dur, 99)), 2),
                                     "max": round(float(dur.max()), 2)}})
        if name.startswith("column-slab"):
            out[-1]["pair_kernel_workgroups"] = int(len(pair_part))
            out[-1]["pair_kernel_span_us"] = round(pair_span, 1)
    psk.psk_cu_trace_set(None)
    print(json.dumps({"metric": "per-CU busy time of the SpMV schedules (instrumented build; ratios, not absolute times)",
                      "config": {"workload": "%s: %d x %d, nnz %d" % (args.workload, A.rows, A.cols, A.nnz)},
                      "schedules": out}))


def bench_calibration(args, torch, psk):
    """The machine rates the design is argued with, from the library's calibration kernels."""
    dev = torch.device("cuda:0")
    stream = torch.cuda.current_stream()
    rng = np.random.default_rng(200100532)
    if args.workload == "stream_read":
        bufs = [torch.ones(1 << 28, device=dev) for _ in range(2)]          # two buffers of 1 GiB, alternated
        sink = torch.zeros(64, device=dev)
        work, unit, per = 4.0 * (1 << 28), "GB/s", "bytes"
        what = "stream_read: 2^28 fp32 read once per launch with 16-byte non-temporal loads"
        run = lambda i: psk.psk_calibrate_stream_read(bufs[i % 2], sink, stream=stream)
    elif args.workload == "gather":
        n = 1 << 26
        elems = max(1024, int(args.table_mb * (1 << 20) / 4))
        table = torch.zeros(elems, device=dev)
        idx = [torch.from_numpy(rng.integers(0, elems, size=n, dtype=np.int32)).to(dev) for _ in range(2)]
        out = torch.empty(n // 8, device=dev)
        work, unit, per = float(n), "Ggather/s", "gathers"
        what = "gather: 2^26 uniform random 4-byte gathers from a table of %.2f MB in global memory" % (elems * 4 / 2 ** 20)
        run = lambda i: psk.psk_calibrate_gather(table, idx[i % 2], out, stream=stream)
    else:
        n = 1 << 26
        elems = 32736
        table = torch.zeros(elems, device=dev)
        idx = [torch.from_numpy(rng.integers(0, elems, size=n, dtype=np.int16)).to(dev) for _ in range(2)]
        out = torch.empty(256 * 1024, device=dev)
        work, unit, per = float(n), "Ggather/s", "gathers"
        what = "gather_lds: 2^26 uniform random gathers from a table of 32736 floats held in LDS by each workgroup"
        run = lambda i: psk.psk_calibrate_gather_lds(table, idx[i % 2], out, stream=stream)
    for i in range(args.warmup):
        run(i)
    torch.cuda.synchronize()
    ts = []
    for i in range(args.steps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        run(i)
        e1.record(stream)
        e1.synchronize()
        ts.append(e0.elapsed_time(e1))
    med = statistics.median(ts)
    print(json.dumps({"metric": "calibration: %s per second" % per, "value": round(work / (med * 1e-3) / 1e9, 3), "unit": unit,
                      "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(med, 6),
                      "ms_min": round(min(ts), 6), "ps_per_item": round(med * 1e9 / work, 3),
                      "config": {"workload": what}}))


def bench_mttkrp(args, torch, psk, wl):
    """MTTKRP on the synthetic three-level tensor; same record layout as the matrix workloads."""
    J = args.rank
    t_gen = time.time()
    T = wl.csf3_powerlaw(500_000, 100_000, 100_000, 8, 1.8, 4096, wl.BASE_SEED + 9)
    I, K, L = T.dims
    Ch = wl.dense_uniform(K * J, wl.BASE_SEED + 9, wl.S_B).reshape(K, J)
    Dh = wl.dense_uniform(L * J, wl.BASE_SEED + 10, wl.S_B).reshape(L, J)
    t_gen = time.time() - t_gen
    nnz, nfib = T.nnz, T.nfibers
    tile = args.tile or psk.psk_default_tile(psk.PSK_OP_MTTKRP_CSF3)
    comp = 8 * nnz + 8 * nfib + 4 * (I + 1) + 4 * J * (K + L) + 4 * J * I
    noreuse = 8 * nnz + 4 * J * nnz + 4 * J * nfib + 8 * nfib + 4 * (I + 1) + 4 * J * I
    fl = 2 * J * nnz + 2 * J * nfib      # sum_l b*D(l,:) per fiber, then one multiply-add with C(k,:) per fiber
    dev = torch.device("cuda:0")
    copies = args.copies or 2
    sets = []
    for _ in range(copies):
        s = {k_: torch.from_numpy(getattr(T, k_)).to(dev) for k_ in ("pos_k", "crd_k", "pos_l", "crd_l", "vals")}
        s["C"], s["D"] = torch.from_numpy(Ch).to(dev), torch.from_numpy(Dh).to(dev)
        s["A"] = torch.empty((I, J), device=dev)
        s["ws"] = psk.workspace(psk.PSK_OP_MTTKRP_CSF3, T.nslices, nnz, k=J, tile=tile, device=dev)
        sets.append(s)
    stream = torch.cuda.current_stream()

    def step(s, phases=psk.PSK_PHASE_ALL):
        psk.psk_mttkrp_csf3(T.dims, None, s["pos_k"], s["crd_k"], s["pos_l"], s["crd_l"], s["vals"], s["C"], s["D"],
                            s["A"], tile=tile, phases=phases, ws=s["ws"], stream=stream)

    for i in range(args.warmup):
        step(sets[i % copies])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(sets[i % copies])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    def time_phase(phases, reps=16, warm=8):
        ts = []
        for i in range(warm + reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            step(sets[i % copies], phases)
            e1.record(stream)
            e1.synchronize()
            if i >= warm:
                ts.append(e0.elapsed_time(e1))
        return ts

    main_ms = time_phase(psk.PSK_PHASE_MAIN)
    all_ms = time_phase(psk.PSK_PHASE_ALL)
    main_avg = sum(main_ms) / len(main_ms)
    # C and D (4*J*(K+L) bytes) stay in the 256 MB memory-side cache, so HBM sees each operand once:
    # the roofline is priced on those compulsory bytes.  What the kernel is bound by is the rate at which
    # L2 misses on D rows are served (no-reuse bytes / time, reported beside it).
    achieved = comp / (main_avg * 1e-3) / 1e9
    traffic, traffic_src = profile_traffic("mttkrp", tile, 1) if J == 64 else (None, "measured for j = 64 only")
    rec = {
        "metric": "SpMV/SpMM GFLOP/s and achieved HBM GB/s (% of MI355X peak), 1 GPU",
        "value": round(fl / (wall / args.steps) / 1e9, 3), "unit": "GFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(wall / args.steps * 1e3, 6), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "mttkrp: %d x %d x %d, %d fibers, nnz %d, j %d, tile %d, %d operand copies rotated"
                               % (I, K, L, nfib, nnz, J, tile, copies),
                   "dims": [I, K, L], "fibers": nfib, "nnz": nnz, "j": J, "tile": tile, "seed": wl.BASE_SEED + 9},
        "ns_per_nnz": round(wall / args.steps * 1e9 / nnz, 6),
        "phases_us_median": {"main": round(statistics.median(main_ms) * 1e3, 2),
                             "all": round(statistics.median(all_ms) * 1e3, 2)},
        "roofline": {"bound": "hbm", "kernel": "k_mttkrp_pos", "achieved": round(achieved, 2), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                     "traffic_source": traffic_src, "algorithmic_bytes": comp, "no_reuse_bytes": noreuse,
                     "no_reuse_GBs": round(noreuse / (main_avg * 1e-3) / 1e9, 2),
                     "avg_launch_us": round(main_avg * 1e3, 2), "launches_per_step": 1,
                     "byte_model": "every operand once (factor matrices are cache resident); no_reuse_* counts one "
                                   "D row per nonzero and one C row per fiber, the requests the L2 actually serves"},
    }
    if not args.no_cpu:
        import oracle

        cores = oracle.threads_used(len(os.sched_getaffinity(0)))
        frac = 1.0
        tmed, nruns = time_cpu(lambda: oracle.mttkrp_csf3(T.pos_k, T.crd_k, T.pos_l, T.crd_l, T.vals, Ch, Dh, threads=cores))
        rec["cpu_baseline"] = {"value": round(fl * frac / tmed / 1e9, 3), "unit": "GFLOP/s", "cores": cores,
                               "kind": "oracle",
                               "sample": "the whole tensor, fp64, OpenMP over slices, 1 warm-up + %d runs, median %.3f s"
                                         % (nruns, tmed)}
    rec["generate_s"] = round(t_gen, 2)
    print(json.dumps(rec))


def bench_dcsr(args, torch, psk, wl):
    """SpMV on the synthetic hypersparse matrix, cut at the column level or at the row level."""
    t_gen = time.time()
    Ls = wl.zipf_lengths(1_000_000, 1.8, 1, 50_000, wl.BASE_SEED + 11)
    A = wl.dcsr_from_lengths(1 << 26, Ls, 1 << 21, seed=wl.BASE_SEED + 11)
    xh = wl.dense_uniform(A.cols, wl.BASE_SEED + 11, wl.S_X)
    t_gen = time.time() - t_gen
    cut = psk.PSK_CUT_POSITIONS if args.cut == "positions" else psk.PSK_CUT_ROWS
    passes = args.col_passes or 1
    tile = args.tile or (1024 if passes > 1 else psk.psk_default_tile(psk.PSK_OP_SPMV_CSR))
    nnz, ns = A.nnz, A.nstored
    comp = 8 * nnz + 4 * (ns + 1) + 4 * ns + 4 * A.cols + 4 * A.rows
    fl = 2 * nnz
    dev = torch.device("cuda:0")
    copies = args.copies or 3
    sets = []
    for _ in range(copies):
        s = {k_: torch.from_numpy(getattr(A, k_)).to(dev) for k_ in ("crd_i", "pos", "crd", "vals")}
        s["x"] = torch.from_numpy(xh).to(dev)
        s["y"] = torch.empty(A.rows, device=dev)
        s["ws"] = psk.workspace(psk.PSK_OP_SPMV_CSR, ns, nnz, tile=tile, device=dev)
        sets.append(s)
    stream = torch.cuda.current_stream()

    def step(s, phases=psk.PSK_PHASE_ALL):
        psk.psk_spmv_dcsr(A.rows, A.cols, nnz, s["crd_i"], s["pos"], s["crd"], s["vals"], s["x"], s["y"], cut=cut,
                          tile=tile, col_passes=passes, phases=phases, ws=s["ws"], stream=stream)

    for i in range(args.warmup):
        step(sets[i % copies])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(sets[i % copies])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    def time_phase(phases, reps=16, warm=8):
        ts = []
        for i in range(warm + reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            step(sets[i % copies], phases)
            e1.record(stream)
            e1.synchronize()
            if i >= warm:
                ts.append(e0.elapsed_time(e1))
        return ts

    main_ms = time_phase(psk.PSK_PHASE_MAIN)
    all_ms = time_phase(psk.PSK_PHASE_ALL)
    main_avg = sum(main_ms) / len(main_ms)
    achieved = comp / (main_avg * 1e-3) / 1e9
    dcsr_traffic, dcsr_traffic_src = (profile_traffic("dcsr", tile, passes) if args.cut == "positions"
                                      else (None, "not measured for the row-level cut"))
    rec = {
        "metric": "SpMV/SpMM GFLOP/s and achieved HBM GB/s (% of MI355X peak), 1 GPU",
        "value": round(fl / (wall / args.steps) / 1e9, 3), "unit": "GFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(wall / args.steps * 1e3, 6), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "dcsr: %d rows (%d stored), %d cols, nnz %d (max row %d), cut at the %s level, tile %d, "
                               "%d operand copies rotated" % (A.rows, ns, A.cols, nnz, int(Ls.max()), args.cut, tile, copies),
                   "rows": A.rows, "stored_rows": ns, "cols": A.cols, "nnz": nnz, "cut": args.cut, "tile": tile,
                   "col_passes": passes,
                   "seed": wl.BASE_SEED + 11},
        "ns_per_nnz": round(wall / args.steps * 1e9 / nnz, 6),
        "phases_us_median": {"main": round(statistics.median(main_ms) * 1e3, 2),
                             "all": round(statistics.median(all_ms) * 1e3, 2)},
        "roofline": {"bound": "hbm", "kernel": "k_fill_zero + " + ("k_spmv_pos" if args.cut == "positions" else "k_spmv_wave_per_row"),
                     "achieved": round(achieved, 2), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": dcsr_traffic, "traffic_source": dcsr_traffic_src,
                     "algorithmic_bytes": comp,
                     "avg_launch_us": round(main_avg * 1e3, 2), "launches_per_step": 2,
                     "byte_model": "A once + x once + y once (the zero-fill of y is part of the main phase)"},
    }
    if not args.no_cpu:
        import oracle

        tmed, nruns = time_cpu(lambda: oracle.spmv_dcsr(A.rows, A.crd_i, A.pos, A.crd, A.vals, xh))
        rec["cpu_baseline"] = {"value": round(fl / tmed / 1e9, 3), "unit": "GFLOP/s", "cores": 1, "kind": "oracle",
                               "sample": "the whole workload, fp64 accumulation, single thread, 1 warm-up + %d runs, "
                                         "median %.3f s" % (nruns, tmed)}
    rec["generate_s"] = round(t_gen, 2)
    print(json.dumps(rec))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="powerlaw", choices=sorted(WORKLOADS))
    ap.add_argument("--tile", type=int, default=0, help="position-tile size (0 = library default)")
    ap.add_argument("--col-passes", type=int, default=0,
                    help="column passes of the CSR SpMV (0 = ask psk_analyze_csr)")
    ap.add_argument("--skew-base", type=float, default=1.00256, help="base of the expskew workload")
    ap.add_argument("--skew-rows", type=int, default=65536, help="rows of the expskew workload")
    ap.add_argument("--skew-nnz", type=int, default=4_000_000, help="nonzeros of the expskew workload")
    ap.add_argument("--copies", type=int, default=0, help="operand copies rotated between steps (0 = auto)")
    ap.add_argument("--parts", type=int, action="append",
                    help="--baselines: number of parts for the divided variant (repeatable; default 0 = 2048)")
    ap.add_argument("--cut", choices=["positions", "rows"], default="positions",
                    help="dcsr: level of the position cut (column level = equal nonzeros, row level = equal stored rows)")
    ap.add_argument("--k", type=int, default=0, help="spmm workloads: number of dense columns (0 = the configuration's)")
    ap.add_argument("--bs", type=int, default=4, choices=[2, 4, 8],
                    help="bcsr_spmv / bcsr_spmm: block edge (the 10^6 x 10^6 matrix with 32 entries per row is re-blocked)")
    ap.add_argument("--f64", action="store_true", help="CSR SpMV workloads: fp64 values, vector and result")
    ap.add_argument("--table-mb", type=float, default=8.0, help="gather: size of the table in MB")
    ap.add_argument("--rank", type=int, default=64, help="mttkrp: number of columns j of the factor matrices")
    ap.add_argument("--path", choices=["auto", "csr", "slab"], default="auto",
                    help="CSR SpMV workloads: multiply from the CSR arrays (position cut per call) or from the "
                         "column-slab copy of A built once by the analysis step; auto = slab when psk_analyze_csr "
                         "finds the columns scattered over an x larger than the caches, else csr")
    ap.add_argument("--cu-trace", action="store_true",
                    help="CSR SpMV workloads: load the instrumented build (libpsk_trace.so) and report the busy time of "
                         "every compute unit (max / mean) for the position cut, the slab path and the two row-split kernels")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing")
    ap.add_argument("--baselines", action="store_true", help="also time the row-split kernels")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.stderr.write("bench.py: this build is single-GPU (no sharding, no collectives); run with --gpus 1\n")
        sys.exit(2)

    import torch

    import paper_2001_00532_amd as psk
    import workloads as wl

    if not torch.cuda.is_available():
        sys.stderr.write("bench.py: no GPU visible\n")
        sys.exit(1)
    if args.cu_trace:
        psk.use_instrumented_library()
    psk.lib()   # fail loudly when the HIP library is missing

    cfg_no, kind = WORKLOADS[args.workload]
    if kind == "copy":
        return bench_copy(args, torch)
    if kind == "calibration":
        return bench_calibration(args, torch, psk)
    if kind == "mttkrp":
        return bench_mttkrp(args, torch, psk, wl)
    if kind == "dcsr":
        return bench_dcsr(args, torch, psk, wl)
    t_gen = time.time()
    if args.workload == "uniform28":
        A28 = wl.csr_uniform(2_000_000, 2_000_000, 28, wl.BASE_SEED + 6)
        cfg = {"A": A28, "x": wl.dense_uniform(2_000_000, wl.BASE_SEED + 6, wl.S_X)}
    elif args.workload == "spmm_dense32":
        As = wl.csr_uniform(100_000, 100_000, 1000, wl.BASE_SEED + 12)
        cfg = {"A": As, "k": 32, "B": wl.dense_uniform(100_000 * 32, wl.BASE_SEED + 12, wl.S_B).reshape(100_000, 32)}
    elif args.workload == "fewlong":
        Af = wl.csr_uniform(100, 100_000, 10_000, wl.BASE_SEED + 7)
        cfg = {"A": Af, "x": wl.dense_uniform(100_000, wl.BASE_SEED + 7, wl.S_X)}
    elif args.workload == "expskew":
        Ls = wl.exponential_lengths(args.skew_rows, args.skew_nnz, args.skew_base, 1_000_000, wl.BASE_SEED + 8)
        Ae = wl.csr_from_lengths(Ls, 1_000_000, wl.BASE_SEED + 8)
        cfg = {"A": Ae, "x": wl.dense_uniform(1_000_000, wl.BASE_SEED + 8, wl.S_X)}
    elif kind.startswith("bcsr") and args.bs != 4:
        br = 1_000_000 // args.bs
        Ab = wl.csr_uniform(br, br, 32 // args.bs, wl.BASE_SEED + 5, bs=args.bs)
        cfg = {"A": Ab, "k": 64, "x": wl.dense_uniform(br * args.bs, wl.BASE_SEED + 5, wl.S_X),
               "B": wl.dense_uniform(br * args.bs * 64, wl.BASE_SEED + 5, wl.S_B).reshape(br * args.bs, 64)}
    else:
        cfg = wl.config(cfg_no)
    A = cfg["A"]
    k = cfg.get("k", 1) if kind.endswith("spmm") else 1
    if kind.endswith("spmm") and args.k and args.k != k:     # same matrix, another width of the dense operand
        k = args.k
        cfg["B"] = wl.dense_uniform(A.cols * A.bs * k, wl.BASE_SEED + cfg_no, wl.S_B).reshape(A.cols * A.bs, k)
    dense_h = cfg["B"] if kind.endswith("spmm") else cfg["x"]
    f64 = args.f64
    if f64 and kind != "csr_spmv":
        sys.stderr.write("bench.py: --f64 applies to the CSR SpMV workloads\n")
        sys.exit(2)
    vals_h = A.vals
    if f64:
        vals_h = wl.dense_uniform_f64(A.nnz, wl.BASE_SEED + cfg_no, wl.S_VALS)
        dense_h = wl.dense_uniform_f64(A.cols, wl.BASE_SEED + cfg_no, wl.S_X)
    t_gen = time.time() - t_gen
    out_rows = A.rows * A.bs
    L = np.diff(A.pos)
    comp_bytes, noreuse_bytes = algorithmic_bytes(kind, A, k)
    if f64:
        comp_bytes = noreuse_bytes = 12 * A.nnz + 4 * (A.rows + 1) + 8 * A.cols + 8 * A.rows
    fl = flops(kind, A, k)

    op = {"csr_spmv": psk.PSK_OP_SPMV_CSR, "csr_spmm": psk.PSK_OP_SPMM_CSR, "bcsr_spmv": psk.PSK_OP_SPMV_BCSR,
          "bcsr_spmm": psk.PSK_OP_SPMM_BCSR}[kind]
    if f64:
        op = psk.PSK_OP_SPMV_CSR_F64
    tile = args.tile or (psk.psk_default_tile_bcsr(op, A.bs) if kind.startswith("bcsr") else psk.psk_default_tile(op))
    tile_given = bool(args.tile)

    # rotate over enough operand copies that a step never finds its inputs in the 256 MB memory-side cache
    copies = args.copies or max(2, min(8, int(np.ceil(1.0e9 / comp_bytes))))
    dev = torch.device("cuda:0")
    sets = []
    for _ in range(copies):
        s = {"pos": torch.from_numpy(A.pos).to(dev), "crd": torch.from_numpy(A.crd).to(dev),
             "vals": torch.from_numpy(vals_h).to(dev), "dense": torch.from_numpy(dense_h).to(dev)}
        s["out"] = torch.empty((out_rows, k) if kind.endswith("spmm") else (out_rows,), device=dev,
                               dtype=torch.float64 if f64 else torch.float32)
        sets.append(s)
    stream = torch.cuda.current_stream()

    # plan step, outside the timed region like the workspace allocation: depends only on A
    col_passes = 1
    if kind == "csr_spmv" and f64:
        # the same probe; an fp64 x is twice as large per column, so the slices are sized on 8-byte entries
        col_passes = args.col_passes
        if not col_passes:
            col_passes = 1
            if psk.psk_analyze_csr(A.rows, A.cols, A.nnz, sets[0]["pos"], sets[0]["crd"], stream=stream) > 1:
                col_passes = int(min(4, -(-(8 * A.cols) // (6 << 20))))
    path = "csr"
    analysis = None
    if kind == "csr_spmv" and f64:
        suggested64 = psk.psk_analyze_csr(A.rows, A.cols, A.nnz, sets[0]["pos"], sets[0]["crd"], stream=stream)
        path = args.path if args.path != "auto" else ("slab" if suggested64 > 1 and not args.col_passes else "csr")
    if kind == "csr_spmv" and not f64:
        suggested = psk.psk_analyze_csr(A.rows, A.cols, A.nnz, sets[0]["pos"], sets[0]["crd"], stream=stream)
        path = args.path if args.path != "auto" else ("slab" if suggested > 1 and not args.col_passes else "csr")
        col_passes = args.col_passes or suggested
        if col_passes > 1 and not tile_given:
            tile = 1024      # what tile = 0 selects inside the library when column passes are on
    for s in sets:
        s["ws"] = psk.workspace(op, A.rows, A.nnz, k=k, bs=A.bs, tile=tile, device=dev)
    csr_tile, csr_passes = tile, col_passes
    if path == "slab":
        # the analysis step: once per matrix, outside the timed region like the column-pass probe; its time is
        # reported beside the product's so that the number of products that repay it can be read off
        build_ms = []
        for i, s in enumerate(sets):
            torch.cuda.synchronize()
            t_b = time.perf_counter()
            build = psk.psk_slab_build_csr_f64 if f64 else psk.psk_slab_build_csr
            s["slab"] = build(A.rows, A.cols, A.nnz, s["pos"], s["crd"], s["vals"], stream=stream)
            torch.cuda.synchronize()
            build_ms.append((time.perf_counter() - t_b) * 1e3)
            s["slab_ws"] = psk.psk_slab_spmv_workspace(s["slab"], dev)
        d0 = sets[0]["slab"].desc
        analysis = {"call": "psk_slab_build_csr_f64" if f64 else "psk_slab_build_csr", "ms_median": round(statistics.median(build_ms), 3),
                    "ms_first": round(build_ms[0], 3), "builds": len(build_ms),
                    "slabs": int(d0.nslabs), "slots": int(d0.nslots), "pairs": int(d0.npairs),
                    "listed_pairs": int(d0.nq), "structure_bytes": int((2 + d0.value_bytes) * d0.nslots + 4 * (d0.nchunks + 1) + 4 * (d0.nslabs + 1)
                                                                   + 4 * (A.rows + 1) + 4 * d0.nq)}
        tile, col_passes = int(d0.tile), 1

    def step(s, phases=psk.PSK_PHASE_ALL):
        if f64 and path == "slab":
            psk.psk_spmv_slab_f64(s["slab"], s["dense"], s["out"], phases=phases, ws=s["slab_ws"], stream=stream)
        elif f64:
            psk.psk_spmv_csr_f64(A.rows, A.cols, A.nnz, s["pos"], s["crd"], s["vals"], s["dense"], s["out"], tile=tile,
                                 col_passes=col_passes, phases=phases, ws=s["ws"], stream=stream)
        elif kind == "csr_spmv" and path == "slab":
            psk.psk_spmv_slab(s["slab"], s["dense"], s["out"], phases=phases, ws=s["slab_ws"], stream=stream)
        elif kind == "csr_spmv":
            # tile = 0 unless one was asked for: the library then also takes a matrix of one tile in one launch
            psk.psk_spmv_csr(A.rows, A.cols, A.nnz, s["pos"], s["crd"], s["vals"], s["dense"], s["out"],
                             tile=tile if tile_given else 0, col_passes=col_passes, phases=phases, ws=s["ws"], stream=stream)
        elif kind == "csr_spmm":
            psk.psk_spmm_csr(A.rows, A.cols, A.nnz, s["pos"], s["crd"], s["vals"], s["dense"], s["out"], tile=tile,
                             phases=phases, ws=s["ws"], stream=stream)
        elif kind == "bcsr_spmv":
            psk.psk_spmv_bcsr(A.rows, A.cols, A.nnz, A.bs, s["pos"], s["crd"], s["vals"], s["dense"], s["out"],
                              tile=tile, phases=phases, ws=s["ws"], stream=stream)
        else:
            psk.psk_spmm_bcsr(A.rows, A.cols, A.nnz, A.bs, s["pos"], s["crd"], s["vals"], s["dense"], s["out"],
                              tile=tile, phases=phases, ws=s["ws"], stream=stream)

    if args.cu_trace:
        if kind != "csr_spmv" or f64:
            sys.stderr.write("bench.py: --cu-trace applies to the fp32 CSR SpMV workloads\n")
            sys.exit(2)
        return cu_trace_report(args, torch, psk, A, sets[0], tile, col_passes, path, stream)

    # ---- warm-up, then exactly K timed steps bracketed by synchronize
    for i in range(args.warmup):
        step(sets[i % copies])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(sets[i % copies])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall / args.steps * 1e3

    # ---- the phases on their own, HIP events on the stream the kernels run on (median of 16 samples, 4 warm-ups)
    # Each sample brackets `inner` back-to-back calls with one event pair and divides: the host-side cost of
    # recording an event and of the first launch after an idle stream (about 5-10 us) would otherwise be charged to
    # kernels that now take about 100 us; the calls of a sample rotate over the operand copies like the timed steps.
    def time_phase(phases, reps=16, warm=4, inner=8):
        ts = []
        for i in range(warm + reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for j in range(inner):
                step(sets[(i * inner + j) % copies], phases)
            e1.record(stream)
            e1.synchronize()
            if i >= warm:
                ts.append(e0.elapsed_time(e1) / inner)
        return ts

    main_ms = time_phase(psk.PSK_PHASE_MAIN)
    part_ms = time_phase(psk.PSK_PHASE_PARTITION)
    fix_ms = time_phase(psk.PSK_PHASE_FIXUP)
    all_ms = time_phase(psk.PSK_PHASE_ALL)
    # With column passes the tile kernel is launched col_passes times per product; the algorithmic bytes
    # (A, x and y once) are charged once, against the time of all its launches together, so that the
    # re-streaming of A by the later passes counts as overhead, not as achieved bandwidth.
    main_avg = sum(main_ms) / len(main_ms)
    kernel_bytes = noreuse_bytes if kind.endswith("spmm") else comp_bytes
    achieved = kernel_bytes / (main_avg * 1e-3) / 1e9
    traffic, traffic_src = profile_traffic(args.workload + ("_f64" if f64 else ""), tile, col_passes, path)
    if kind.startswith("bcsr") and A.bs != 4 or (kind.endswith("spmm") and k != cfg.get("k", 1)):
        traffic, traffic_src = None, "measured for the configuration's block size and width only"

    rec = {
        "metric": "SpMV/SpMM GFLOP/s and achieved HBM GB/s (% of MI355X peak), 1 GPU",
        "value": round(fl / (wall / args.steps) / 1e9, 3),
        "unit": "GFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 6),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f64" if f64 else "f32",
        "data": "synthetic",
        "config": {
            "workload": "%s: %s%s, %d x %d%s, nnz %d (max row %d, mean %.2f), tile %d, col_passes %d, k %d, %d operand copies rotated"
                        % (args.workload, kind, " over the column-slab copy of A (built once by %s)" % analysis["call"] if path == "slab" else "",
                           A.rows * A.bs, A.cols * A.bs, " in %dx%d blocks" % (A.bs, A.bs) if A.bs > 1 else "",
                           A.nnz * A.bs * A.bs, int(L.max()) if L.size else 0, float(L.mean()) if L.size else 0.0,
                           tile, col_passes, k, copies),
            "rows": A.rows * A.bs, "cols": A.cols * A.bs, "nnz": A.nnz * A.bs * A.bs, "k": k, "tile": tile,
            "col_passes": col_passes,
            "path": path,
            "seed": wl.BASE_SEED + cfg_no,
            "input_hash": input_hash(A.pos, A.crd, vals_h, dense_h),
        },
        "gbps_algorithmic_whole_step": round(comp_bytes / (wall / args.steps) / 1e9, 2),
        "pct_of_hbm_peak_whole_step": round(100.0 * comp_bytes / (wall / args.steps) / 1e9 / HBM_PEAK_GBS, 2),
        "ns_per_nnz": round(wall / args.steps * 1e9 / max(1, A.nnz * A.bs * A.bs), 6),
        "phases_us_median": {
            "partition": round(statistics.median(part_ms) * 1e3, 2),
            "main": round(statistics.median(main_ms) * 1e3, 2),
            "fixup": round(statistics.median(fix_ms) * 1e3, 2),
            "all": round(statistics.median(all_ms) * 1e3, 2),
            "all_min": round(min(all_ms) * 1e3, 2),
        },
        "roofline": {
            "bound": "hbm",
            "kernel": ("k_slab_pairs<double> + k_spmv_pos_f64<256,8,*,unit values>" if path == "slab" else "k_spmv_pos_f64") if f64
                      else ("k_slab_pairs<float> + k_spmv_pos<256,8,*,6>" if path == "slab" else
                       {"csr_spmv": "k_spmv_pos", "csr_spmm": "k_spmm_pos<1,*>", "bcsr_spmv": "k_spmv_bcsr4",
                        "bcsr_spmm": "k_spmm_pos<4,*>"}[kind]),
            "achieved": round(achieved, 2),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBS, 4),
            "traffic": traffic,
            "traffic_source": traffic_src,
            "algorithmic_bytes": kernel_bytes,
            "avg_launch_us": round(main_avg * 1e3 / (2 if path == "slab" else col_passes), 2),
            "launches_per_step": 2 if path == "slab" else col_passes,
            "byte_model": ("one dense row per stored position (no reuse)" if kind.endswith("spmm")
                           else "A once + dense operand once + output once"),
        },
    }

    if kind == "csr_spmv" and not f64 and path == "csr" and not tile_given and col_passes <= 1 and 0 < A.nnz <= 16384:
        # a problem of one tile: the library takes it as one launch of one workgroup; what counts is time per call
        rec["roofline"]["launches_per_step"] = 1
        rec["roofline"]["kernel"] = "k_spmv_pos<1024,16,*,7> (the whole matrix as one tile)"
        iso = time_phase(psk.PSK_PHASE_ALL, reps=32, warm=8, inner=1)     # one call between two events, stream idle before
        # the same product with the arguments marshalled once (the Python side of a call costs more than the kernel)
        calls = [psk.psk_spmv_csr_prepared(A.rows, A.cols, A.nnz, s_["pos"], s_["crd"], s_["vals"], s_["dense"], s_["out"],
                                           ws=s_["ws"], stream=stream) for s_ in sets]
        for i in range(200):
            calls[i % copies]()
        torch.cuda.synchronize()
        t_p = time.perf_counter()
        for i in range(2000):
            calls[i % copies]()
        torch.cuda.synchronize()
        prepared_us = (time.perf_counter() - t_p) / 2000 * 1e6
        rec["latency"] = {"launches_per_product": 1,
                          "us_per_call_back_to_back": round(ms_per_step * 1e3, 2),
                          "us_per_call_back_to_back_prepared": round(prepared_us, 2),
                          "us_per_call_isolated_with_events": round(statistics.median(iso) * 1e3, 2),
                          "note": "launch-latency bound: 94 KB of operands; the roofline fraction is not meaningful here"}

    if path == "slab":
        # the same product from the CSR arrays (position cut, tile kernel, fix-up in every call), for comparison
        ts = []
        for i in range(24):
            s_ = sets[i % copies]
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            csr_call = psk.psk_spmv_csr_f64 if f64 else psk.psk_spmv_csr
            csr_call(A.rows, A.cols, A.nnz, s_["pos"], s_["crd"], s_["vals"], s_["dense"], s_["out"], tile=csr_tile,
                     col_passes=csr_passes, ws=s_["ws"], stream=stream)
            e1.record(stream)
            e1.synchronize()
            if i >= 8:
                ts.append(e0.elapsed_time(e1))
        csr_us = statistics.median(ts) * 1e3
        slab_us = statistics.median(all_ms) * 1e3
        analysis["repaid_after_products"] = (int(np.ceil(analysis["ms_median"] * 1e3 / (csr_us - slab_us)))
                                             if csr_us > slab_us else None)
        # the same throughput with the analysis charged to the products of one matrix (10, 100, 1000 of them)
        analysis["gflops_with_analysis_over_products"] = {
            str(n): round(fl * n / ((n * slab_us + analysis["ms_median"] * 1e3) * 1e-6) / 1e9, 1) for n in (10, 100, 1000)}
        rec["analysis"] = analysis
        rec["csr_path"] = {"call": "psk_spmv_csr_f64" if f64 else "psk_spmv_csr", "tile": csr_tile, "col_passes": csr_passes,
                           "us_median": round(csr_us, 2), "gflops": round(fl / (csr_us * 1e-6) / 1e9, 3),
                           "frac_of_hbm_peak_whole_call": round(comp_bytes / (csr_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)}

    if args.baselines and kind == "csr_spmv" and not f64:
        base = {}
        for name, variant in (("thread_per_row", 0), ("wave_per_row", 1)):
            ts = []
            for i in range(12):
                s = sets[i % copies]
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                psk.psk_spmv_csr_rowsplit(A.rows, A.cols, A.nnz, s["pos"], s["crd"], s["vals"], s["dense"], s["out"],
                                          variant=variant, stream=stream)
                e1.record(stream)
                e1.synchronize()
                if i >= 4:
                    ts.append(e0.elapsed_time(e1))
            base[name + "_us_median"] = round(statistics.median(ts) * 1e3, 2)
        ts = []
        for i in range(12):     # the schedule's atomics strategy: zero-fill + tile kernel, no fix-up
            s = sets[i % copies]
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            psk.psk_spmv_csr_atomics(A.rows, A.cols, A.nnz, s["pos"], s["crd"], s["vals"], s["dense"], s["out"],
                                     tile=args.tile, ws=s["ws"], stream=stream)
            e1.record(stream)
            e1.synchronize()
            if i >= 4:
                ts.append(e0.elapsed_time(e1))
        base["position_space_atomics_us_median"] = round(statistics.median(ts) * 1e3, 2)
        for parts in (args.parts or [0]):     # the position space divided into a fixed number of parts
            ts = []
            for i in range(12):
                s = sets[i % copies]
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                psk.psk_spmv_csr_divide(A.rows, A.cols, A.nnz, s["pos"], s["crd"], s["vals"], s["dense"], s["out"],
                                        parts=parts, ws=s["ws"], stream=stream)
                e1.record(stream)
                e1.synchronize()
                if i >= 4:
                    ts.append(e0.elapsed_time(e1))
            base["position_space_divided_parts_%d_us_median" % parts] = round(statistics.median(ts) * 1e3, 2)
        for name, phases in (("position_space_no_temporary_us_median", psk.PSK_PHASE_ALL),
                             ("position_space_no_temporary_main_us_median", psk.PSK_PHASE_MAIN)):
            ts = []
            for i in range(12):     # ablation: rolled load loop, no register temporary (Section 8.3)
                s = sets[i % copies]
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                psk.psk_spmv_csr_notemp(A.rows, A.cols, A.nnz, s["pos"], s["crd"], s["vals"], s["dense"], s["out"],
                                        tile=args.tile, phases=phases, ws=s["ws"], stream=stream)
                e1.record(stream)
                e1.synchronize()
                if i >= 4:
                    ts.append(e0.elapsed_time(e1))
            base[name] = round(statistics.median(ts) * 1e3, 2)
        rec["rowsplit_baselines"] = base

    # ---- the CPU oracle on this machine's host cores (a baseline, not a target)
    if not args.no_cpu:
        import oracle

        cores = oracle.threads_used(len(os.sched_getaffinity(0)))
        sel = None
        sample = "full workload"
        if kind == "csr_spmm":
            sel = np.arange(0, A.rows, 8, dtype=np.int64)           # every 8th row
            sample = "every 8th row of the workload (1/8 of the flops)"
        elif kind == "bcsr_spmm":
            sel = np.arange(0, A.rows, 4, dtype=np.int64)
            sample = "every 4th block row of the workload (1/4 of the flops)"
        frac = 1.0 if sel is None else len(sel) / A.rows

        def run_oracle():
            if f64:
                oracle.spmv_csr_f64(A.pos, A.crd, vals_h, dense_h, threads=cores)
            elif kind == "csr_spmv":
                oracle.spmv_csr(A.pos, A.crd, A.vals, dense_h, threads=cores)
            elif kind == "csr_spmm":
                oracle.spmm_csr(A.pos, A.crd, A.vals, dense_h, sel=sel, threads=cores)
            elif kind == "bcsr_spmv":
                oracle.spmv_bcsr(A.pos, A.crd, A.vals, dense_h, A.bs, threads=cores)
            else:
                oracle.spmm_bcsr(A.pos, A.crd, A.vals, dense_h, A.bs, sel=sel, threads=cores)

        tmed, nruns = time_cpu(run_oracle)
        cores_all, cores = cores, 1
        t1, n1 = time_cpu(run_oracle, budget_s=3.0, max_runs=5)      # the same oracle on one thread
        cores = cores_all
        rec["cpu_baseline_single_thread"] = {"value": round(fl * frac / t1 / 1e9, 3), "unit": "GFLOP/s", "cores": 1,
                                             "kind": "oracle", "sample": "%s, 1 warm-up + %d runs, median %.3f s"
                                                                         % (sample, n1, t1)}
        rec["cpu_baseline"] = {
            "value": round(fl * frac / tmed / 1e9, 3),
            "unit": "GFLOP/s",
            "cores": cores,
            "kind": "oracle",
            "sample": "%s, fp64 accumulation, OpenMP over rows, 1 warm-up + %d runs, median %.3f s"
                      % (sample, nruns, tmed),
        }
    rec["generate_s"] = round(t_gen, 2)
    print(json.dumps(rec))


if __name__ == "__main__":
    main()
