#!/usr/bin/env python3
"""Benchmark of the sparse x dense contraction library on one MI355X.

A "step" is one pass of the hot path over one batch of synthetic input: one call of an operation
through the C ABI (main kernel + carry fix-up + any result clearing), inputs resident in HBM.
The headline workload is the SpMM configuration (CSR 1e6 x 1e6, Zipf(1.8) row lengths capped at
10,000, B dense 1e6 x 32, fp64); `value` is its GFLOP/s.  The other four configurations of the
baseline (SpMV, TTV, TTM, MTTKRP at rank 16 and 64) are timed the same way and reported under
"kernels" in the same JSON line.

For every operation the line carries the algorithmic (compulsory) bytes of one launch, the
achieved GB/s = those bytes / mean launch time, and the fraction of the 8 TB/s HBM peak.
"cpu_baseline" is the CPU oracle timed on this host on a bounded sample of the headline workload.

  python bench.py [--gpus 1] [--steps 25] [--warmup 5] [--ops spmv,spmm,ttv,ttv_coo,ttm,mttkrp16,mttkrp64]
                  [--scale 1.0] [--variant 0] [--no-cpu-baseline]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
ALL_OPS = ["spmm", "spmv", "spmv_large", "ttv", "ttv_coo", "ttm", "mttkrp16", "mttkrp64", "ttv_m0", "ttm_m0", "mttkrp16_m1",
           "spmm_dcsr", "read", "gather_l2", "gather_c64", "gather_b16", "gather_b32", "gather_b64"]
# calibration legs (no tensor): a plain 2 GiB read and row gathers by lane groups of 8 from tables of
# (rows x R doubles): 16384 x 16 (2 MB, L2-resident), 20000 x 64 (10 MB: the C factor of MTTKRP at rank 64),
# 10^6 x 16 / 32 / 64 (128 / 256 / 512 MB: the B operands of MTTKRP and SpMM)
CALIBRATION = {"gather_l2": (16384, 16), "gather_c64": (20000, 64), "gather_b16": (1000000, 16),
               "gather_b32": (1000000, 32), "gather_b64": (1000000, 64)}
# "<op>_m<n>": the same operation along / for mode n of the same tensor, on the storage that
# comet_tensor_reorder builds for it (first-mode TTV and TTM are the forms Section 8.2 writes out)


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def time_steps(fn, steps, warmup):
    """Mean milliseconds of `steps` back-to-back calls of fn (one event pair around the whole run, on the
    current stream, synchronised on both sides), then per-call median / min from a second, separately
    timed run with an event pair per call (those events would otherwise sit between the timed calls)."""
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    first, last = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    first.record()
    for _ in range(steps):
        fn()
    last.record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) * 1e3 / steps
    total = first.elapsed_time(last) / steps
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for a, b in evs:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    per = sorted(a.elapsed_time(b) for a, b in evs)
    return {"mean_ms": total, "median_ms": per[len(per) // 2], "min_ms": per[0], "wall_ms": wall}


def small_problem_latency(fn, out, dev):
    """Per-call latency figures for a launch-bound problem: cold (after a 1 GiB cache flush) and as a
    replayed HIP graph of 20 calls (checked against the eager result on every replay)."""
    import torch
    res = {}
    flush = torch.empty(1 << 27, dtype=torch.float64, device=dev)
    cold = []
    for _ in range(5):
        flush.fill_(1.0)
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        fn()
        b.record()
        torch.cuda.synchronize()
        cold.append(a.elapsed_time(b) * 1e3)
    res["cold_us"] = round(sorted(cold)[len(cold) // 2], 2)
    del flush
    try:
        fn()
        torch.cuda.synchronize()
        want = out.clone()
        calls = 20
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for _ in range(calls):
                fn()
        ok = True
        times = []
        for _ in range(10):
            out.fill_(float("nan"))
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            g.replay()
            b.record()
            torch.cuda.synchronize()
            times.append(a.elapsed_time(b) * 1e3 / calls)
            ok = ok and bool(torch.equal(out, want))
        res["graph_replay_us_per_call"] = round(sorted(times)[len(times) // 2], 2)
        res["graph_replay_matches_eager"] = ok
    except Exception as e:                                  # capture not possible here: report, do not fail the bench
        res["graph_replay_us_per_call"] = None
        res["graph_replay_error"] = str(e)[:200]
    return res


def count_distinct(t):
    import torch
    return int(torch.unique(t).numel())


_TRAFFIC = None


def kernel_sources_digest():
    """sha256 over the HIP sources of the library (file names and contents, sorted): which kernels a figure belongs to."""
    import hashlib
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2102_05187_amd", "csrc")
    for name in sorted(os.listdir(d)):
        if name.endswith((".hip", ".hpp")):
            h.update(name.encode())
            with open(os.path.join(d, name), "rb") as f:
                h.update(f.read())
    return h.hexdigest()


def measured_traffic(op):
    """HBM bytes of one call (fetch + write) from the committed rocprofv3 counter summary, or None.

    The counters cannot be read from inside this process; profiles/hbm_traffic.json holds what
    `rocprofv3 --pmc FETCH_SIZE` / `WRITE_SIZE` measured for this same command at full size, together with the
    digest of the kernel sources it was collected with.  A figure collected with other kernels is not reported."""
    global _TRAFFIC
    if _TRAFFIC is None:
        try:
            with open(os.path.join(ROOT, "profiles", "hbm_traffic.json")) as f:
                doc = json.load(f)
            _TRAFFIC = doc.get("ops", {}) if doc.get("kernel_sources_sha256") == kernel_sources_digest() else {}
            if not _TRAFFIC:
                log("[bench] profiles/hbm_traffic.json was collected with other kernel sources: roofline.traffic left out")
        except (OSError, ValueError):
            _TRAFFIC = {}
    e = _TRAFFIC.get(op)
    return None if e is None else int(e["fetch_bytes"]) + int(e["write_bytes"])


TRAFFIC_SOURCE = ("profiles/hbm_traffic.json: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of this command at full size, "
                  "collected in separate runs with these same kernel sources (digest checked; the counters cannot be "
                  "read in-process); not measured in this run")


def roofline(bytes_per_launch, ms, op=None, full_size=True):
    gbs = bytes_per_launch / (ms * 1e-3) / 1e9
    traffic = measured_traffic(op) if (op and full_size) else None
    out = {"bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
           "frac": round(gbs / HBM_PEAK_GBS, 4), "traffic": traffic, "bytes_per_launch": int(bytes_per_launch)}
    if traffic is not None:
        out["traffic_gbs"] = round(traffic / (ms * 1e-3) / 1e9, 1)
        out["traffic_source"] = TRAFFIC_SOURCE
    return out


def relabel_matrix(c, sweeps):
    """(rows, cols, vals) of a generated matrix configuration, relabelled and re-sorted when sweeps > 0; the
    dense operand follows the new column labels so that the product is the relabelled original one."""
    if not sweeps:
        return c["coo"]
    import torch
    from synth import lexi
    (rows, cols), labels = lexi.lexi_relabel(c["coo"][:2], c["dims"], sweeps)
    (rows, cols), vals = lexi.sort_nonzeros((rows, cols), c["dims"], c["coo"][2])
    moved = torch.empty_like(c["B"])
    moved[labels[1]] = c["B"]
    c["B"] = moved
    c["coo"] = (rows, cols, vals)
    return rows, cols, vals


def run_op(op, args, comet, dev):
    """Generate the op's configuration on the GPU, time it, return the report entry (+ inputs for the baseline)."""
    import torch
    from synth import formats as fmt
    from synth import generate as gen
    t_gen = time.perf_counter()
    sc = args.scale
    keep = {}
    if op == "read":
        n = 1 << 28
        src = torch.ones(n, dtype=torch.float64, device=dev)
        sink = torch.zeros(1, dtype=torch.float64, device=dev)
        fn = lambda: comet.comet_calibrate_read(src, sink)
        nnz, flops, nbytes = n, 0, 8 * n
        desc = "plain read of %d bytes (calibration)" % (8 * n)
        extra = {}
        keep = dict(src=src, sink=sink)
    elif op in CALIBRATION:
        rows_, R_ = CALIBRATION[op]
        table = torch.ones((rows_, R_), dtype=torch.float64, device=dev)
        sink = torch.zeros(1, dtype=torch.float64, device=dev)
        gathers = 1 << 26
        fn = lambda: comet.comet_calibrate_gather(table, gathers, sink)
        nnz, flops, nbytes = gathers, 0, gathers * 8 * R_
        desc = "%d gathers of %d-byte rows from a %.1f MB table (calibration; bytes = gathered bytes, not HBM traffic)" % (
            gathers, 8 * R_, rows_ * R_ * 8 / 1e6)
        extra = {"rows_per_s": None, "table_bytes": rows_ * R_ * 8, "row_bytes": 8 * R_}
        keep = dict(table=table, sink=sink)
    elif op == "copy":
        # calibration only: a plain 1 GiB device-to-device copy, to scale the rocprofv3 HBM byte counters
        n = 1 << 27
        src = torch.ones(n, dtype=torch.float64, device=dev)
        dst = torch.empty_like(src)
        fn = lambda: dst.copy_(src)
        nnz, flops, nbytes = n, 0, 16 * n
        desc = "plain copy of %d bytes (counter calibration)" % (8 * n)
        extra = {}
        keep = dict(src=src, dst=dst)
    elif op == "spmv":
        c = gen.config_spmv(seed=0, device=dev)
        rows, cols, vals = c["coo"]
        n = c["dims"][0]
        L = fmt.pack_csr(n, n, rows, cols, vals)
        A = comet.from_levels(L).set_variant(args.variant)
        x, y = c["x"], torch.empty(n, dtype=torch.float64, device=dev)
        fn = lambda: comet.comet_spmv(A, x, y)
        nnz = vals.numel()
        flops = 2 * nnz
        nbytes = 12 * nnz + 12 * n + 8 * n
        desc = "SpMV CSR %dx%d, %d nnz (10 per row)" % (n, n, nnz)
        extra = {"nnz": nnz, "rows": n}
        keep = dict(A=A, L=L, x=x, y=y)
    elif op == "spmv_large":
        # the SpMM matrix with one dense column: x (8 MB) does not fit in LDS, gathers go through L1 / L2
        c = gen.config_spmm(seed=0, device=dev, scale=sc, R=1)
        rows, cols, vals = relabel_matrix(c, args.lexi_sweeps)
        n = c["dims"][0]
        L = fmt.pack_csr(n, n, rows, cols, vals)
        A = comet.from_levels(L).set_variant(args.variant)
        x, y = c["B"].reshape(-1).contiguous(), torch.empty(n, dtype=torch.float64, device=dev)
        fn = lambda: comet.comet_spmv(A, x, y)
        nnz = vals.numel()
        flops = 2 * nnz
        nbytes = 12 * nnz + 12 * n + 8 * n
        desc = "SpMV CSR %dx%d, %d nnz, Zipf(1.8) rows capped at 10000" % (n, n, nnz)
        extra = {"nnz": nnz, "rows": n}
        keep = dict(A=A, L=L, x=x, y=y)
    elif op in ("spmm", "spmm_dcsr"):
        c = gen.config_spmm(seed=0, device=dev, scale=sc, R=32)
        rows, cols, vals = relabel_matrix(c, args.lexi_sweeps)
        n = c["dims"][0]
        R = 32
        L = fmt.pack_csr(n, n, rows, cols, vals) if op == "spmm" else fmt.pack_dcsr(n, n, rows, cols, vals)
        A = comet.from_levels(L).set_variant(args.variant)
        B, C = c["B"], torch.empty((n, R), dtype=torch.float64, device=dev)
        fn = lambda: comet.comet_spmm(A, B, C)
        nnz = vals.numel()
        touched = count_distinct(cols)
        flops = 2 * R * nnz
        nbytes = 12 * nnz + (4 + 8 * R) * n + 8 * R * touched
        desc = "SpMM %s %dx%d, %d nnz, Zipf(1.8) rows capped at 10000, B %dx%d" % ("CSR" if op == "spmm" else "DCSR", n, n, nnz, n, R)
        hrows, hnnz = A.heavy_plan()
        extra = {"nnz": nnz, "rows": n, "R": R, "touched_B_rows": touched, "gather_bytes": 8 * R * nnz,
                 "touched_row_bytes": 8 * R * touched, "heavy_rows": hrows, "heavy_nnz": hnnz,
                 "heavy_stream_bytes": A.heavy_stream_bytes()}
        keep = dict(A=A, L=L, B=B, C=C, coo=(rows, cols, vals), n=n)
    else:
        full_op, mode_n = op, None
        if "_m" in op:
            op, mode_n = op.split("_m")[0], int(op.split("_m")[1])
        R = {"ttv": 1, "ttv_coo": 1, "ttm": 16, "mttkrp16": 16, "mttkrp64": 64}[op]
        kw = {"permute": not args.identity_ranks}
        if op.startswith("ttv"):
            c = gen.config_ttv(seed=0, device=dev, scale=sc, **kw)
        elif op == "ttm":
            c = gen.config_ttm(seed=0, device=dev, scale=sc, R=R, **kw)
        else:
            c = gen.config_mttkrp(seed=0, device=dev, scale=sc, R=R, **kw)
        dims = c["dims"]
        if args.lexi_sweeps:
            from synth import lexi
            (i, j, k), labels = lexi.lexi_relabel(c["coo"][:3], dims, args.lexi_sweeps)
            (i, j, k), vals = lexi.sort_nonzeros((i, j, k), dims, c["coo"][3])
            for name, m in (("v", 2), ("U", 2), ("C", 2), ("B", 1)):      # dense operands follow their mode's new labels
                if name in c:
                    moved = torch.empty_like(c[name])
                    moved[labels[m]] = c[name]
                    c[name] = moved
            del labels
        else:
            i, j, k, vals = c["coo"]
        nnz = vals.numel()
        L = fmt.pack_coo(dims, (i, j, k), vals) if op == "ttv_coo" else fmt.pack_csf3(dims, i, j, k, vals)
        touched_k = count_distinct(k)
        if op == "ttv_coo":
            nfib = count_distinct(i * dims[1] + j)
            n1 = count_distinct(i)
        else:
            nfib, n1 = int(L.crd[1].numel()), int(L.crd[0].numel())
        del i, j, k
        X = comet.from_levels(L).set_variant(args.variant)
        extra = {"nnz": nnz, "nfib": nfib, "n1": n1, "dims": list(dims), "R": R, "draws": c["info"]["draws"]}
        # level order of the storage the operation runs on, and the mode it contracts / produces
        if mode_n is None:
            order, mode = (0, 1, 2), (0 if op.startswith("mttkrp") else 2)
        else:
            rest = [m for m in range(3) if m != mode_n]
            order, mode = ((mode_n, *rest) if op.startswith("mttkrp") else (*rest, mode_n)), mode_n
            t0 = time.perf_counter()
            Xr = comet.comet_tensor_reorder(X, order).set_variant(args.variant)
            torch.cuda.synchronize()
            extra["reorder_s"] = round(time.perf_counter() - t0, 4)
            touched_k = count_distinct(Xr.crd(2))
            nfib, n1 = int(Xr.crd(1).numel()), int(Xr.crd(0).numel())
            extra.update(nfib=nfib, n1=n1, level_order=list(order))
            keep["X0"], X = X, Xr
        ld = [dims[m] for m in order]           # sizes per level
        where = "%s, levels hold modes %s" % ("x".join(map(str, dims)), "".join(str(m + 1) for m in order))
        if op in ("ttv", "ttv_coo"):
            v = c["v"] if mode_n is None else gen.dense_operand(0, 8, (ld[2],), dev)
            Y = comet.comet_ttv(X, mode, v)
            fn = lambda: comet.comet_ttv(X, mode, v, Y)
            flops = 2 * nnz
            nbytes = (12 if op == "ttv" else 20) * nnz + 16 * nfib + 8 * touched_k
            desc = "TTV mode %d %s %s, %d nnz, %d fibers, Zipf(1.3)" % (mode + 1, "CSF" if op == "ttv" else "COO", where, nnz, nfib)
            keep.update(X=X, L=L, v=v, Y=Y)
        elif op == "ttm":
            U = c["U"] if mode_n is None else gen.dense_operand(0, 8, (ld[2], R), dev)
            Y = comet.comet_ttm(X, mode, U)
            fn = lambda: comet.comet_ttm(X, mode, U, Y)
            flops = 2 * R * nnz
            nbytes = 12 * nnz + (8 + 8 * R) * nfib + 8 * R * touched_k
            desc = "TTM mode %d CSF %s, %d nnz, %d fibers, U %dx%d" % (mode + 1, where, nnz, nfib, ld[2], R)
            extra["gather_bytes"] = 8 * R * nnz
            extra["touched_row_bytes"] = 8 * R * touched_k
            keep.update(X=X, L=L, U=U, Y=Y)
        else:
            if mode_n is None:
                fs = [None, c["B"], c["C"]]
            else:
                fs = [None if m == mode else gen.dense_operand(0, 8 + m, (dims[m], R), dev) for m in range(3)]
            M = torch.empty((ld[0], R), dtype=torch.float64, device=dev)
            fn = lambda: comet.comet_mttkrp(X, mode, fs, M)
            touched_j = count_distinct(L.crd[1]) if mode_n is None else count_distinct(X.crd(1))
            flops = 2 * R * (nnz + nfib)
            nbytes = 12 * nnz + 8 * nfib + 8 * n1 + 8 * R * (touched_j + touched_k + ld[0])
            desc = "MTTKRP mode %d CSF %s, %d nnz, %d fibers, %d slices, R=%d" % (mode + 1, where, nnz, nfib, n1, R)
            extra["gather_bytes"] = 8 * R * (nnz + nfib)
            extra["touched_row_bytes"] = 8 * R * (touched_j + touched_k)
            keep.update(X=X, L=L, fs=fs, M=M)
        op = full_op
    torch.cuda.synchronize()
    gen_s = time.perf_counter() - t_gen
    steps = args.steps
    tm = time_steps(fn, steps, args.warmup)
    ms = tm["mean_ms"]
    if op == "spmv":
        extra.update(small_problem_latency(fn, keep["y"], dev))
    if op in CALIBRATION:
        extra["rows_per_s"] = round(nnz / (ms * 1e-3), 1)
        extra["bytes_per_clk_per_cu"] = round(nbytes / (ms * 1e-3) / 2.4e9 / 256, 2)
    if "gather_bytes" in extra:
        # second roofline: every operand-row gather counted as HBM traffic (no cache reuse at all) instead of
        # each touched row once -- the upper bracket of what the call has to move
        streamed = nbytes - extra.get("touched_row_bytes", 0)
        extra["roofline_no_reuse"] = roofline(streamed + extra["gather_bytes"], ms)
    entry = {"workload": desc, "ms": round(ms, 5), "median_ms": round(tm["median_ms"], 5),
             "min_ms": round(tm["min_ms"], 5), "gflops": round(flops / (ms * 1e-3) / 1e9, 2), "flops": int(flops),
             "roofline": roofline(nbytes, ms, op, args.scale == 1.0 and not args.identity_ranks), "setup_s": round(gen_s, 2), **extra}
    log("[bench] %-9s %s: %.4f ms/step  %.1f GFLOP/s  %.1f GB/s (%.1f%% of 8 TB/s)  [setup %.1fs]" % (
        op, desc, ms, entry["gflops"], entry["roofline"]["achieved"], 100 * entry["roofline"]["frac"], gen_s))
    if op == "spmv":
        log("[bench]           launch-bound: cold %s us, graph replay %s us per call (matches eager: %s)" % (
            extra.get("cold_us"), extra.get("graph_replay_us_per_call"), extra.get("graph_replay_matches_eager")))
    return entry, keep


def cpu_baseline_spmm(keep, budget_nnz=40_000_000):
    """The CPU oracle, as it stands, on the leading rows of the headline matrix: once on one thread, and once
    on every core this process may use -- the same C function called on row-disjoint pieces of the coordinate
    list from a thread pool (the rows of C are disjoint, so the arithmetic per element is unchanged)."""
    import concurrent.futures
    import numpy as np
    import torch
    import oracle
    rows, cols, vals = keep["coo"]
    n = keep["n"]
    nnz = int(vals.numel())
    m = min(nnz, budget_nnz)
    last_row = int(rows[m - 1]) if m else 0
    nrows = last_row            # rows 0 .. last_row-1 are complete within the first m nonzeros
    if nrows <= 0:
        nrows, m = n, nnz
    else:
        m = int(torch.searchsorted(rows, torch.tensor([nrows], device=rows.device))[0])
    r_h, c_h, v_h = rows[:m].cpu().numpy(), cols[:m].cpu().numpy(), vals[:m].cpu().numpy()
    B_h = keep["B"].cpu().numpy()
    R = B_h.shape[1]
    t0 = time.perf_counter()
    ref, absum = oracle.spmm(r_h, c_h, v_h, (nrows, n), B_h)
    dt = time.perf_counter() - t0
    got = keep["C"][:nrows].cpu().numpy()
    ok = bool(np.all(np.abs(got - ref) <= 1e-10 * np.abs(ref) + 1e-12 * absum))
    # all cores: pieces of about equal nonzero count, cut at row boundaries
    cores = len(os.sched_getaffinity(0))
    cuts = [0]
    for q in range(1, cores):
        p = int(np.searchsorted(r_h, r_h[min(m - 1, q * m // cores)], side="left"))
        if p > cuts[-1]:
            cuts.append(p)
    cuts.append(m)
    pieces = []
    for a, b in zip(cuts[:-1], cuts[1:]):
        r0 = int(r_h[a])
        r1 = int(r_h[b - 1]) + 1
        pieces.append((r0, r1, (r_h[a:b] - r0).astype(np.int32), c_h[a:b], v_h[a:b]))

    def run(piece):
        r0, r1, rr, cc, vv = piece
        return r0, r1, oracle.spmm(rr, cc, vv, (r1 - r0, n), B_h)[0]

    t0 = time.perf_counter()
    with concurrent.futures.ThreadPoolExecutor(max_workers=len(pieces)) as pool:
        outs = list(pool.map(run, pieces))
    dt_all = time.perf_counter() - t0
    same = all(np.array_equal(o[np.unique(p[2])], ref[r0:r1][np.unique(p[2])]) for (r0, r1, o), p in zip(outs, pieces))
    return {"value": round(2 * R * m / dt / 1e9, 3), "unit": "GFLOP/s", "cores": 1, "kind": "oracle",
            "sample": "rows 0..%d of the SpMM matrix (%d of %d nnz), %.1f s" % (nrows - 1, m, nnz, dt),
            "parity_on_sample": ok,
            "all_cores": {"value": round(2 * R * m / dt_all / 1e9, 3), "unit": "GFLOP/s", "cores": len(pieces),
                          "cores_available": cores, "seconds": round(dt_all, 2), "same_values_as_one_thread": bool(same),
                          "how": "the same oracle function on row-disjoint pieces, one thread each"}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=25)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--ops", type=str, default=",".join(ALL_OPS))
    ap.add_argument("--scale", type=float, default=1.0, help="shrink every configuration (testing only)")
    ap.add_argument("--variant", type=int, default=0, help="0 auto, 1 simple kernels, 2 tiled kernels")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--lexi-sweeps", type=int, default=0,
                    help="relabel the coordinates lexicographically (synth/lexi.py, Section 7 of the paper) this many "
                         "sweeps over all modes before packing; the on/off experiment of the reordering")
    ap.add_argument("--identity-ranks", action="store_true",
                    help="tensor configs: Zipf rank r maps to coordinate r (clusters the nonzeros) instead of a seeded permutation")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        log("bench.py: this build runs on one GPU only (no sharding, no collectives); run it with --gpus 1.")
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        sys.exit(1)
    from paper_2102_05187_amd import build as hipbuild
    hipbuild.build_if_missing()
    import paper_2102_05187_amd as comet
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    ops = [o for o in args.ops.split(",") if o]
    if "spmm" in ops:                       # headline first
        ops = ["spmm"] + [o for o in ops if o != "spmm"]
    kernels, head_keep = {}, None
    cpu = None
    for op in ops:
        entry, keep = run_op(op, args, comet, dev)
        kernels[op] = entry
        if op == "spmm":
            head_keep = keep
            if not args.no_cpu_baseline:
                cpu = cpu_baseline_spmm(keep)
                log("[bench] cpu oracle: %s GFLOP/s on %s (parity on sample: %s); all %d cores: %s GFLOP/s" % (
                    cpu["value"], cpu["sample"], cpu["parity_on_sample"], cpu["all_cores"]["cores"], cpu["all_cores"]["value"]))
        del keep
        head_keep = None
        torch.cuda.empty_cache()
    head = kernels.get("spmm") or next(iter(kernels.values()))
    line = {
        "metric": "GFLOP/s + achieved HBM GB/s (% of peak) for SpMV, SpMM, TTM, MTTKRP",
        "value": head["gflops"], "unit": "GFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64", "data": "synthetic",
        "config": {"workload": head["workload"], "index_dtype": "int32", "scale": args.scale, "variant": args.variant,
                   "zipf_rank_to_coordinate": "identity" if args.identity_ranks else "seeded permutation"},
        "roofline": head["roofline"], "cpu_baseline": cpu, "kernels": kernels,
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
