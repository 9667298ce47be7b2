#!/usr/bin/env python3
"""Benchmark of the ABFT-checked u8 x s8 -> s32 GEMM on one MI355X (and, under "eb", of the
ABFT-checked EmbeddingBag, the paper's second operator).

A step is one pass of the hot path over one batch of synthetic input already resident
in HBM: the checked GEMM call (product with the checksum column folded in, row sums,
comparison, flags, store of C_temp, plus the requantization epilogue for the workloads
that have one).  The encode/pack of the weight is done once outside the timed region,
as the method prescribes (the weight is encoded once for many products), and its time
is reported separately as pack_ms.

Prints ONE JSON line.  `value` is checked-GEMM TOPS (2*M*N*K per step; the checksum
columns are not counted as useful work).
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

PEAK_INT8_TOPS = 5000.0      # MI355X dense int8 MFMA, published
PEAK_HBM_GBS = 8000.0        # MI355X HBM3E, published


def algorithmic_bytes(wl, want_c=True, want_q=False):
    """Bytes the method itself must move per GEMM: A, B, the checksum column (4 bytes
    per k), the outputs and the flags (+ column offsets and multipliers when requantizing)."""
    M, N, K = wl.M, wl.N, wl.K
    b = M * K + K * N + 4 * K + 4 * M
    if want_c:
        b += 4 * M * N
    if want_q:
        b += M * N + 4 * N + 4 * N
    return b


class Job:
    """Device-resident operands and outputs of one workload."""

    def __init__(self, b, torch, cfg, n_rot=1, mod127=False, accumulate=True):
        self.mod127 = mod127
        # errCount as a counter the caller zeroes and the launches add to (Algorithm 1's errCount++), or overwritten
        self.count_flag = b.ABFT_ERRCOUNT_ACCUMULATE if accumulate else 0
        from paper_2103_00130_amd import workloads as w
        self.b, self.torch = b, torch
        self.ops = w.make_operands(cfg)
        self.wl = wl = self.ops.wl
        self.A = torch.from_numpy(self.ops.A).cuda()
        B = torch.from_numpy(self.ops.B).cuda()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        self.Bp = [b.abft_pack_b_checksum(B)]
        torch.cuda.synchronize()
        self.pack_ms = (time.perf_counter() - t0) * 1e3
        t0 = time.perf_counter()
        for _ in range(n_rot - 1):      # distinct copies so that caches cannot hold the weight
            self.Bp.append(b.abft_pack_b_checksum(B))
        torch.cuda.synchronize()
        if n_rot > 1:
            self.pack_ms = (time.perf_counter() - t0) * 1e3 / (n_rot - 1)
        self.C = torch.empty((wl.M, wl.N), dtype=torch.int32, device="cuda")
        self.flags = torch.empty(wl.M, dtype=torch.int32, device="cuda")
        self.cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
        self.ws = b.Workspace(wl.M, self.Bp[0])
        self.rq = self.Cq = None
        if self.ops.mult is not None:
            self.mult = torch.from_numpy(self.ops.mult).cuda()
            self.rq = b.make_requant(wl.zA, wl.zC, self.mult)
            self.Cq = torch.empty((wl.M, wl.N), dtype=torch.uint8, device="cuda")
        self.i = 0

    def step(self, check=True, inj=None, n_inj=0, variant=0):
        b = self.b
        Bp = self.Bp[self.i % len(self.Bp)]
        self.i += 1
        b.abft_gemm_u8s8s32_checked(self.A, Bp, self.C, self.flags, self.cnt, rq=self.rq, Cq=self.Cq, inj=inj,
                                    n_inj=n_inj, flags=((b.ABFT_MOD127 if self.mod127 else b.ABFT_CHECK) if check else b.ABFT_NOCHECK) | variant | self.count_flag,
                                    workspace=self.ws.tensor)

    def time_steps(self, steps, warmup, check=True, variant=0, graph=True):
        """Average milliseconds per step: HIP events on the launching stream around `steps` launches.
        With graph=True the `steps` launches are captured once into a HIP graph and replayed, so that
        the figure is the device's back-to-back rate and not the Python caller's launch rate."""
        torch = self.torch
        for _ in range(warmup):
            self.step(check, variant=variant)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        if graph:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                for _ in range(steps):
                    self.step(check, variant=variant)
            g.replay()                      # untimed first replay
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            e0.record()
            g.replay()
            e1.record()
        else:
            t0 = time.perf_counter()
            e0.record()
            for _ in range(steps):
                self.step(check, variant=variant)
            e1.record()
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3 / steps
        return e0.elapsed_time(e1) / steps, wall_ms


def detection_sample(job, n=200):
    """Seeded single-bit flips in C accumulators; returns (detected, corrupted, false_pos_rows)."""
    import numpy as np
    from paper_2103_00130_amd import workloads as w
    torch, b, wl = job.torch, job.b, job.wl
    r, c, bit = w.draw_flips(wl.index, "C", n)
    detected = wrong_rows = 0
    for t in range(n):
        inj = b.make_injections([(int(r[t]), int(c[t]), 1 << int(bit[t]))])
        job.cnt.zero_()
        job.step(True, inj=inj, n_inj=1)
        f = job.flags
        hit = int(f[int(r[t])].item())
        total = int(job.cnt.item())
        detected += hit
        wrong_rows += total - hit
    return detected, n, wrong_rows


def recovery_sample(job, rows=(1, 64)):
    """Wall time of detect -> recompute for a launch in which `n` rows were hit: the checked GEMM with n
    injected faults in distinct rows, then abft_recompute_flagged_rows (which synchronises)."""
    import numpy as np
    from paper_2103_00130_amd import workloads as w
    torch, b, wl = job.torch, job.b, job.wl
    out = {}
    r, c, bit = w.draw_flips(wl.index, "C", 4 * max(rows))
    _, first = np.unique(r, return_index=True)
    first = np.sort(first)
    scratch = torch.empty(b.abft_recover_scratch_bytes(wl.M, 256, job.Bp[0]), dtype=torch.uint8, device="cuda")
    for n in rows:
        if n > min(wl.M, len(first)):
            continue
        sel = first[:n]
        inj = b.make_injections([(int(r[t]), int(c[t]), 1 << int(bit[t])) for t in sel])
        best = None
        for _ in range(5):
            job.cnt.zero_()
            job.step(True, inj=inj, n_inj=n)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            before, after = b.abft_recompute_flagged_rows(job.A, job.Bp[0], job.C, job.flags, job.cnt, rq=job.rq, Cq=job.Cq,
                                                          max_rows_per_pass=256, scratch=scratch)
            dt = (time.perf_counter() - t0) * 1e6
            assert (before, after) == (n, 0), (before, after)
            best = dt if best is None else min(best, dt)
        out[f"{n}_rows_us"] = best
    # recomputation without the host round trip (the row count bounds the kernels on the device): device time
    t = int(first[0])
    inj1 = b.make_injections([(int(r[t]), int(c[t]), 1 << int(bit[t]))])
    scratch64 = torch.empty(b.abft_recover_scratch_bytes(wl.M, 64, job.Bp[0]), dtype=torch.uint8, device="cuda")
    status = torch.empty(2, dtype=torch.int32, device="cuda")
    best = None
    for _ in range(5):
        job.cnt.zero_()
        job.step(True, inj=inj1, n_inj=1)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        b.abft_recompute_flagged_rows_async(job.A, job.Bp[0], job.C, job.flags, job.cnt, rq=job.rq, Cq=job.Cq, max_rows=64,
                                            scratch=scratch64, status=status)
        e1.record()
        torch.cuda.synchronize()
        assert status.cpu().tolist() == [1, 0], status
        dt = e0.elapsed_time(e1) * 1e3
        best = dt if best is None else min(best, dt)
    out["recompute_async_1_row_us"] = best
    # the other recovery path: locate the one faulty element with the column check (Eq. 2a) and rewrite it
    # (asynchronous; device time between two events on the launching stream, best of five)
    if job.rq is None or job.C is not None:
        t = int(first[0])
        inj = b.make_injections([(int(r[t]), int(c[t]), 1 << int(bit[t]))])
        loc_scratch = torch.empty(b.abft_locate_scratch_bytes(job.Bp[0]), dtype=torch.uint8, device="cuda")
        report = torch.empty(8, dtype=torch.int32, device="cuda")
        best = None
        for _ in range(5):
            job.cnt.zero_()
            job.step(True, inj=inj, n_inj=1)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            b.abft_locate_correct(job.A, job.Bp[0], job.C, job.flags, job.cnt, rq=job.rq, Cq=job.Cq, report=report, scratch=loc_scratch)
            e1.record()
            torch.cuda.synchronize()
            rep = report.cpu().numpy()
            assert int(rep[0]) == b.ABFT_LOCATE_CORRECTED and (int(rep[1]), int(rep[2])) == (int(r[t]), int(c[t])), rep
            dt = e0.elapsed_time(e1) * 1e3
            best = dt if best is None else min(best, dt)
        out["locate_correct_1_element_us"] = best
    return out


def cpu_baseline(job, target_s=12.0):
    """The CPU oracle as it stands, timed on a bounded row sample of the same workload."""
    import numpy as np
    from oracle import abft_oracle as oracle
    wl, ops = job.wl, job.ops
    probe_rows = min(wl.M, 64)
    t0 = time.perf_counter()
    oracle.gemm_u8s8s32(ops.A[:probe_rows], ops.B)
    dt = time.perf_counter() - t0
    rows = int(min(wl.M, max(probe_rows, probe_rows * target_s / max(dt, 1e-6))))
    A = np.ascontiguousarray(ops.A[:rows])
    t0 = time.perf_counter()
    S = oracle.b_checksum(ops.B)
    C = oracle.gemm_u8s8s32(A, ops.B)
    chk = oracle.row_checksum(A, S)
    rs = oracle.row_sums(C)
    oracle.compare(rs, chk)
    dt = time.perf_counter() - t0
    return {"value": 2.0 * rows * wl.N * wl.K / dt / 1e12, "unit": "TOPS", "cores": oracle.num_threads(),
            "kind": "oracle", "sample": f"first {rows} of {wl.M} rows of A against the full B "
            f"(checksum, product, row sums, comparison), {dt:.1f} s wall"}


def smallm_sweep(b, torch, steps, warmup, count_flag=0, M=16,
                 shapes=((4096, 2048), (4096, 4096), (8192, 8192), (16384, 16384), (16384, 32768))):
    """The streaming kernel on weights from 8 MiB to 512 MiB (N x K int8), M = 16: how close to the HBM
    roofline it gets once the weight is large enough to amortise the launch.  Operands are seeded draws on
    the device (timing only; parity of these kernels is the tests' business)."""
    out = []
    gen = torch.Generator(device="cuda")
    gen.manual_seed(210300130)
    A = torch.randint(0, 256, (M, max(k for _, k in shapes)), dtype=torch.uint8, device="cuda", generator=gen)
    for N, K in shapes:
        n_rot = max(2, -(-(768 << 20) // (N * K)))
        Bps = []
        for _ in range(n_rot):
            B = torch.randint(-127, 128, (K, N), dtype=torch.int8, device="cuda", generator=gen)
            Bps.append(b.abft_pack_b_checksum(B))
            del B
        a = A[:, :K]
        C = torch.empty((M, N), dtype=torch.int32, device="cuda")
        flags = torch.empty(M, dtype=torch.int32, device="cuda")
        cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
        ws = b.Workspace(M, Bps[0])
        n_steps = max(n_rot * 2, min(steps, (4 << 30) // (N * K)))

        def run(check, n):
            for i in range(n):
                b.abft_gemm_u8s8s32_checked(a, Bps[i % n_rot], C, flags, cnt,
                                            flags=(b.ABFT_CHECK if check else b.ABFT_NOCHECK) | count_flag, workspace=ws.tensor)

        def timed(check):
            run(check, min(warmup, n_rot * 2))
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                run(check, n_steps)
            g.replay()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            g.replay()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / n_steps
        ms_c = min(timed(True), timed(True))
        ms_u = min(timed(False), timed(False))
        by = M * K + K * N + 4 * K + 4 * M * N + 4 * M
        out.append({"M": M, "N": N, "K": K, "weight_MiB": N * K / 2**20, "weight_copies_rotated": n_rot, "steps": n_steps,
                    "us_checked": ms_c * 1e3, "us_unchecked": ms_u * 1e3, "abft_overhead_pct": 100.0 * (ms_c - ms_u) / ms_u,
                    "algorithmic_bytes": by, "gbs": by / ms_c / 1e6, "hbm_frac": by / ms_c / 1e6 / PEAK_HBM_GBS,
                    "tops_checked": 2.0 * M * N * K / ms_c / 1e9})
        for Bp in Bps:
            Bp.destroy()
        del Bps, C
        torch.cuda.empty_cache()
    return out


def clock_trace(b, torch, args):
    """Shader clock evidence for the matrix-core roofline (needs the diagnostic library:
    `python -m paper_2103_00130_amd.build --clock-trace`, then ABFT_LIBRARY=<.../libabftgemm_clocktrace.so>).
    Three measurements, each from cycle counter / 100 MHz wall counter pairs taken on the device:
    the idle clock, a register-only MFMA load (no operand traffic), and the phases of the tiled GEMM itself."""
    import statistics
    out = {}
    probe = torch.zeros(4, dtype=torch.int64, device="cuda")
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    b.abft_clock_probe(probe, 2000)
    torch.cuda.synchronize()
    o = probe.cpu().tolist()
    out["idle_clock_ghz"] = (o[3] - o[1]) / ((o[2] - o[0]) / 100.0) / 1e3
    peak = torch.zeros(4 * 256, dtype=torch.int64, device="cuda")
    iters = 40000
    for _ in range(3):
        b.abft_mfma_peak_probe(peak, iters)
    torch.cuda.synchronize()
    pk = peak.cpu().view(256, 4).tolist()
    us = statistics.median((r1 - r0) / 100.0 for c0, r0, c1, r1 in pk)
    out["register_only_mfma"] = {
        "clock_ghz": statistics.median((c1 - c0) / ((r1 - r0) / 100.0) / 1e3 for c0, r0, c1, r1 in pk),
        "cycles_per_mfma": statistics.median((c1 - c0) / (4.0 * iters) for c0, r0, c1, r1 in pk),
        "pops": 256 * 4 * iters * 4 * 65536.0 / us / 1e9, "us": us,
        "note": "256 workgroups x 4 wavefronts x %d rounds of 4 independent 32x32x32 int8 MFMAs, operands in registers" % iters}
    job = Job(b, torch, args.workload, accumulate=not args.overwrite_count)
    wl = job.wl
    n_wg = ((wl.M + 63) // 64) * ((wl.N + 63) // 64)
    trace = torch.zeros(6 * n_wg, dtype=torch.int64, device="cuda")
    for check in (True, False):
        b.abft_clock_trace(None)
        for _ in range(args.warmup):
            job.step(check)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for _ in range(200):
                job.step(check)
        trace.zero_()
        torch.cuda.synchronize()
        b.abft_clock_trace(trace)
        # the trace pointer travels in the kernel arguments, which the graph captured without it: the traced
        # launches are plain launches at the end of a warm run of graph replays
        g.replay()
        g.replay()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        with torch.cuda.stream(side):
            b.abft_clock_probe(probe, 5000, stream=side)
        e0.record()
        for _ in range(50):
            job.step(check)
        e1.record()
        g.replay()
        torch.cuda.synchronize()
        b.abft_clock_trace(None)
        o = probe.cpu().tolist()
        rows = [r for r in trace.cpu().view(n_wg, 6).tolist() if r[1] != 0 and r[5] != 0]
        stages = (wl.K + 127) // 128
        loop_cyc = [r[2] - r[0] for r in rows]
        loop_us = [(r[3] - r[1]) / 100.0 for r in rows]
        epi_cyc = [r[4] - r[2] for r in rows]
        epi_us = [(r[5] - r[3]) / 100.0 for r in rows]
        out["checked" if check else "unchecked"] = {
            "workgroups_traced": len(rows), "us_per_launch_traced": e0.elapsed_time(e1) * 1e3 / 50,
            "k_loop_us": statistics.median(loop_us), "k_loop_cycles_per_stage": statistics.median(loop_cyc) / stages,
            "k_loop_clock_ghz": statistics.median(c / u / 1e3 for c, u in zip(loop_cyc, loop_us) if u > 0),
            "epilogue_us": statistics.median(epi_us),
            "epilogue_clock_ghz": statistics.median(c / u / 1e3 for c, u in zip(epi_cyc, epi_us) if u > 0),
            "concurrent_probe_clock_ghz": (o[3] - o[1]) / max((o[2] - o[0]) / 100.0, 1e-9) / 1e3,
            "k_loop_pops": 2.0 * wl.M * wl.N * wl.K / statistics.median(loop_us) / 1e9,
            "mfma_cycles_per_stage_at_full_rate": 2048 if max(wl.M, wl.N) >= 2048 else None}
    out["workload"] = wl.name
    out["note"] = ("clock = shader cycles / wall time between two samples on the device; the peak of 5.0 POP/s is quoted at 2.4 GHz, "
                   "so the matrix-core ceiling at a sustained clock f is 5.0 * f / 2.4")
    return out


def splitk_points(b, torch, steps, count_flag, shapes=((256, 1024, 8192), (128, 128, 16384), (256, 512, 4096))):
    """Few 64x64 tiles and a long K: the library splits K across workgroups when the workspace has room for the
    partial tiles; the same launch on a workspace of the row words alone runs unsplit.  Seeded draws on the device."""
    out = []
    gen = torch.Generator(device="cuda")
    gen.manual_seed(210300131)
    for M, N, K in shapes:
        A = torch.randint(0, 256, (M, K), dtype=torch.uint8, device="cuda", generator=gen)
        B = torch.randint(-127, 128, (K, N), dtype=torch.int8, device="cuda", generator=gen)
        Bp = b.abft_pack_b_checksum(B)
        C = torch.empty((M, N), dtype=torch.int32, device="cuda")
        flags = torch.empty(M, dtype=torch.int32, device="cuda")
        cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
        full = b.Workspace(M, Bp).tensor
        rows_only = torch.zeros(b.lib.abft_gemm_workspace_bytes(M, None) // 4, dtype=torch.int32, device="cuda")
        n = max(50, min(steps, 400))

        def timed(ws, check):
            def run():
                b.abft_gemm_u8s8s32_checked(A, Bp, C, flags, cnt, flags=(b.ABFT_CHECK if check else b.ABFT_NOCHECK) | count_flag,
                                            workspace=ws)
            for _ in range(20):
                run()
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                for _ in range(n):
                    run()
            g.replay()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            g.replay()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) * 1e3 / n
        out.append({"M": M, "N": N, "K": K, "split": full.numel() > rows_only.numel(),
                    "us_checked": timed(full, True), "us_unchecked": timed(full, False),
                    "us_checked_unsplit": timed(rows_only, True), "us_unchecked_unsplit": timed(rows_only, False)})
        Bp.destroy()
    return out


CALIB_COPY_BYTES = 256 << 20
GEMM_KERNEL_TAGS = ("gemm_tile_async_kernel", "gemm_tile_kernel", "gemm_smallm_kernel")


def pmc_child(args):
    """Body of the profiled child process: one calibration copy of known size, then a few
    checked launches of the workload (no graph, no timing)."""
    import torch
    from paper_2103_00130_amd import binding as b
    torch.cuda.set_device(0)
    src = torch.zeros(CALIB_COPY_BYTES // 4, dtype=torch.int32, device="cuda")
    dst = torch.empty_like(src)
    job = Job(b, torch, args.workload, mod127=args.mod127, accumulate=not args.overwrite_count)
    torch.cuda.synchronize()
    b.abft_calib_copy(src, dst)
    for _ in range(4):
        job.step(True, variant=args.variant)
    torch.cuda.synchronize()


def measure_traffic(args, child_args=None, tags=None):
    """HBM bytes per checked launch from two counter passes of rocprofv3 (FETCH_SIZE, then
    WRITE_SIZE), each over a child process running pmc_child, each scaled by what the same
    counter reads for the calibration copy.  Runs before this process touches the GPU.
    Returns (dict or None, note)."""
    import csv
    import glob
    import shutil
    import subprocess
    import tempfile
    if shutil.which("rocprofv3") is None:
        return None, "rocprofv3 not found"
    out = {}
    for counter, key in (("FETCH_SIZE", "read"), ("WRITE_SIZE", "write")):
        tmp = tempfile.mkdtemp(prefix="abft_pmc_")
        env = dict(os.environ, TMPDIR=tmp)
        cmd = ["timeout", "-s", "KILL", "170", "rocprofv3", "--pmc", counter, "-d", tmp, "-o", "pmc",
               "--output-format", "csv", "--", sys.executable, os.path.join(ROOT, "bench.py")]
        cmd += child_args if child_args is not None else (
            ["--pmc-child", "--workload", str(args.workload), "--variant", str(args.variant)] + (["--mod127"] if args.mod127 else [])
            + (["--overwrite-count"] if args.overwrite_count else []))
        try:
            r = subprocess.run(cmd, cwd=tmp, env=env, capture_output=True, text=True)
            files = glob.glob(os.path.join(tmp, "**", "*counter_collection.csv"), recursive=True)
            if r.returncode != 0 or not files:
                return None, f"{counter} pass failed (exit {r.returncode})"
            per_dispatch = {}
            for row in csv.DictReader(open(files[0])):
                if row["Counter_Name"] != counter:
                    continue
                k = (row["Dispatch_Id"], row["Kernel_Name"])
                per_dispatch[k] = per_dispatch.get(k, 0.0) + float(row["Counter_Value"])
            cal = [v for (d, n), v in per_dispatch.items() if "calib_copy_kernel" in n]
            gemm = [v for (d, n), v in sorted(per_dispatch.items(), key=lambda kv: int(kv[0][0]))
                    if any(t in n for t in (tags or GEMM_KERNEL_TAGS))]
            if len(cal) != 1 or cal[0] <= 0 or len(gemm) < 2:
                return None, f"{counter} pass: unexpected dispatch list"
            gemm = gemm[1:]           # the first launch also pays for cold instruction and data caches
            scale = CALIB_COPY_BYTES / cal[0]
            out[key] = sum(gemm) / len(gemm) * scale
            out[key + "_counter_units_per_byte"] = 1.0 / scale
        finally:
            shutil.rmtree(tmp, ignore_errors=True)
    return out, "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE per checked launch, scaled by a 256 MiB copy kernel"


# ------------------------------------------------------------------------------------------------
# Second operator: the ABFT-checked EmbeddingBag (include/abft_eb.h).  A step is one call of
# abft_eb_u8_checked over one batch of lookups; the 4,000,000-row tables of Table I are laid end to
# end in one allocation of at least 2 GiB and every step of a pass uses an index set of its own, so
# that lookups are not served from cache (the paper flushes its caches for the same reason).
EB_KERNEL_TAGS = ("eb_batch_kernel", "eb_group_kernel")
EB_TABLE_MIN_BYTES = 2 << 30


class EbJob:
    def __init__(self, b, torch, wl, max_sets=2048, aligned=False, bits=8):
        import numpy as np
        from paper_2103_00130_amd import eb_workloads as ew
        self.b, self.torch, self.wl = b, torch, wl
        self.bits = bits
        rec = wl.d * bits // 8 + 16
        rng = ew.rng_for(900 + wl.d)
        self.T, self.scale, self.bias = ew.draw_table(rng, wl.rows, wl.d, wl.regime, bits)
        copies = max(1, -(-EB_TABLE_MIN_BYTES // (wl.rows * rec)))
        self.rows_big = wl.rows * copies
        T = torch.from_numpy(self.T).cuda().repeat(copies, 1)
        scale = torch.from_numpy(self.scale).cuda().repeat(copies)
        bias = torch.from_numpy(self.bias).cuda().repeat(copies)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        self.Tp = b.abft_eb_pack_rowsum(T, scale, bias, (b.ABFT_EB_PACK_LINE_ALIGNED if aligned else b.ABFT_EB_PACK_COMPACT) |
                                        (b.ABFT_EB_PACK_INT4 if bits == 4 else 0))
        torch.cuda.synchronize()
        self.pack_ms = (time.perf_counter() - t0) * 1e3
        del T
        self.table_bytes = self.rows_big * b.abft_eb_table_dims(self.Tp)[2]
        touched = wl.n_bags * wl.pooling * rec
        self.n_sets = int(min(max_sets, max(4, (1 << 30) // touched)))
        self.host_sets, self.sets, n_idx = [], [], 0
        for s_ in range(self.n_sets):
            indices, offsets = ew.draw_bags(rng, self.rows_big, wl.n_bags, wl.pooling, "spread")
            weights = ew.draw_weights(rng, indices.size) if wl.weighted else None
            if s_ < 64:
                self.host_sets.append((indices, offsets, weights))
            self.sets.append((torch.from_numpy(indices).cuda(), torch.from_numpy(offsets).cuda(),
                              None if weights is None else torch.from_numpy(weights).cuda()))
            n_idx += indices.size
        self.mean_indices = n_idx / self.n_sets
        self.R = torch.empty((wl.n_bags, wl.d), dtype=torch.float32, device="cuda")
        self.flags = torch.empty(wl.n_bags, dtype=torch.int32, device="cuda")
        # bytes the method itself must move per call: records and indices (and weights) of the pooled
        # rows, offsets, the pooled rows written, one flag per lookup
        self.bytes_per_call = self.mean_indices * (rec + 8 + (4 if wl.weighted else 0)) + wl.n_bags * (4 * wl.d + 8 + 4)

    def call(self, s_, check=True):
        b = self.b
        idx, off, wts = self.sets[s_ % self.n_sets]
        b.abft_eb_u8_checked(self.Tp, idx, off, self.R, self.flags, weights=wts,
                             flags=b.ABFT_EB_CHECK if check else b.ABFT_EB_NOCHECK)

    def time_calls(self, check=True, reps=3):
        """Average microseconds per call: one HIP graph holding one call per index set, replayed."""
        torch = self.torch
        for s_ in range(min(self.n_sets, 8)):
            self.call(s_, check)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for s_ in range(self.n_sets):
                self.call(s_, check)
        g.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            g.replay()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / (reps * self.n_sets)

    def false_positives(self, n=32):
        bad = tot = 0
        for s_ in range(min(n, self.n_sets)):
            self.call(s_, True)
            bad += int((self.flags != 0).sum().item())
            tot += self.wl.n_bags
        return 100.0 * bad / tot

    def cpu_baseline(self, target_s=4.0):
        """The CPU oracle on the 4,000,000-row table with the same index sets folded into it."""
        from oracle import eb_oracle as oracle
        wl = self.wl
        C_T = oracle.table_rowsums(self.T, self.bits)
        t0 = time.perf_counter()
        n = 0
        while True:
            indices, offsets, weights = self.host_sets[n % len(self.host_sets)]
            oracle.checked_eb(self.T, self.scale, self.bias, indices % wl.rows, offsets, weights, C_T=C_T, bits=self.bits)
            n += 1
            dt = time.perf_counter() - t0
            if dt > target_s or n >= 4 * len(self.host_sets):
                break
        return {"value": self.bytes_per_call * n / dt / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
                "us_per_call": dt / n * 1e6,
                "sample": f"{n} calls of the oracle (lookup in float, RSum, CSum, comparison; row sums precomputed), {dt:.1f} s wall"}


def measure_eb(b, torch, wl, cpu=True, aligned=False, bits=8):
    job = EbJob(b, torch, wl, aligned=aligned, bits=bits)
    us_c = min(job.time_calls(True), job.time_calls(True))
    us_u = min(job.time_calls(False), job.time_calls(False))
    res = {
        "workload": wl.name + ("_int4" if bits == 4 else "") + ("_line_aligned" if aligned else ""), "rows": wl.rows, "d": wl.d,
        "code_bits": bits,
        "record_stride_bytes": job.table_bytes // job.rows_big, "n_bags": wl.n_bags, "pooling": wl.pooling, "weighted": wl.weighted,
        "us_per_call": us_c, "us_per_call_unchecked": us_u, "abft_overhead_pct": 100.0 * (us_c - us_u) / us_u,
        "pooled_rows_per_s": job.mean_indices / us_c * 1e6, "table_bytes": job.table_bytes,
        "index_sets_rotated": job.n_sets, "pack_ms": job.pack_ms, "false_positive_pct": job.false_positives(),
        "roofline": {"bound": "hbm", "achieved": job.bytes_per_call / us_c / 1e3, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": job.bytes_per_call / us_c / 1e3 / PEAK_HBM_GBS, "traffic": None,
                     "algorithmic_bytes": job.bytes_per_call},
    }
    if cpu:
        res["cpu_baseline"] = job.cpu_baseline()
    job.Tp.destroy()
    return res


def pmc_child_eb(spec):
    """Profiled child for the EmbeddingBag: one calibration copy, then a few checked calls (d:n_bags)."""
    import torch
    from paper_2103_00130_amd import binding as b
    from paper_2103_00130_amd import eb_workloads as ew
    torch.cuda.set_device(0)
    parts = spec.split(":")
    d, n_bags = int(parts[0]), int(parts[1])
    aligned = len(parts) > 2 and parts[2] == "aligned"      # D:N_BAGS[:aligned]  (records on 128-byte lines)
    src = torch.zeros(CALIB_COPY_BYTES // 4, dtype=torch.int32, device="cuda")
    dst = torch.empty_like(src)
    job = EbJob(b, torch, ew.EbWorkload("pmc", 4_000_000, d, n_bags, 100, False, "uniform"), max_sets=5, aligned=aligned)
    torch.cuda.synchronize()
    b.abft_calib_copy(src, dst)
    for s_ in range(5):
        job.call(s_, True)
    torch.cuda.synchronize()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--workload", type=int, default=4, help="index into the five workloads (default: dense 4096^3)")
    ap.add_argument("--others", action="store_true", help="EmbeddingBag: every width of Table I, weighted sums, 4-bit codes")
    ap.add_argument("--only-headline", action="store_true", help="time only --workload (no per-workload list, no small-M sweep)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-detection", action="store_true")
    ap.add_argument("--variant", type=lambda s: int(s, 0), default=0)
    ap.add_argument("--no-traffic", action="store_true", help="skip the two rocprofv3 counter passes")
    ap.add_argument("--mod127", action="store_true", help="check with the paper's printed modulus (8-bit checksum column, "
                    "comparison modulo 127) instead of the exact int32 checksum; tiled kernels only")
    ap.add_argument("--overwrite-count", action="store_true", help="errCount overwritten by every launch (the library's default) "
                    "instead of a counter that the launches add to (ABFT_ERRCOUNT_ACCUMULATE, what this benchmark times by default)")
    ap.add_argument("--clock-trace", action="store_true", help="print only the shader-clock evidence (idle, register-only MFMA load, "
                    "phases of the tiled GEMM); needs ABFT_LIBRARY to point at the library built with `build --clock-trace`")
    ap.add_argument("--pmc-child", action="store_true", help=argparse.SUPPRESS)
    ap.add_argument("--pmc-child-eb", type=str, default=None, help=argparse.SUPPRESS)
    ap.add_argument("--no-eb", action="store_true", help="skip the EmbeddingBag entries (reported under 'eb')")
    ap.add_argument("--eb-only", type=str, default=None, metavar="D:N_BAGS",
                    help="time only the EmbeddingBag at row width D and batch N_BAGS (Table I table, pooling 100) and print its entry")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    if args.pmc_child:
        pmc_child(args)
        return
    if args.pmc_child_eb:
        pmc_child_eb(args.pmc_child_eb)
        return
    if args.clock_trace:
        import torch
        from paper_2103_00130_amd import binding as b
        torch.cuda.set_device(0)
        print(json.dumps({"clock_trace": clock_trace(b, torch, args)}))
        return
    if args.eb_only:
        import torch
        from paper_2103_00130_amd import binding as b
        from paper_2103_00130_amd import eb_workloads as ew
        torch.cuda.set_device(0)
        d, n_bags = (int(x) for x in args.eb_only.split(":"))
        ewl = ew.EbWorkload(f"rows4000000_d{d}_pool100_batch{n_bags}", 4_000_000, d, n_bags, 100, False, "uniform")
        print(json.dumps({"eb": [measure_eb(b, torch, ewl, cpu=False)]}))
        return
    traffic, traffic_note = (None, "skipped") if args.no_traffic else measure_traffic(args)
    eb_traffic = eb_traffic_aligned = None
    if not args.no_traffic and not args.no_eb:
        eb_traffic, _ = measure_traffic(args, ["--pmc-child-eb", "64:16384"], EB_KERNEL_TAGS)
        eb_traffic_aligned, _ = measure_traffic(args, ["--pmc-child-eb", "64:16384:aligned"], EB_KERNEL_TAGS)

    import torch
    from paper_2103_00130_amd import binding as b     # fails loudly if the HIP library is missing
    from paper_2103_00130_amd import workloads as w
    torch.cuda.set_device(0)

    def measure(cfg, steps, warmup, variant=0):
        wl = w.WORKLOADS[cfg]
        hbm_bound = wl.M <= 64 and wl.K * wl.N >= (4 << 20) and not args.mod127
        # HBM-bound shapes: rotate through enough packed copies of the weight to exceed the caches
        n_rot = max(1, (768 << 20) // (wl.K * wl.N)) if hbm_bound else 1
        n_rot = min(n_rot, 128)
        job = Job(b, torch, cfg, n_rot=n_rot, mod127=args.mod127, accumulate=not args.overwrite_count)
        ms_c, wall_c = job.time_steps(steps, warmup, True, variant)
        ms_u, _ = job.time_steps(steps, warmup, False, variant)
        ms_c2, _ = job.time_steps(steps, warmup, True, variant)
        ms_u2, _ = job.time_steps(steps, warmup, False, variant)
        ms_c, ms_u = min(ms_c, ms_c2), min(ms_u, ms_u2)
        ops_per_step = 2.0 * wl.M * wl.N * wl.K
        res = {
            "workload": wl.name, "M": wl.M, "N": wl.N, "K": wl.K, "requant": wl.requant,
            "ms_per_step": ms_c, "tops_checked": ops_per_step / ms_c / 1e9, "tops_unchecked": ops_per_step / ms_u / 1e9,
            "abft_overhead_pct": 100.0 * (ms_c - ms_u) / ms_u, "pack_ms": job.pack_ms, "weight_copies_rotated": n_rot,
            "host_wall_ms_per_step": wall_c,
        }
        by = algorithmic_bytes(wl, True, job.rq is not None)
        hbm = {"bound": "hbm", "achieved": by / ms_c / 1e6, "peak": PEAK_HBM_GBS, "unit": "GB/s",
               "frac": by / ms_c / 1e6 / PEAK_HBM_GBS, "traffic": None, "algorithmic_bytes": by}
        mfma = {"bound": "mfma", "achieved": ops_per_step / ms_c / 1e9 / 1e3, "peak": PEAK_INT8_TOPS / 1e3,
                "unit": "POP/s", "frac": ops_per_step / ms_c / 1e9 / PEAK_INT8_TOPS, "traffic": None}
        if hbm_bound:
            res["roofline"] = hbm
        elif ops_per_step < 1e9:
            # ideal times of these shapes (0.03-0.16 us on either roofline) are below the latency of a launch:
            # reported as latency-bound, with both fractions for the record
            res["roofline"] = {"bound": "latency", "achieved": ms_c * 1e3, "unit": "us per launch", "peak": None, "frac": None,
                               "traffic": None, "mfma_frac": mfma["frac"], "hbm_frac": hbm["frac"],
                               "note": "launch/latency-bound: neither roofline applies at this size"}
        else:
            res["roofline"] = mfma
        return job, res

    job, main_res = measure(args.workload, args.steps, args.warmup, args.variant)
    wl = job.wl
    out = {
        "metric": "checked u8s8s32 GEMM TOPS, ABFT overhead % vs unchecked, bit-flip detection %",
        "value": main_res["tops_checked"], "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": main_res["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8", "data": "synthetic",
        "config": {"workload": wl.name, "M": wl.M, "N": wl.N, "K": wl.K, "requant": wl.requant,
                   "baseline_config_index": wl.index,
                   "check": "int8 checksum column, comparison modulo 127" if args.mod127 else "exact int32 checksum, comparison modulo 2^32",
                   "err_count": "overwritten per launch" if args.overwrite_count else
                   "a counter zeroed by the caller that launches add to (ABFT_ERRCOUNT_ACCUMULATE)"},
        "abft_overhead_pct": main_res["abft_overhead_pct"], "tops_unchecked": main_res["tops_unchecked"],
        "pack_ms": main_res["pack_ms"], "roofline": main_res["roofline"],
        "launch": "the timed steps are captured in one HIP graph and replayed (events bracket the replay)",
    }
    if traffic is not None:
        out["roofline"]["traffic"] = traffic["read"] + traffic["write"]
        out["roofline"]["traffic_read"] = traffic["read"]
        out["roofline"]["traffic_write"] = traffic["write"]
        out["roofline"]["traffic_unit"] = "bytes per launch"
        out["roofline"]["algorithmic_bytes"] = algorithmic_bytes(wl, True, job.rq is not None)
    out["roofline"]["traffic_note"] = traffic_note
    if not args.no_detection:
        det, n, wrong = detection_sample(job, 200)
        out["detection_pct"] = 100.0 * det / n
        out["detection_sample"] = f"{n} seeded single-bit flips in C accumulators, one per launch; " \
                                  f"{wrong} rows flagged other than the injected one"
    if not args.no_detection and not args.mod127:
        out["recovery"] = recovery_sample(job)
        out["recovery_note"] = ("N_rows_us: host wall time of abft_recompute_flagged_rows (gather, re-checked GEMM, scatter; synchronises); "
                                "recompute_async_1_row_us: device time of abft_recompute_flagged_rows_async (no synchronisation, one pass of up to 64 rows); "
                                "locate_correct_1_element_us: device time of abft_locate_correct (column check of Eq. 2a, repair of the located element)")
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(job)
    if not args.only_headline:
        # every workload of the baseline's list, same timing method (the headline's entry repeats the figures above)
        out["configs"] = []
        for cfg in range(len(w.WORKLOADS)):
            if cfg == args.workload:
                r = dict(main_res)
                r["roofline"] = {k: v for k, v in out["roofline"].items() if not k.startswith("traffic_note")}
            else:
                _, r = measure(cfg, args.steps, args.warmup)
            r["baseline_config_index"] = cfg
            out["configs"].append(r)
        torch.cuda.empty_cache()
        out["smallm_sweep"] = smallm_sweep(b, torch, args.steps, args.warmup, 0 if args.overwrite_count else b.ABFT_ERRCOUNT_ACCUMULATE)
        out["splitk"] = splitk_points(b, torch, args.steps, 0 if args.overwrite_count else b.ABFT_ERRCOUNT_ACCUMULATE)
        out["splitk_note"] = ("few 64x64 tiles, long K: K split across workgroups (chosen from about forty 128-k stages on) against the same "
                              "launch unsplit (a workspace without room for the partial tiles); the third shape sits below the threshold")
        out["smallm_sweep_note"] = ("streaming kernel, M = 16, weights of growing size rotated through >= 768 MiB of packed "
                                    "copies (nothing served from cache): algorithmic bytes / time against 8 TB/s")
    if not args.no_eb:
        # second operator (Algorithm 2): Table I at d = 64 and the same table under a large batch; with
        # --others every width of Table I, regular and weighted sum
        from paper_2103_00130_amd import eb_workloads as ew
        import dataclasses
        del job
        torch.cuda.empty_cache()
        eb_list = [ew.TABLE1[64], ew.LARGE_BATCH[64]]
        if args.others:
            eb_list = [ew.TABLE1[d] for d in (32, 64, 128, 256)]
            eb_list += [dataclasses.replace(ew.TABLE1[d], name=ew.TABLE1[d].name + "_weighted", weighted=True) for d in (32, 64, 128, 256)]
            eb_list += [ew.LARGE_BATCH[d] for d in (32, 64, 128, 256)]
        out["eb"] = []
        # (workload, records line-aligned): the large batches of narrow rows are also run on records that
        # never straddle a 128-byte line
        eb_runs = [(ewl, False, 8) for ewl in eb_list] + [(ewl, True, 8) for ewl in eb_list if ewl.n_bags > 1000 and ewl.d <= 64]
        if args.others:   # 4-bit codes: Table I at d = 128 (the same 64 code bytes a row as d = 64 at 8 bits) and its large batch
            eb_runs += [(ew.TABLE1[128], False, 4), (ew.LARGE_BATCH[128], False, 4)]
        for ewl, aligned, bits in eb_runs:
            r = measure_eb(b, torch, ewl, cpu=not args.no_cpu_baseline and not aligned, aligned=aligned, bits=bits)
            tr = eb_traffic_aligned if aligned else eb_traffic
            if tr is not None and ewl.name == ew.LARGE_BATCH[64].name and bits == 8:
                r["roofline"]["traffic"] = tr["read"] + tr["write"]
                r["roofline"]["traffic_read"] = tr["read"]
                r["roofline"]["traffic_write"] = tr["write"]
            out["eb"].append(r)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
