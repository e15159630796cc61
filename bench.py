#!/usr/bin/env python3
"""Benchmark of the LUT mpGEMV/mpGEMM hot path on one MI355X.

A step = one pass of the whole hot path (table precompute, lookup, bit-plane accumulate, scale
and zero, reduce, store) over the three Llama-2-7B-shaped W4A16 decode GEMVs (N=1; M x K =
4096x4096, 11008x4096, 4096x11008; group 128), inputs resident in HBM.  By default the three
GEMVs are ONE launch of tmac_mpgemv_fused_multi (tables built inside the lookup kernel, the
workgroups of one grid dealt out over the three matrices); --separate times one
tmac_mpgemv_fused launch per GEMV, --two-call tmac_precompute_lut + tmac_mpgemm per GEMV.  Every
shape cycles through a ring of distinct packed weight copies larger than twice the 256 MB
Infinity Cache, so weights come from HBM.

Launches are replayed from HIP graphs (captured once, outside the timed region) so that the
host-side cost of issuing microsecond kernels from Python does not hide the GPU time; the timed
region is bracketed by HIP events on the launching stream and by synchronize().  Before the
warm-up an untimed pre-roll of PREROLL_STEPS steps brings the clocks up, and the fixed cost of an
event pair around a graph replay (25-45 us) is cancelled by bracketing twice, once around L
calibration steps and once around L + K steps (see timed_exact), so that a short timed region
(20 steps) reads like a long one.

Prints ONE JSON line: whole-step throughput (algorithmic GB/s), the roofline of the dominant
kernel, the CPU oracle timed on the host cores as a reported baseline, and under `detail` the rest
of the metric: time per call at 1-4 bit on two shapes with the linear fit, the BitNet-shaped
ternary GEMVs, one decoder block, and TOPS-equivalent at N = 256 against the measured lookup
ceiling.  Every per-kernel figure takes at least MIN_LAUNCHES launches whatever --steps says.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
RING_MB = 576        # > 2 x 256 MB Infinity Cache
PREROLL_STEPS = 400  # untimed steps before the warm-up (clock ramp), independent of --steps
LEAD_IN_STEPS = 600  # untimed steps in front of every event bracket (about 8 ms of continuous work)
MIN_LAUNCHES = 300   # launches behind every per-kernel figure, independent of --steps

# HBM bytes of one step's launch(es) from two rocprofv3 --pmc passes (FETCH_SIZE, then WRITE_SIZE),
# each dispatch's counter scaled by what the same counter reads for the plain read kernel on a blob
# of known size; summary under profiles/.  The figures belong to the kernel sources they were taken
# with: they are emitted only while the hash of those sources is unchanged.
MEASURED_TRAFFIC = {
    "sources_sha256_16": "ecc535d5d779ce80",
    "multi": 57619129,  # bytes per step, one launch (27961 counts fetched x 2057.9 bytes per count + 76811 bytes written)
    "separate": None,   # bytes per step, three launches
}
KERNEL_SOURCES = ["paper_2407_00088_amd/csrc/tmac_perm.hip", "paper_2407_00088_amd/csrc/tmac_perm_core.h",
                  "paper_2407_00088_amd/csrc/tmac_internal.h"]


def kernel_sources_hash():
    h = hashlib.sha256()
    for f in KERNEL_SOURCES:
        with open(os.path.join(ROOT, f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def algorithmic_bytes(M, K, bits, group, N=1, act_bytes=2, out_bytes=4):
    """Bytes the method must move per call: packed indices + scales and zeros + activations + output."""
    w = M * K * bits // 8
    sz = 0 if group == 0 else M * (K // group) * 4
    return w + sz + N * K * act_bytes + N * M * out_bytes


def linear_fit(xs, ys):
    import numpy as np
    xs, ys = np.asarray(xs, dtype=np.float64), np.asarray(ys, dtype=np.float64)
    c, t0 = np.polyfit(xs, ys, 1)
    ss_res = float(((ys - (c * xs + t0)) ** 2).sum())
    ss_tot = float(((ys - ys.mean()) ** 2).sum())
    return {"us_per_bit": round(float(c), 4), "t0_us": round(float(t0), 4),
            "r2": round(1 - ss_res / ss_tot, 5) if ss_tot > 0 else None}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--ring-mb", type=int, default=RING_MB)
    ap.add_argument("--rows", type=int, default=0, help="tmac_tuning.rows_per_group override (8 or 16)")
    ap.add_argument("--sweep", action="store_true",
                    help="also: eager one-copy protocol, int8 tables, stacked and 70B-sized matrices, small batches, g sweep")
    ap.add_argument("--headline-only", action="store_true", help="skip the detail rows (for profiling the step)")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly from Python instead of graph replay")
    ap.add_argument("--prefill-only", action="store_true",
                    help="time only the N=256 rows and print them (for profiling that kernel)")
    ap.add_argument("--valu-rates-only", action="store_true",
                    help="run only the probe of the vector-instruction issue rates and print it")
    ap.add_argument("--small-batch-only", action="store_true",
                    help="time only the N = 2..64 rows and print them (for profiling those kernels)")
    ap.add_argument("--separate", action="store_true",
                    help="step = one tmac_mpgemv_fused launch per GEMV instead of one launch for the three")
    ap.add_argument("--two-call", action="store_true",
                    help="step = tmac_precompute_lut + tmac_mpgemm (two launches per GEMV)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(no collectives or sharding are part of the path)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2407_00088_amd as T
    import tmac_workloads as wl
    from paper_2407_00088_amd import bench_helpers as H
    from paper_2407_00088_amd.binding import tmac_tuning
    from paper_2407_00088_amd.runner import from_problem

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = "cuda"
    tuning = tmac_tuning(args.rows) if args.rows else None
    stream = torch.cuda.Stream()
    sink = torch.zeros(256, dtype=torch.uint8, device=dev)

    class Case:
        def __init__(self, p, ring_mb=None, lut_t=None, layout=None, g=4):
            self.p = p
            # layout None: register-table layout for N <= 8 (g = 4), batched layout otherwise
            self.lin = from_problem(p, lut_t=lut_t, layout=layout, g=g)
            self.bytes = algorithmic_bytes(p.M, p.K, p.bits, p.group, p.N, act_bytes=1 if p.int_path else 2)
            n_copies = max(2, ((args.ring_mb if ring_mb is None else ring_mb) << 20) // self.lin.packed_bytes + 1)
            self.ring = [self.lin.packed] + [self.lin.packed.clone() for _ in range(n_copies - 1)]
            self.A = torch.from_numpy(p.act_q if p.int_path else p.act).to(dev)
            self.s_a = torch.from_numpy(p.act_scale).to(dev) if p.int_path else None
            self.out = torch.empty((p.N, p.M), dtype=torch.float32, device=dev)
            self.i = 0
            # the launch-shape knob belongs to the register-table kernel with 16-bit tables
            self.tuning = tuning if (self.lin.layout == 2 and self.lin.lut_t != T.TMAC_LUT_I8Q) else None

        def next_packed(self):
            packed = self.ring[self.i % len(self.ring)]
            self.i += 1
            return packed

        def precompute(self):
            self.lin.precompute(self.A)

        def mpgemm(self):
            self.lin.mpgemm(self.p.N, self.out, T.TMAC_OUT_F32, act_scale=self.s_a, tuning=self.tuning,
                            packed=self.next_packed())

        def fused(self):
            self.lin.mpgemv_fused(self.A, self.p.N, self.out, T.TMAC_OUT_F32, act_scale=self.s_a,
                                  packed=self.next_packed(), tuning=self.tuning)

        def one_call(self):
            self.lin.mpgemm_fused(self.A, self.p.N, self.out, T.TMAC_OUT_F32, act_scale=self.s_a,
                                  packed=self.next_packed())

        def item(self):
            """This matrix as an item of tmac_mpgemv_fused_multi, on the ring's next copy."""
            return (self.lin.desc, self.next_packed(), self.A, self.out, self.s_a, self.lin.weight_scale)

        def stream_read(self):
            """Plain read of the same packed bytes: what a read-only kernel reaches on this ring."""
            H.stream_read(self.next_packed(), sink, 1, True)

    def multi(cases_, act=None):
        """One launch for several matrices (tmac_mpgemv_fused_multi); act = T.TMAC_ACT_F16_TQ quantises the
        tables to int8 inside the kernel (Section 3.3)."""
        T.tmac_mpgemv_fused_multi([c.item() for c in cases_], cases_[0].p.N, T.TMAC_OUT_F32, act=act,
                                  tuning=None if act is not None else tuning)

    class Replay:
        """`body` issued `reps` times per launch, either eagerly or as one captured HIP graph."""

        def __init__(self, body, reps):
            self.body, self.reps, self.graph = body, reps, None
            with torch.cuda.stream(stream):
                body()  # warm-up outside capture (first-use attribute calls, lazy module load)
            stream.synchronize()
            if not args.no_graph:
                self.graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(self.graph, stream=stream):
                    for _ in range(reps):
                        body()

        def run(self):
            if self.graph is not None:
                self.graph.replay()
            else:
                for _ in range(self.reps):
                    self.body()

    def timed(replay, launches, warm):
        """Returns microseconds per body execution."""
        with torch.cuda.stream(stream):
            for _ in range(warm):
                replay.run()
            stream.synchronize()
            for _ in range(launches):
                replay.run()  # untimed lead-in as long as the timed region: the GPU is busy while the host
                              # enqueues, and the clocks have recovered from the idle gap of the synchronize()
            t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            t0.record(stream)
            for _ in range(launches):
                replay.run()
            t1.record(stream)
            stream.synchronize()
        return t0.elapsed_time(t1) * 1e3 / (launches * replay.reps)

    last_brackets = []  # the raw event brackets of the latest steady_us call

    def steady_us(body, reps, steps):
        """Time of exactly `steps` executions of `body` in steady state, in microseconds per execution.

        A pair of HIP events around a graph replay carries a fixed cost of 25-45 us on this runtime (the
        events' own packets and the start of a graph that did not run just before), which a region of
        20 steps = 0.27 ms would show as +2 us per step.  So the region is bracketed twice, each time by
        events on the launching stream with synchronize() on both sides: once around a calibration graph of
        L executions (L = `reps`, one pass over the weight ring) and once around the timed sequence, whose
        last graph holds L + r executions; the difference of the two brackets is the time of exactly
        `steps` = q * 4 * reps + r executions with the fixed cost cancelled.  Each bracket is preceded by
        untimed replays of its own first graph (the GPU is busy while the host enqueues, the bracket
        starts with a graph that has just run, and the clocks have recovered from the idle gap of the
        synchronize()).  The pair is measured three times and the median difference is returned."""
        big = 4 * reps
        cache = {}

        def graph(n):
            if n not in cache:
                cache[n] = Replay(body, n)
            return cache[n]

        def bracket(seq):
            # untimed lead-in: about LEAD_IN_STEPS executions of the bracket's own first graph
            lead = max(2, -(-LEAD_IN_STEPS // seq[0].reps))
            with torch.cuda.stream(stream):
                for _ in range(lead):
                    seq[0].run()
                t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                t0.record(stream)
                for g in seq:
                    g.run()
                t1.record(stream)
                stream.synchronize()
            return t0.elapsed_time(t1) * 1e3

        q = (steps - 1) // big
        r = steps - q * big                      # 1 .. big
        cal_seq = [graph(reps)]
        timed_seq = [graph(big)] * q + [graph(reps + r)]
        diffs, dbg = [], []
        for _ in range(3 if steps >= 16 else 9):   # a handful of steps is within the noise of one pair
            ca = bracket(cal_seq)
            tb = bracket(timed_seq)
            diffs.append(tb - ca)
            dbg.append((round(ca, 1), round(tb, 1)))
        last_brackets[:] = [{"calibration_steps": reps, "bracket_steps": reps + steps, "calibration_us": c, "bracket_us": t}
                            for c, t in dbg]
        d = sorted(diffs)[len(diffs) // 2]
        if d <= 0:   # (cannot happen with more than a few steps) fall back to the whole bracket's average
            return dbg[-1][1] / (reps + r + q * big)
        return d / steps

    def timed_exact(body, reps, steps, warm_steps, preroll):
        """`preroll` + `warm_steps` untimed executions of `body`, then steady_us over exactly `steps`."""
        n = preroll + warm_steps
        if n > 0:
            g = Replay(body, min(n, 4 * reps))
            with torch.cuda.stream(stream):
                done = 0
                while done < n:   # whole replays: at least n executions
                    g.run()
                    done += g.reps
                stream.synchronize()
        return steady_us(body, reps, steps)

    def per_launch(body, reps, min_launches=MIN_LAUNCHES):
        """Microseconds per execution of `body` in steady state over at least `min_launches` executions: the
        same answer whatever --steps says."""
        return steady_us(body, reps, max(min_launches, reps))

    def ring_len(c):
        return len(c.ring)

    def measure_kernel(c, body=None, min_launches=MIN_LAUNCHES):
        return per_launch(body or c.mpgemm, ring_len(c), min_launches)

    def gemv_row(c, name=None, with_two_call=False):
        """One decode GEMV shape: the fused launch, the plain read of the same bytes, rates."""
        fu = measure_kernel(c, c.fused)
        ru = measure_kernel(c, c.stream_read)
        row = {"name": name or c.p.name, "M": c.p.M, "K": c.p.K, "bits": c.p.bits, "fused_us": round(fu, 3),
               "plain_read_of_same_bytes_us": round(ru, 3), "bytes": c.bytes, "GBps": round(c.bytes / fu / 1e3, 1),
               "frac_hbm_peak": round(c.bytes / fu / 1e3 / HBM_PEAK_GBPS, 4)}
        if with_two_call:
            row["mpgemm_us"] = round(measure_kernel(c), 3)
            row["precompute_us"] = round(per_launch(c.precompute, 50), 3)
        return row

    def small_batch_rows():
        """Small batches (N = 2..64) on the 4096 x 4096 W4 shape: precompute + lookup per call, in both
        packed layouts where the register-table kernel takes the N (at most 8 rows)."""
        small = []
        for N in (2, 4, 8, 16, 32, 64):
            p = wl.make_grouped(3, 60 + N, N, 4096, 4096, 4, 128, name=f"small_batch_4096x4096_w4_n{N}")
            row = {"name": p.name, "N": N, "bytes": algorithmic_bytes(p.M, p.K, p.bits, p.group, N)}
            for lay, key in ((2, "register_table"), (3, "batched")):
                if lay == 2 and N > 8:
                    continue
                c = Case(p, layout=lay)

                def both(c=c):
                    c.precompute()
                    c.mpgemm()
                us = per_launch(both, ring_len(c))
                row[key + "_call_us"] = round(us, 3)
                row[key + "_TOPS_equiv"] = round(2.0 * N * p.M * p.K / us / 1e6, 3)
                # the same rows through the one-call entry point (tables built in the lookup kernel)
                row[key + "_one_call_us"] = round(measure_kernel(c, c.one_call), 3)
                del c
                torch.cuda.empty_cache()
            small.append(row)
        return small

    def lds_lookup_ceiling():
        """Lookup rate of LDS alone (LDS probe of libtmac_bench.so): the ceiling of the batched kernels'
        lookups.  One 16-byte read of a wavefront serves 64 lanes x 8 activation rows = 512 lookups."""
        wgs, rounds = 256 * 5 * 4, 2000

        def probe():
            H.lds_lookup_probe(wgs, rounds, sink)
        us = timed(Replay(probe, 1), 5, 2)
        wave_reads = wgs * 4 * rounds * 16
        return {"workgroups": wgs, "rounds": rounds, "us": round(us, 1),
                "wave_reads_per_s": round(wave_reads / us * 1e6, -6),
                "lookups_per_s": round(wave_reads * 512 / us * 1e6, -9)}

    def valu_issue_rates():
        """Issue rate of the vector instructions the register-table lookups consist of (probe of
        libtmac_bench.so): nanoseconds per wavefront instruction and SIMD, for 1, 2 and 4 wavefronts per SIMD."""
        rows = []
        n_simd = torch.cuda.get_device_properties(0).multi_processor_count * 4
        for kind, name, per_iter in ((0, "v_and_b32", 64), (1, "v_perm_b32", 64), (2, "v_dot2c_f32_f16", 64),
                                     (3, "lookup sequence of one index dword (17 instructions)", 8 * 17)):
            row = {"instruction": name}
            for wps in (1, 2, 4):
                wgs, iters = n_simd * wps // 4, 2000

                def probe(kind=kind, wgs=wgs, iters=iters):
                    H.valu_rate_probe(kind, wgs, iters, sink)
                us = timed(Replay(probe, 1), 5, 2)
                row[f"ns_per_wave_instr_per_simd_at_{wps}_waves"] = round(us * 1e3 / (iters * per_iter * wps), 3)
            rows.append(row)
        return rows

    def prefill_rows(ceiling_lookups_per_s):
        """Prefill mpGEMM, N = 256 (batched lookup kernel): precompute + mpgemm per call.  The roofline
        of this path is the lookup rate (lookup-and-add, no dense contraction): lookups per second
        against what LDS alone delivers with the same table layout and addressing, measured in this run."""
        rows = []
        for bits in (2, 4):
            for i in range(3):
                p = wl.config5(i, bits)
                c = Case(p, ring_mb=0)

                def both(c=c):
                    c.precompute()
                    c.mpgemm()
                us = timed(Replay(both, 2), 10, 2)
                pu = timed(Replay(c.precompute, 2), 10, 2)
                flops = 2.0 * p.N * p.M * p.K
                lookup_adds = p.N * p.M * (p.K / 4) * bits
                rate = lookup_adds / us * 1e6
                rows.append({"name": p.name, "bits": bits, "N": p.N, "call_us": round(us, 2),
                             "precompute_us": round(pu, 2),
                             "TOPS_equiv": round(flops / us / 1e6, 2),
                             "lookups_per_s": round(rate, -6),
                             "roofline": {"bound": "lds lookup rate", "unit": "lookups/s",
                                          "peak": ceiling_lookups_per_s, "achieved": round(rate, -6),
                                          "frac": round(rate / ceiling_lookups_per_s, 4)}})
                del c
                torch.cuda.empty_cache()
        return rows

    def isolated_rows(cases_):
        """The paper's own protocol (Section 5.1: warm-up, then the mean of 100 runs) on ONE copy of the
        weights, an event pair around every call, launched eagerly: cache-hot and launch-dominated;
        printed next to the steady-state figures, never instead of them."""
        rows = []
        for c in cases_:
            row = {"name": c.p.name}
            for key, body in (("fused_us", c.fused), ("mpgemm_us", c.mpgemm), ("precompute_us", c.precompute)):
                ring, c.ring = c.ring, c.ring[:1]
                ts = []
                with torch.cuda.stream(stream):
                    for it in range(110):
                        t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                        t0.record(stream)
                        body()
                        t1.record(stream)
                        stream.synchronize()
                        if it >= 10:
                            ts.append(t0.elapsed_time(t1) * 1e3)
                c.ring = ring
                ts.sort()
                row[key] = {"mean": round(sum(ts) / len(ts), 2), "median": round(ts[len(ts) // 2], 2)}
            rows.append(row)
        return rows

    if args.valu_rates_only:
        print(json.dumps({"valu_issue_rates": valu_issue_rates()}))
        return

    if args.small_batch_only:
        print(json.dumps({"small_batch": small_batch_rows()}))
        return

    if args.prefill_only:
        ceil = lds_lookup_ceiling()
        print(json.dumps({"prefill_n256": prefill_rows(ceil["lookups_per_s"]), "lds_lookup_ceiling": ceil}))
        return

    # ------------------------------------------------------------------ the step ----
    cases = [Case(wl.config2(i)) for i in range(3)]
    step_bytes = sum(c.bytes for c in cases)
    mode = "two_call" if args.two_call else ("separate" if args.separate else "multi")

    def step_multi():
        multi(cases)

    def step_separate():
        for c in cases:
            c.fused()

    def step_two_call():
        for c in cases:
            c.precompute()
            c.mpgemm()

    step = {"multi": step_multi, "separate": step_separate, "two_call": step_two_call}[mode]
    reps = max(ring_len(c) for c in cases)
    steps_done = max(1, args.steps)
    step_us = timed_exact(step, reps, steps_done, max(0, args.warmup), PREROLL_STEPS)
    headline_brackets = list(last_brackets)
    ms_per_step = step_us * 1e-3
    value = step_bytes / (step_us * 1e-6) / 1e9

    detail = {}
    launches_per_step = {"multi": 1, "separate": 3, "two_call": 6}[mode]
    if mode == "two_call":
        # the step also launches the precompute kernel: the lookup kernel alone, back to back over the ring
        mp_us = [measure_kernel(c) for c in cases]
        achieved = step_bytes / (sum(mp_us) * 1e-6) / 1e9
        how = "HIP events over back-to-back launches of this kernel alone (the step also launches the precompute kernel)"
        avg_launch_us, launch_us = sum(mp_us) / 3, mp_us
    else:
        # the timed region consists of launches of the dominant kernel only
        achieved = value
        how = (f"HIP events over the timed region: {launches_per_step} launch(es) of this kernel per step, "
               f"{step_bytes // launches_per_step} algorithmic bytes per launch on average")
        avg_launch_us, launch_us = step_us / launches_per_step, None
    traffic = None
    if mode in ("multi", "separate") and not args.rows and MEASURED_TRAFFIC["sources_sha256_16"] == kernel_sources_hash():
        traffic = MEASURED_TRAFFIC[mode]

    if args.headline_only:
        # a few plain reads of the same blobs: a kernel of known size in the same trace (it calibrates
        # the byte counters of a profiler run)
        with torch.cuda.stream(stream):
            for _ in range(20):
                for c in cases:
                    c.stream_read()
        stream.synchronize()
    else:
        # the same step the other ways, each over at least MIN_LAUNCHES steps
        variants = {}
        for key, fn in (("one_launch_for_the_three_us", step_multi), ("three_fused_launches_us", step_separate),
                        ("precompute_plus_lookup_six_launches_us", step_two_call)):
            us = per_launch(fn, reps)
            variants[key] = round(us, 3)
            variants[key.replace("_us", "_frac_hbm_peak")] = round(step_bytes / us / 1e3 / HBM_PEAK_GBPS, 4)

        def step_read():
            for c in cases:
                c.stream_read()
        # the paper's table quantisation (Section 3.3, int8 tables built in the kernel): outside the
        # fp tolerance of the headline (about 4e-3 relative error), shown beside it
        us = per_launch(lambda: multi(cases, act=T.TMAC_ACT_F16_TQ), reps)
        variants["one_launch_int8_tables_quantised_in_kernel_us"] = round(us, 3)
        variants["one_launch_int8_tables_quantised_in_kernel_frac_hbm_peak"] = round(step_bytes / us / 1e3 / HBM_PEAK_GBPS, 4)
        variants["plain_read_of_the_same_bytes_three_launches_us"] = round(per_launch(step_read, reps), 3)
        variants["empty_kernel_us"] = round(per_launch(H.empty_kernel, 100), 3)
        detail["step_variants"] = variants
        detail["shapes"] = [gemv_row(c, with_two_call=True) for c in cases]
        if launch_us is None:
            launch_us = [r["fused_us"] for r in detail["shapes"]]

        # one Llama-2-7B decoder block, N = 1 (seven projections, 107.7 MB of packed weights), weights of
        # every projection from its own ring: Q,K,V in one launch, O, gate and up in one launch, down
        blk_shapes = [("q", 4096, 4096), ("k", 4096, 4096), ("v", 4096, 4096), ("o", 4096, 4096),
                      ("gate", 11008, 4096), ("up", 11008, 4096), ("down", 4096, 11008)]
        cs = {k: Case(wl.make_grouped(3, 90 + i, 1, M, K, 4, 128, name=f"block_{k}"), ring_mb=args.ring_mb // 2)
              for i, (k, M, K) in enumerate(blk_shapes)}
        nbytes = sum(c.bytes for c in cs.values())

        def block_multi():
            multi([cs["q"], cs["k"], cs["v"]])
            cs["o"].fused()
            multi([cs["gate"], cs["up"]])
            cs["down"].fused()

        def block_separate():
            for k, _, _ in blk_shapes:
                cs[k].fused()

        def block_one():
            # all seven in ONE launch: what the kernel does with 108 MB behind one start; a real block
            # cannot do this (O needs the attention output, down needs gate and up)
            multi([cs[k] for k, _, _ in blk_shapes])
        breps = max(ring_len(c) for c in cs.values())
        blk = {}
        for key, fn in (("four_launches_qkv_and_gate_up_grouped", block_multi), ("seven_launches", block_separate),
                        ("one_launch_ignoring_the_data_dependencies", block_one)):
            us = per_launch(fn, breps)
            blk[key] = {"us": round(us, 3), "bytes": nbytes, "GBps": round(nbytes / us / 1e3, 1),
                        "frac_hbm_peak": round(nbytes / us / 1e3 / HBM_PEAK_GBPS, 4)}
        del cs
        torch.cuda.empty_cache()
        detail["decoder_block_llama2_7b"] = blk
        keep = cases if args.sweep else []
        if not args.sweep:
            del cases[:]
            torch.cuda.empty_cache()

        # W1..W4 at N = 1 on two shapes (config 3 and its 11008 x 4096 sibling): time per call, rate,
        # and the fit t(b) = t0 + c b
        sweep = {}
        for M, K in ((4096, 4096), (11008, 4096)):
            rows = []
            for b in (1, 2, 3, 4):
                p = wl.config3(b) if (M, K) == (4096, 4096) else wl.make_grouped(3, 10 + b, 1, M, K, b, 128)
                c = Case(p)
                rows.append(gemv_row(c, with_two_call=(M == 4096)))
                del c
                torch.cuda.empty_cache()
            sweep[f"{M}x{K}"] = {"rows": rows,
                                 "fit_fused": linear_fit([r["bits"] for r in rows], [r["fused_us"] for r in rows]),
                                 "fit_plain_read": linear_fit([r["bits"] for r in rows],
                                                              [r["plain_read_of_same_bytes_us"] for r in rows])}
        # the whole step (the three config-2 shapes in one launch) at 1..4 bit: with three matrices behind
        # one launch the fixed cost of a launch weighs less and the line through the four points shows
        # how time follows the bit-width
        srows = []
        for b in (1, 2, 3, 4):
            cs3 = [Case(wl.make_grouped(3, 20 + 4 * i + b, 1, M, K, b, 128, name=f"step_{M}x{K}_w{b}"), ring_mb=args.ring_mb // 2)
                   for i, (M, K) in enumerate(((4096, 4096), (11008, 4096), (4096, 11008)))]
            nb = sum(c.bytes for c in cs3)
            r3 = max(ring_len(c) for c in cs3)
            us = per_launch(lambda: multi(cs3), r3)

            def read3():
                for c in cs3:
                    c.stream_read()
            ru = per_launch(read3, r3)
            srows.append({"bits": b, "one_launch_us": round(us, 3), "bytes": nb, "GBps": round(nb / us / 1e3, 1),
                          "frac_hbm_peak": round(nb / us / 1e3 / HBM_PEAK_GBPS, 4),
                          "plain_read_three_launches_us": round(ru, 3)})
            del cs3
            torch.cuda.empty_cache()
        sweep["three_shapes_one_launch"] = {"rows": srows,
                                            "fit_one_launch": linear_fit([r["bits"] for r in srows],
                                                                         [r["one_launch_us"] for r in srows])}
        detail["bit_sweep_n1"] = sweep

        # BitNet-b1.58-3B-shaped ternary GEMVs (config 4): int8 activations, exact integers
        bn = [Case(wl.config4(i)) for i in range(3)]
        bn_rows = [gemv_row(c) for c in bn]
        bn_bytes = sum(c.bytes for c in bn)
        us = per_launch(lambda: multi(bn), max(ring_len(c) for c in bn))
        detail["bitnet_ternary_n1"] = {"rows": bn_rows,
                                       "one_launch_for_the_three": {"us": round(us, 3), "bytes": bn_bytes,
                                                                    "GBps": round(bn_bytes / us / 1e3, 1),
                                                                    "frac_hbm_peak": round(bn_bytes / us / 1e3 / HBM_PEAK_GBPS, 4)}}
        del bn
        torch.cuda.empty_cache()

        # N = 256 (config 5)
        ceil = lds_lookup_ceiling()
        detail["lds_lookup_ceiling"] = ceil
        detail["prefill_n256"] = prefill_rows(ceil["lookups_per_s"])
        cases = keep

    if args.sweep:
        detail["valu_issue_rates"] = valu_issue_rates()
        detail["isolated_one_copy_eager"] = isolated_rows(cases)
        del cases[:]
        torch.cuda.empty_cache()
        # int8 table quantisation (Section 3.3): lookup kernel with int8 tables, two-call path
        tq = []
        for i in range(3):
            c = Case(wl.config2(i), lut_t=T.TMAC_LUT_I8Q)
            us = measure_kernel(c)
            pu = per_launch(c.precompute, 50)
            tq.append({"name": c.p.name + "_int8_tables", "mpgemm_us": round(us, 3), "precompute_us": round(pu, 3),
                       "bytes": c.bytes, "GBps": round(c.bytes / us / 1e3, 1),
                       "frac_hbm_peak": round(c.bytes / us / 1e3 / HBM_PEAK_GBPS, 4)})
            del c
            torch.cuda.empty_cache()
        detail["table_quantisation"] = tq
        # one bigger matrix per call: stacked projections (Q,K,V and gate,up stacked along M by the caller)
        # and Llama-2-70B-shaped matrices (34-125 MB per call)
        big = []
        for M, K in ((12288, 4096), (22016, 4096), (8192, 8192), (28672, 8192), (8192, 28672)):
            c = Case(wl.make_grouped(3, 40 + M // 1000 + K // 4000, 1, M, K, 4, 128, name=f"{M}x{K}_w4_n1"))
            big.append(gemv_row(c))
            del c
            torch.cuda.empty_cache()
        detail["larger_matrices"] = big
        detail["small_batch"] = small_batch_rows()
        # LUT group size g = 2, 4, 8 in the batched kernel (Section 4 on the choice of g): fewer,
        # larger tables against more look-ups; precompute + lookup per call
        gs = []
        for p in (wl.make_grouped(3, 76, 16, 4096, 4096, 4, 128, name="g_sweep_4096x4096_w4_n16"),
                  wl.config5(0, 4)):
            for g in (2, 4, 8):
                c = Case(p, layout=3, g=g, ring_mb=0 if p.N > 16 else None)

                def both(c=c):
                    c.precompute()
                    c.mpgemm()
                us = per_launch(both, ring_len(c)) if p.N <= 16 else timed(Replay(both, 2), 10, 2)
                pu = timed(Replay(c.precompute, 20), 5, 1)
                gs.append({"name": p.name, "N": p.N, "g": g, "call_us": round(us, 2), "precompute_us": round(pu, 2),
                           "lut_bytes": int(c.lin.lut.numel()),
                           "TOPS_equiv": round(2.0 * p.N * p.M * p.K / us / 1e6, 2)})
                del c
                torch.cuda.empty_cache()
        detail["g_sweep"] = gs

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import tmac_oracle as orc
        n_threads = len(os.sched_getaffinity(0))
        ps = [wl.config2(i) for i in range(3)]
        pbytes = [algorithmic_bytes(p.M, p.K, p.bits, p.group) for p in ps]
        done_bytes, t_used, calls = 0, 0.0, 0
        orc.mpgemm_definition(ps[0].act, ps[0].q, ps[0].scales, ps[0].zeros, ps[0].group)  # warm-up
        while t_used < args.cpu_seconds:
            p = ps[calls % 3]
            t0 = time.perf_counter()
            orc.mpgemm_definition(p.act, p.q, p.scales, p.zeros, p.group)
            t_used += time.perf_counter() - t0
            done_bytes += pbytes[calls % 3]
            calls += 1
        # numpy's element-wise de-quantisation dominates the oracle and runs on one thread whatever
        # the BLAS pool of the matvec is set to: one core is what it uses
        cpu = {"value": round(done_bytes / t_used / 1e9, 4), "unit": "GB/s", "cores": 1,
               "kind": "oracle", "host_threads_available": n_threads,
               "sample": f"{calls} oracle calls (dequantise to fp64 + fp64 matvec) cycling the three "
                         f"config-2 shapes, {t_used:.1f} s"}

    how_step = {"multi": "ONE launch of tmac_mpgemv_fused_multi for the three shapes (table precompute + lookup in the kernel)",
                "separate": "one fused launch (table precompute + lookup) per shape",
                "two_call": "precompute_lut + mpgemm per shape"}[mode]
    line = {
        "metric": "mpgemv_w4a16_llama2_7b_decode_algorithmic_GBps",
        "value": round(value, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": steps_done,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 6),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16",
        "data": "synthetic",
        "config": {"workload": "configs[1]: Llama-2-7B-shaped W4A16 decode GEMV, N=1, "
                               "(M,K) in {(4096,4096),(11008,4096),(4096,11008)}, group 128; step = "
                               + how_step + f", weights cycled through a {args.ring_mb} MiB ring per shape",
                   "launch": "eager" if args.no_graph else "hip graph replay",
                   "untimed_preroll_steps": PREROLL_STEPS,
                   "timing": "HIP events around a graph of L + K steps minus the same around a graph of L steps "
                             "(L = one pass over the weight ring): the fixed cost of an event pair around a graph "
                             "replay cancels; each bracket follows about 600 untimed steps of its first graph; median of three pairs",
                   "event_brackets": headline_brackets,
                   "frac_hbm_peak_whole_step": round(value / HBM_PEAK_GBPS, 4)},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4),
                     "traffic": traffic,
                     "traffic_unit": "bytes per step, rocprofv3 FETCH_SIZE + WRITE_SIZE, calibrated; null when the "
                                     "kernel sources changed since the counters were read",
                     "algorithmic_bytes": step_bytes,
                     "kernel": "mpgemv_perm_kernel<f16 tables, 4 bit, chunk scales, "
                               + ("fused table build>" if mode != "two_call" else "tables from the LUT buffer>"),
                     "measured": how,
                     "avg_launch_us": round(avg_launch_us, 3),
                     "launch_us_one_shape_at_a_time": None if launch_us is None else [round(u, 3) for u in launch_us]},
        "cpu_baseline": cpu,
        "detail": detail,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
