#!/usr/bin/env python3
"""Benchmark of the LUT mpGEMV hot path on one MI355X.

A step = one pass of the whole hot path (table precompute, lookup, bit-plane accumulate, scale
and zero, reduce, store) over the three Llama-2-7B-shaped W4A16 decode GEMVs (N=1; M x K =
4096x4096, 11008x4096, 4096x11008; group 128), inputs resident in HBM.  By default every GEMV
is ONE launch of tmac_mpgemv_fused (tables built inside the lookup kernel); --two-call times
tmac_precompute_lut + tmac_mpgemm instead.  Every shape cycles through a ring of distinct
packed weight copies larger than twice the 256 MB Infinity Cache, so weights come from HBM.

Launches are replayed from HIP graphs (captured once, outside the timed region) so that the
host-side cost of issuing ~3 us kernels from Python does not hide the GPU time; the timed
region is bracketed by HIP events on the launching stream and by synchronize().

Prints ONE JSON line: whole-step throughput (algorithmic GB/s), the roofline of the dominant
kernel (the lookup kernel: back-to-back launches over the weight ring, HIP events) and the CPU
oracle timed on the host cores as a reported baseline.
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

HBM_PEAK_GBPS = 8000.0
ALU_PEAK_LANE_OPS = 256 * 64 * 2.4e9   # one vector instruction per lane and cycle on every CU
ALU_OPS_PER_LOOKUP_ADD = 83.0 / 128.0  # batched kernel, sixteen activation rows per workgroup (N >= 128)
RING_MB = 576  # > 2 x 256 MB Infinity Cache

# HBM bytes of the three launches of one step (default configuration: fused kernel, 8 rows per
# workgroup), from two rocprofv3 --pmc passes (FETCH_SIZE, then WRITE_SIZE), each dispatch's
# counter scaled by what the same counter reads for the plain read kernel on a blob of the same
# size (2093 / 2051 bytes per count); summary under profiles/.
MEASURED_TRAFFIC_BYTES = {"fetch": [9.26e6, 24.14e6, 24.28e6], "write": [16384, 44032, 16384]}


def algorithmic_bytes(M, K, bits, group, N=1, act_bytes=2, out_bytes=4):
    """Bytes the method must move per call: packed indices + scales and zeros + activations + output."""
    w = M * K * bits // 8
    sz = 0 if group == 0 else M * (K // group) * 4
    return w + sz + N * K * act_bytes + N * M * out_bytes


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--ring-mb", type=int, default=RING_MB)
    ap.add_argument("--rows", type=int, default=0, help="tmac_tuning.rows_per_group override (8 or 16)")
    ap.add_argument("--sweep", action="store_true", help="also time the W1..W4 and BitNet shapes")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly from Python instead of graph replay")
    ap.add_argument("--prefill-only", action="store_true",
                    help="time only the N=256 rows of the sweep and print them (for profiling that kernel)")
    ap.add_argument("--small-batch-only", action="store_true",
                    help="time only the N = 2..64 rows of the sweep and print them (for profiling those kernels)")
    ap.add_argument("--two-call", action="store_true",
                    help="step = tmac_precompute_lut + tmac_mpgemm (two launches per GEMV) instead of the fused call")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(no collectives or sharding are part of the path)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2407_00088_amd as T
    import tmac_workloads as wl
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

        def precompute(self):
            self.lin.precompute(self.A)

        def mpgemm(self):
            packed = self.ring[self.i % len(self.ring)]
            self.i += 1
            self.lin.mpgemm(self.p.N, self.out, T.TMAC_OUT_F32, act_scale=self.s_a, tuning=self.tuning, packed=packed)

        def fused(self):
            packed = self.ring[self.i % len(self.ring)]
            self.i += 1
            self.lin.mpgemv_fused(self.A, self.p.N, self.out, T.TMAC_OUT_F32, act_scale=self.s_a, packed=packed,
                                  tuning=self.tuning)

        def one_call(self):
            packed = self.ring[self.i % len(self.ring)]
            self.i += 1
            self.lin.mpgemm_fused(self.A, self.p.N, self.out, T.TMAC_OUT_F32, act_scale=self.s_a, packed=packed)

        def stream_read(self):
            """Plain read of the same packed bytes: what a read-only kernel reaches on this ring."""
            packed = self.ring[self.i % len(self.ring)]
            self.i += 1
            T.tmac_stream_read(packed, sink, 1, True)

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
            t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            t0.record(stream)
            for _ in range(launches):
                replay.run()
            t1.record(stream)
            stream.synchronize()
        return t0.elapsed_time(t1) * 1e3 / (launches * replay.reps)

    def timed_exact(body, reps, steps, warm_steps):
        """Exactly `warm_steps` untimed and `steps` timed executions of `body`: whole replays of `reps`
        executions plus one shorter replay for the remainder.  Returns microseconds per execution."""
        full = Replay(body, reps)
        tails = {}

        def plan(n):
            seq = [full] * (n // reps)
            if n % reps:
                if n % reps not in tails:
                    tails[n % reps] = Replay(body, n % reps)
                seq.append(tails[n % reps])
            return seq

        warm_seq, timed_seq = plan(warm_steps), plan(steps)
        with torch.cuda.stream(stream):
            for r in warm_seq:
                r.run()
            stream.synchronize()
            t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            t0.record(stream)
            for r in timed_seq:
                r.run()
            t1.record(stream)
            stream.synchronize()
        return t0.elapsed_time(t1) * 1e3 / steps

    def ring_len(c):
        return len(c.ring)

    def measure_kernel(c, total, body=None):
        reps = ring_len(c)
        launches = max(1, total // reps)
        return timed(Replay(body or c.mpgemm, reps), launches, max(1, launches // 10))

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
                us = timed(Replay(both, ring_len(c)), max(1, args.steps // ring_len(c)), 2)
                row[key + "_call_us"] = round(us, 3)
                row[key + "_TOPS_equiv"] = round(2.0 * N * p.M * p.K / us / 1e6, 3)
                # the same rows through the one-call entry point (tables built in the lookup kernel)
                fu = measure_kernel(c, args.steps, c.one_call)
                row[key + "_one_call_us"] = round(fu, 3)
                del c
                torch.cuda.empty_cache()
            small.append(row)
        return small

    def prefill_rows():
        """Prefill mpGEMM, N = 256 (batched lookup kernel): precompute + mpgemm per call."""
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
                rows.append({"name": p.name, "bits": bits, "N": p.N, "call_us": round(us, 2),
                             "precompute_us": round(pu, 2),
                             "TOPS_equiv": round(flops / us / 1e6, 2),
                             "lookups_per_s": round(lookup_adds / us * 1e6, -6),
                             # plain-ALU roofline of the batched kernel: 83 vector instructions per 128
                             # lookup-adds of a lane is what the method needs in this kernel (3 offset
                             # instructions, 8 address permutes, 56 packed adds, 16 widening multiply-adds
                             # per chunk and plane of sixteen activation rows); peak = 256 CUs x 64 lanes
                             # x 2.4 GHz
                             "roofline": {"bound": "alu", "unit": "lane-op/s", "peak": ALU_PEAK_LANE_OPS,
                                          "achieved": round(lookup_adds * ALU_OPS_PER_LOOKUP_ADD / (us - pu) * 1e6, -9),
                                          "frac": round(lookup_adds * ALU_OPS_PER_LOOKUP_ADD / (us - pu) * 1e6
                                                        / ALU_PEAK_LANE_OPS, 4)}})
                del c
                torch.cuda.empty_cache()
        return rows

    def lds_lookup_ceiling():
        """Lookup rate of LDS alone (tmac_lds_lookup_probe): the ceiling of the batched kernels' lookups.
        One 16-byte read of a wavefront serves 64 lanes x 8 activation rows = 512 lookups."""
        wgs, rounds = 256 * 5 * 4, 2000

        def probe():
            T.tmac_lds_lookup_probe(wgs, rounds, sink)
        us = timed(Replay(probe, 1), 5, 2)
        wave_reads = wgs * 4 * rounds * 16
        return {"workgroups": wgs, "rounds": rounds, "us": round(us, 1),
                "wave_reads_per_s": round(wave_reads / us * 1e6, -6),
                "bytes_per_clk_per_cu_at_2.4GHz": round(wave_reads * 1024 / us * 1e6 / 256 / 2.4e9, 1),
                "lookups_per_s": round(wave_reads * 512 / us * 1e6, -9)}

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

    if args.small_batch_only:
        print(json.dumps({"small_batch": small_batch_rows()}))
        return

    if args.prefill_only:
        print(json.dumps({"prefill_n256": prefill_rows(), "lds_lookup_ceiling": lds_lookup_ceiling()}))
        return

    cases = [Case(wl.config2(i)) for i in range(3)]
    step_bytes = sum(c.bytes for c in cases)

    fused = not args.two_call

    def step():
        for c in cases:
            if fused:
                c.fused()
            else:
                c.precompute()
                c.mpgemm()

    reps = max(ring_len(c) for c in cases)
    step_us = timed_exact(step, reps, max(1, args.steps), max(0, args.warmup))
    steps_done = max(1, args.steps)
    ms_per_step = step_us * 1e-3
    value = step_bytes / (step_us * 1e-6) / 1e9

    # dominant kernel: the lookup kernel alone (the fused one when the step uses it), back-to-back
    # over the weight ring
    mp_us = [measure_kernel(c, args.steps) for c in cases]
    fu_us = [measure_kernel(c, args.steps, c.fused) for c in cases]
    per_us = fu_us if fused else mp_us
    if fused:
        # the timed region consists of launches of the dominant kernel only (one per shape): its average
        # launch duration over that region is step_us / 3, for step_bytes / 3 bytes per launch
        achieved, how = value, "HIP events over the timed region: three launches of this kernel per step"
    else:
        achieved = sum(c.bytes for c in cases) / (sum(per_us) * 1e-6) / 1e9
        how = "HIP events over back-to-back launches of this kernel alone (the step also launches the precompute kernel)"
    pre_us = [timed(Replay(c.precompute, 50), max(1, args.steps // 50), 2) for c in cases]
    read_us = [measure_kernel(c, args.steps, c.stream_read) for c in cases]
    detail = {"shapes": []}
    for c, us, fu, pu, ru in zip(cases, mp_us, fu_us, pre_us, read_us):
        dom = fu if fused else us
        detail["shapes"].append({"M": c.p.M, "K": c.p.K, "bits": c.p.bits, "mpgemm_us": round(us, 3),
                                 "fused_us": None if fu is None else round(fu, 3),
                                 "precompute_us": round(pu, 3), "bytes": c.bytes,
                                 "GBps": round(c.bytes / dom / 1e3, 1),
                                 "frac_hbm_peak": round(c.bytes / dom / 1e3 / HBM_PEAK_GBPS, 4),
                                 "plain_read_of_same_bytes_us": round(ru, 3)})

    if args.sweep:
        detail["isolated_one_copy_eager"] = isolated_rows(cases)
        sweep = []
        del cases[1:]
        torch.cuda.empty_cache()
        extra = [wl.config3(b) for b in (1, 2, 3, 4)] + [wl.config4(i) for i in range(3)]
        for p in extra:
            c = Case(p)
            us = measure_kernel(c, args.steps)
            fu = measure_kernel(c, args.steps, c.fused)
            pu = timed(Replay(c.precompute, 50), max(1, args.steps // 50), 2)
            ru = measure_kernel(c, args.steps, c.stream_read)
            sweep.append({"name": p.name, "bits": p.bits, "mpgemm_us": round(us, 3),
                          "fused_us": None if fu is None else round(fu, 3), "precompute_us": round(pu, 3),
                          "plain_read_of_same_bytes_us": round(ru, 3),
                          "bytes": c.bytes, "GBps": round(c.bytes / us / 1e3, 1),
                          "frac_hbm_peak": round(c.bytes / us / 1e3 / HBM_PEAK_GBPS, 4)})
            del c
            torch.cuda.empty_cache()
        detail["sweep"] = sweep
        # int8 table quantisation (Section 3.3): lookup kernel with int8 tables, two-call path
        tq = []
        for i in range(3):
            c = Case(wl.config2(i), lut_t=T.TMAC_LUT_I8Q)
            us = measure_kernel(c, args.steps)
            pu = timed(Replay(c.precompute, 50), max(1, args.steps // 50), 2)
            tq.append({"name": c.p.name + "_int8_tables", "mpgemm_us": round(us, 3), "precompute_us": round(pu, 3),
                       "bytes": c.bytes, "GBps": round(c.bytes / us / 1e3, 1),
                       "frac_hbm_peak": round(c.bytes / us / 1e3 / HBM_PEAK_GBPS, 4)})
            del c
            torch.cuda.empty_cache()
        detail["table_quantisation"] = tq
        # stacked projections in one call (Q,K,V and gate,up of Llama-2-7B stacked along M): the
        # fraction of the roofline the same kernel reaches once a call moves more bytes
        stacked = []
        for M, K in ((12288, 4096), (22016, 4096)):
            c = Case(wl.make_grouped(3, 50 + M // 1000, 1, M, K, 4, 128, name=f"stacked_{M}x{K}_w4_n1"))
            fu = measure_kernel(c, args.steps, c.fused)
            ru = measure_kernel(c, args.steps, c.stream_read)
            stacked.append({"name": c.p.name, "fused_us": round(fu, 3), "plain_read_of_same_bytes_us": round(ru, 3),
                            "bytes": c.bytes, "GBps": round(c.bytes / fu / 1e3, 1),
                            "frac_hbm_peak": round(c.bytes / fu / 1e3 / HBM_PEAK_GBPS, 4)})
            del c
            torch.cuda.empty_cache()
        detail["stacked_projections"] = stacked
        # the same kernel on Llama-2-70B-shaped matrices (34-125 MB per call): how the fraction of the
        # roofline grows once the fixed cost of a launch is spread over more bytes
        larger = []
        for M, K in ((8192, 8192), (28672, 8192), (8192, 28672)):
            c = Case(wl.make_grouped(3, 40 + M // 1000 + K // 4000, 1, M, K, 4, 128, name=f"llama2_70b_{M}x{K}_w4_n1"))
            fu = measure_kernel(c, max(200, args.steps // 4), c.fused)
            ru = measure_kernel(c, max(200, args.steps // 4), c.stream_read)
            larger.append({"name": c.p.name, "fused_us": round(fu, 3), "plain_read_of_same_bytes_us": round(ru, 3),
                           "bytes": c.bytes, "GBps": round(c.bytes / fu / 1e3, 1),
                           "frac_hbm_peak": round(c.bytes / fu / 1e3 / HBM_PEAK_GBPS, 4)})
            del c
            torch.cuda.empty_cache()
        detail["larger_matrices"] = larger
        # one Llama-2-7B decoder block, N = 1: its seven projections as seven fused launches, and with
        # Q,K,V and gate,up stacked along M (four launches); weights of every launch from its own ring
        blk = {}
        shapes = {"qkv": (12288, 4096), "o": (4096, 4096), "gate_up": (22016, 4096), "down": (4096, 11008),
                  "gate": (11008, 4096)}
        cs = {k: Case(wl.make_grouped(3, 90 + i, 1, M, K, 4, 128, name=f"block_{k}"), ring_mb=args.ring_mb // 2)
              for i, (k, (M, K)) in enumerate(shapes.items())}
        for key, seq in (("stacked_4_launches", ["qkv", "o", "gate_up", "down"]),
                         ("separate_7_launches", ["o", "o", "o", "o", "gate", "gate", "down"])):
            def block_step(seq=seq):
                for k in seq:
                    cs[k].fused()
            reps = max(ring_len(cs[k]) for k in seq)
            us = timed(Replay(block_step, reps), max(1, args.steps // reps), 2)
            nbytes = sum(cs[k].bytes for k in seq)
            blk[key] = {"us": round(us, 3), "bytes": nbytes, "GBps": round(nbytes / us / 1e3, 1),
                        "frac_hbm_peak": round(nbytes / us / 1e3 / HBM_PEAK_GBPS, 4)}
        del cs
        torch.cuda.empty_cache()
        detail["decoder_block_llama2_7b"] = blk
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
                reps = ring_len(c) if p.N <= 16 else 2
                us = timed(Replay(both, reps), max(2, args.steps // (4 * reps)) if p.N <= 16 else 10, 2)
                pu = timed(Replay(c.precompute, 20), 5, 1)
                gs.append({"name": p.name, "N": p.N, "g": g, "call_us": round(us, 2), "precompute_us": round(pu, 2),
                           "lut_bytes": int(c.lin.lut.numel()),
                           "TOPS_equiv": round(2.0 * p.N * p.M * p.K / us / 1e6, 2)})
                del c
                torch.cuda.empty_cache()
        detail["g_sweep"] = gs
        detail["prefill_n256"] = prefill_rows()
        detail["lds_lookup_ceiling"] = lds_lookup_ceiling()
        xs = np.array([s["bits"] for s in sweep[:4]], dtype=np.float64)
        ys = np.array([s["mpgemm_us"] for s in sweep[:4]], dtype=np.float64)
        cfit, t0fit = np.polyfit(xs, ys, 1)
        ss_res = float(((ys - (cfit * xs + t0fit)) ** 2).sum())
        ss_tot = float(((ys - ys.mean()) ** 2).sum())
        detail["bit_linearity"] = {"us_per_bit": round(float(cfit), 4), "t0_us": round(float(t0fit), 4),
                                   "r2": round(1 - ss_res / ss_tot, 5) if ss_tot > 0 else None}

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
        # per shape: median of five oracle calls with the BLAS pool at one thread and at all threads
        def oracle_medians():
            out = []
            for p in ps:
                ts = []
                for _ in range(5):
                    t0 = time.perf_counter()
                    orc.mpgemm_definition(p.act, p.q, p.scales, p.zeros, p.group)
                    ts.append(time.perf_counter() - t0)
                out.append(round(sorted(ts)[2] * 1e6, 1))
            return out
        used, note = n_threads, ""
        try:
            from threadpoolctl import threadpool_limits
            with threadpool_limits(limits=1):
                one = oracle_medians()
            many = oracle_medians()
            detail["cpu_oracle_us_per_call"] = {"shapes": [p.name for p in ps], "threads_1": one,
                                                f"threads_{n_threads}": many}
            if sum(one) < 1.15 * sum(many):
                # numpy's element-wise de-quantisation dominates and runs on one thread: the BLAS pool
                # of the matvec makes no difference to the time
                used, note = 1, f"; same time with the BLAS pool at 1 and at {n_threads} threads"
        except ImportError:
            pass
        cpu = {"value": round(done_bytes / t_used / 1e9, 4), "unit": "GB/s", "cores": used,
               "kind": "oracle",
               "sample": f"{calls} oracle calls (dequantise to fp64 + fp64 matvec) cycling the three "
                         f"config-2 shapes, {t_used:.1f} s{note}"}

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
                               + ("one fused launch (table precompute + lookup) per shape"
                                  if fused else "precompute_lut + mpgemm per shape")
                               + f" for the three shapes, weights cycled through a {args.ring_mb} MiB ring per shape",
                   "launch": "eager" if args.no_graph else "hip graph replay",
                   "frac_hbm_peak_whole_step": round(value / HBM_PEAK_GBPS, 4)},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4),
                     "traffic": (sum(MEASURED_TRAFFIC_BYTES["fetch"]) + sum(MEASURED_TRAFFIC_BYTES["write"])
                                 if (fused and not args.rows) else None),
                     "traffic_unit": "bytes per step (three launches), rocprofv3 FETCH_SIZE + WRITE_SIZE, calibrated",
                     "algorithmic_bytes": step_bytes,
                     "kernel": ("mpgemv_perm_kernel<f16 tables, 4 bit, chunk scales, 8 rows, "
                                + ("fused table build>" if fused else "tables from the LUT buffer>")),
                     "measured": how,
                     "avg_launch_us": round(step_us / 3, 3) if fused else round(sum(per_us) / 3, 3),
                     "launch_us": [round(u, 3) for u in per_us]},
        "cpu_baseline": cpu,
        "detail": detail,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
