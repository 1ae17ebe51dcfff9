"""Benchmark of the LeanAttention decode path on one MI355X.

One step = one call of ``lean_attn_decode`` (the whole hot path: host schedule,
one persistent kernel doing K/V streaming, online softmax, partial exchange
and normalisation) over one seeded synthetic batch whose KV cache already
lives in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 0..8] [--tile-sweep]

Without ``--workload`` all five named configurations are measured one after the
other (generate, time, free).  The top level of the JSON line is the largest of
them, configuration 4 (MHA, batch 16, 32 heads, head dim 128, ragged contexts,
21 GB of KV cache); ``per_config`` holds all five and ``context_sweep`` the
contexts 4k .. 256k at batch 1 and 4.  ``--workload N`` measures only that one
(this is what the committed rocprofv3 summaries under ``profiles/`` run).
Successive steps rotate over distinct copies of the cache so that no step finds
its K/V in the 256 MB last-level cache.

Timing of a configuration: an untimed clock ramp (40 ms of the same launches:
after an idle gap the first launches run 5-10 % slower until the clocks are back
up), W warm-up steps, then exactly K steps enqueued back
to back between two synchronisations (``ms_per_step``, ``value``), with one HIP
event pair around them on the launch stream (``roofline.achieved`` = algorithmic
bytes / average launch duration).  A separate pass times K single launches, each
between its own event pair (``latency_us``).
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

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E peak
LLC_BYTES = 256 << 20           # Infinity Cache
RAMP_MS = 40.0                  # untimed sustained load before a timed region (clock ramp after idle)
HEADLINE = 4                    # the largest single-GPU configuration of the five


def _traffic_from_profiles(workload_name: str):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary of this workload, if there is one.

    Returns (bytes or None, path relative to the repository or None): the figure is read from the
    committed file, it is not measured by this run."""
    rel = os.path.join("profiles", f"hbm_traffic_{workload_name}.txt")
    path = os.path.join(ROOT, rel)
    if not os.path.exists(path):
        return None, None
    vals = {}
    for line in open(path):
        if ":" in line and not line.startswith("#"):
            k, v = line.split(":", 1)
            vals[k.strip()] = v.strip().split()[0] if v.strip() else ""
    try:
        return float(vals["hbm_bytes_per_launch"]), rel
    except (KeyError, ValueError):
        return None, None


def _pct(sorted_vals, q):
    return sorted_vals[min(len(sorted_vals) - 1, int(q * len(sorted_vals)))]


class Bench:
    def __init__(self, args):
        import torch

        import paper_2405_10480_amd as la
        import workloads

        self.torch, self.la, self.workloads, self.args = torch, la, workloads, args
        self.dev = torch.device("cuda:0")
        self.ramp_ms = float(args.ramp_ms)

    # ---- helpers ------------------------------------------------------------------------------
    def event_pair(self):
        t = self.torch
        return t.cuda.Event(enable_timing=True), t.cuda.Event(enable_timing=True)

    def back_to_back_ms(self, calls, reps, rounds=1):
        """Mean ms per call of `reps` calls enqueued back to back under one event pair (median of rounds)."""
        t = self.torch
        got = []
        for _ in range(rounds):
            a, b = self.event_pair()
            a.record()
            for i in range(reps):
                calls[i % len(calls)]()
            b.record()
            t.cuda.synchronize()
            got.append(a.elapsed_time(b) / reps)
        return sorted(got)[len(got) // 2]

    def ramp(self, calls, ms: float = None):
        """Keep the GPU busy with `calls` for `ms` milliseconds, untimed.  After an idle gap (input
        generation, a host-side pause) the first launches run 5-10 % slower until the clocks are back up
        (measured: about 15 ms of sustained load); every timed region starts after such a ramp so that it
        measures the steady state a decode loop runs in."""
        t = self.torch
        ms = self.ramp_ms if ms is None else ms * self.ramp_ms / RAMP_MS
        t0 = time.perf_counter()
        i = 0
        while (time.perf_counter() - t0) * 1e3 < ms:
            for _ in range(16):
                calls[i % len(calls)]()
                i += 1
            t.cuda.synchronize()
        return i

    def settle(self, quiet_s: float = 3.0, limit_s: float = 15.0):
        """Wait until the device streams at its steady rate: memory that an earlier process returned to
        the driver is wiped in the background (about 35 ms per GiB, so seconds after a large process) and
        slows every kernel by about 9 % meanwhile -- at a rate that is steady in itself.  Reads 1 GiB
        with the library's probe in windows of about 30 ms and returns once three windows in a row agree
        within 1.5 % and either the rate has stepped up by more than 4 % since the start (the wipe ended)
        or `quiet_s` seconds have passed without such a step (there was none; covers about 80 GiB).
        Returns (milliseconds waited, GB/s of the last window, GB/s of the first)."""
        t, la = self.torch, self.la
        buf = t.empty(1 << 30, dtype=t.uint8, device=self.dev)
        buf.fill_(1)
        sink = t.zeros(64, dtype=t.int32, device=self.dev)
        t0 = time.perf_counter()
        rates = []
        while time.perf_counter() - t0 < limit_s:
            a, b = self.event_pair()
            a.record()
            for _ in range(200):
                la.lean_attn_read_probe(buf, sink, 256, 2)
            b.record()
            t.cuda.synchronize()
            rates.append(200 * buf.numel() / (a.elapsed_time(b) * 1e-3) / 1e9)
            steady = len(rates) >= 4 and max(rates[-3:]) <= 1.015 * min(rates[-3:])
            stepped_up = len(rates) >= 4 and min(rates[-3:]) > 1.04 * min(rates[1:-2])   # rates[0]: clock ramp
            if steady and (stepped_up or time.perf_counter() - t0 >= quiet_s):
                break
        return round((time.perf_counter() - t0) * 1e3, 1), round(rates[-1], 1), round(rates[min(1, len(rates) - 1)], 1)

    def copies_for(self, one_copy: int) -> int:
        # Cache copies to rotate over: enough that a copy is evicted from the last-level cache before
        # it is read again (at least 2x its capacity between reuses), and at least four while they fit
        # in 16 GiB: the streaming rate depends by a few percent on where the driver happens to place
        # the K and V buffers relative to each other, and a mean over four placements is steadier.
        copies = max(4 if 4 * one_copy <= (16 << 30) else 2, -(-2 * LLC_BYTES // one_copy) + 1)
        if one_copy * copies > 64 << 30:
            copies = 2
        return min(copies, 64)

    # ---- one named configuration ------------------------------------------------------------------
    def measure(self, idx: int, *, full: bool):
        """Time one named workload.  `full`: also graph replay, warm cache and the CPU baseline."""
        t, la, workloads, args = self.torch, self.la, self.workloads, self.args
        w = workloads.named(idx)
        code = la.F16 if w.dtype == "f16" else la.BF16
        one_copy = w.kv_bytes
        copies = self.copies_for(one_copy)
        inp = workloads.generate(w, device=self.dev)
        ks, vs = [inp.k], [inp.v]
        for _ in range(copies - 1):
            ks.append(inp.k.clone())
            vs.append(inp.v.clone())
        problem = la.Problem(B=w.B, N_q=w.N_q, Hq=w.Hq, Hkv=w.Hkv, D=w.D, dtype=code, out_dtype=la.OUT_F32,
                             kv_layout=w.kv_layout, causal=int(w.causal), scale=w.scale, kv_seq_stride=w.n_stride)
        ws = t.empty(la.lean_attn_problem_workspace_size(problem), dtype=t.uint8, device=self.dev)
        la.lean_attn_workspace_init(ws)
        out = t.empty(w.B, w.N_q, w.Hq, w.D, dtype=t.float32, device=self.dev)
        tuning = la.Tuning(grid=args.grid, ctas_per_cu=args.ctas_per_cu, tile_shape=args.tile_shape)
        plan = la.lean_attn_problem_schedule(problem, list(w.seqlens), tuning)

        def prepared(j: int, tn):
            # One step = one call through the C ABI.  The binding's per-call argument checks are done
            # once per cache copy (a serving loop launches on the same buffers again and again): for
            # the smallest workload they would otherwise cost more host time than the launch itself.
            if w.N_q == 1:  # the decode entry point (the same kernels as the general one)
                return la.lean_attn_decode(inp.q, ks[j], vs[j], inp.seqlens, out.view(w.B, w.Hq, w.D), ws, Hkv=w.Hkv,
                                           kv_layout=w.kv_layout, kv_seq_stride=w.n_stride, scale=w.scale, tuning=tn,
                                           prepare_only=True)
            return la.lean_attn_attend(problem, inp.q, ks[j], vs[j], inp.seqlens, out, ws, tuning=tn,
                                       prepare_only=True)

        steps_prepared = [prepared(j, tuning) for j in range(copies)]
        steps, warmup = args.steps, args.warmup
        self.ramp(steps_prepared)
        for i in range(warmup):
            steps_prepared[i % copies]()
        t.cuda.synchronize()
        # The timed region: exactly K steps between two synchronisations, enqueued back to back, with
        # one HIP event pair around them on the launch stream.  Its average launch duration (event
        # time / K, gaps between launches included) prices the kernel against the roofline.
        region_start, region_end = self.event_pair()
        t0 = time.perf_counter()
        region_start.record()
        for i in range(steps):
            steps_prepared[i % copies]()
        region_end.record()
        t.cuda.synchronize()
        wall = time.perf_counter() - t0
        assert la.lean_attn_workspace_status(ws) == 0, "a host workgroup timed out waiting for a peer"
        ms_per_step = wall * 1e3 / steps
        avg_ms = region_start.elapsed_time(region_end) / steps
        gbps_job = one_copy / (wall / steps) / 1e9
        gbps_kernel = one_copy / (avg_ms * 1e-3) / 1e9

        # Single-launch latency (the metric's other half): launches each between their own pair of
        # events, so every launch starts on an idle stream.
        self.ramp(steps_prepared, RAMP_MS / 2)
        n_lat = max(steps, min(200, int(0.3 / max(avg_ms * 1e-3, 1e-6))))
        starts = [t.cuda.Event(enable_timing=True) for _ in range(n_lat)]
        ends = [t.cuda.Event(enable_timing=True) for _ in range(n_lat)]
        for i in range(n_lat):
            starts[i].record()
            steps_prepared[i % copies]()
            ends[i].record()
        t.cuda.synchronize()
        lat = sorted(s.elapsed_time(e) for s, e in zip(starts, ends))
        latency = {"avg": round(sum(lat) / len(lat) * 1e3, 2), "median": round(_pct(lat, 0.5) * 1e3, 2),
                   "p10": round(_pct(lat, 0.1) * 1e3, 2), "p90": round(_pct(lat, 0.9) * 1e3, 2), "launches": n_lat,
                   "note": "single launches, each between its own event pair (separate pass)"}

        # The paper's comparison, reproduced with this library's own kernels: the same workload under
        # the fixed-split schedule (one wave of workgroups, equal parts per output tile) and unsplit.
        # All three schedules are timed the same way: prepared calls, back to back under one event pair.
        schedules = None
        if not args.no_schedule_comparison:
            reps = max(10, min(100, int(0.1 / max(avg_ms * 1e-3, 1e-6))))

            def timed_schedule(tn):
                calls = [prepared(j, tn) for j in range(copies)]
                self.ramp(calls, RAMP_MS / 2)
                return self.back_to_back_ms(calls, reps, rounds=3)

            fs_tn, ns_tn = la.Tuning(fixed_split=-1), la.Tuning(fixed_split=1)
            fs_plan = la.lean_attn_problem_schedule(problem, list(w.seqlens), fs_tn)
            sk_ms, fs_ms, ns_ms = timed_schedule(tuning), timed_schedule(fs_tn), timed_schedule(ns_tn)
            schedules = {"stream_k_ms": round(sk_ms, 5), "fixed_split_ms": round(fs_ms, 5),
                         "fixed_split_factor": int(fs_plan.fixed_split), "no_split_ms": round(ns_ms, 5),
                         "speedup_over_fixed_split": round(fs_ms / sk_ms, 3),
                         "speedup_over_no_split": round(ns_ms / sk_ms, 3),
                         "note": "same kernels and fused reduction, only the schedule differs; prepared calls, "
                                 "back to back under one event pair, median of 3 rounds"}

        balance = self.span_balance(w, inp, ks, vs, out, ws, tuning, int(plan.grid), copies)
        traffic, traffic_source = _traffic_from_profiles(w.name)
        res = {
            "workload": w.name, "kv_bytes": one_copy,
            "ms_per_step": round(ms_per_step, 5), "value_GBps": round(gbps_job, 1),
            "launch_duration_us_avg": round(avg_ms * 1e3, 2),   # HIP events around the K timed steps / K
            "GBps": round(gbps_kernel, 1), "frac": round(gbps_kernel / HBM_PEAK_GBPS, 4),
            "latency_us": latency,
            "kernel": "mfma_group" if plan.kernel else "valu_row", "grid": int(plan.grid),
            "block_threads": int(plan.block_threads), "lean_tile": int(plan.T_n),
            "query_rows_per_tile": int(plan.T_m), "iters": int(plan.total_iters), "cache_copies_rotated": copies,
            "traffic": traffic, "traffic_source": traffic_source,
            "schedule_comparison": schedules,
            "span_balance": balance,
        }
        config = {"workload": w.name, "B": w.B, "N_q": w.N_q, "causal": bool(w.causal), "Hq": w.Hq, "Hkv": w.Hkv,
                  "D": w.D, "query_rows_per_tile": int(plan.T_m), "tiles_per_kv_head": int(plan.C_m),
                  "seqlens": list(w.seqlens) if w.B <= 32 else None, "total_context": w.total_tokens,
                  "kv_bytes": one_copy, "kv_layout": "packed" if w.kv_layout else "padded",
                  "grid": int(plan.grid), "lean_tile": int(plan.T_n), "iters": int(plan.total_iters),
                  "kernel": res["kernel"], "cache_copies_rotated": copies}
        extra = {}
        if full:
            extra = self.headline_extras(w, inp, ks, vs, steps_prepared, prepared, tuning, ws, one_copy, copies)
        # The buffers go back to torch's allocator, NOT to the driver (no empty_cache()): the driver wipes
        # device memory it gets back, in the background, and every kernel streams about 9 % slower for
        # about 35 ms per GiB returned (measured: 7.2 -> 6.5 TB/s for 1.15 s after 32 GiB) -- which the
        # next configuration's timed region would pay for.
        del ks, vs, steps_prepared, inp
        return res, config, extra, w

    def span_balance(self, w, inp, ks, vs, out, ws, tuning, grid, copies):
        """When the workgroups finish streaming their equal spans (Section 4.3), from the library's per-CTA
        clock trace (lean_attn_tuning.cta_clock: 16 words per workgroup at 100 MHz; word 0 kernel entry,
        word 1 end of the span loop, word 3 exit).  Microseconds after the first workgroup entered."""
        t, la = self.torch, self.la
        if w.N_q != 1:
            return None
        import numpy as np
        clk = t.zeros(16 * grid, dtype=t.int64, device=self.dev)
        tn = la.Tuning(grid=tuning.grid, ctas_per_cu=tuning.ctas_per_cu, tile_shape=tuning.tile_shape)
        tn.cta_clock = clk.data_ptr()
        ends, exits = [], []
        for i in range(2 + 6):
            j = i % copies
            clk.zero_()
            la.lean_attn_decode(inp.q, ks[j], vs[j], inp.seqlens, out.view(w.B, w.Hq, w.D), ws, Hkv=w.Hkv,
                                kv_layout=w.kv_layout, kv_seq_stride=w.n_stride, scale=w.scale, tuning=tn)
            t.cuda.synchronize()
            c = clk.cpu().numpy().reshape(grid, 16).astype(np.float64)
            if i >= 2:
                t0 = c[:, 0].min()
                ends.append((c[:, 1] - t0) / 100.0)
                exits.append((c[:, 3] - t0) / 100.0)
        end = np.mean(ends, axis=0)
        last = float(np.mean([e.max() for e in ends]))
        by_xcd = [round(float(np.mean([e.max() - e[x::8].mean() for e in ends])), 2) for x in range(min(8, grid))]
        return {"span_loop_end_us": {"first": round(float(np.mean([e.min() for e in ends])), 2),
                                     "median": round(float(np.median(end)), 2), "last": round(last, 2)},
                "kernel_end_us": round(float(np.mean([e.max() for e in exits])), 2),
                "mean_lead_over_last_us": round(float(np.mean([e.max() - e.mean() for e in ends])), 2),
                "mean_lead_by_workgroup_id_mod_8_us": by_xcd,
                "note": "per-CTA clock trace of 6 launches (the trace adds a few stores per workgroup); workgroup "
                        "i runs on XCD i mod 8 on the default stream; lead = how long before the last workgroup a "
                        "workgroup left its span loop"}

    def headline_extras(self, w, inp, ks, vs, steps_prepared, prepared, tuning, ws, one_copy, copies):
        t, la, args = self.torch, self.la, self.args
        extra = {}
        # Warm cache, for problems that fit the last-level cache (labelled as such, never the headline):
        # the same K/V copy every step.
        warm_us = None
        if one_copy <= LLC_BYTES // 2:
            self.ramp(steps_prepared[:1], RAMP_MS / 2)
            n_warm = 100
            wa = [t.cuda.Event(enable_timing=True) for _ in range(n_warm)]
            wb = [t.cuda.Event(enable_timing=True) for _ in range(n_warm)]
            for i in range(n_warm):   # timed exactly like the cold latency loop
                wa[i].record()
                steps_prepared[0]()
                wb[i].record()
            t.cuda.synchronize()
            lat = sorted(a.elapsed_time(b) for a, b in zip(wa, wb))
            warm_us = round(lat[len(lat) // 2] * 1e3, 2)
        extra["warm_cache_latency_us_median"] = warm_us   # null unless the KV cache fits the last-level cache

        # The same launches captured once in a HIP graph and replayed: the launch path leaves the
        # host, what remains is the GPU-side cost per step (how a serving loop would issue it).
        n_graph = max(copies, min(args.steps, 100))
        graph = t.cuda.CUDAGraph()
        with t.cuda.graph(graph):
            # prepared on the capture stream (a prepared call keeps the stream it was made on)
            captured = [prepared(j, tuning) for j in range(copies)]
            for i in range(n_graph):
                captured[i % copies]()
        for _ in range(max(2, int(self.ramp_ms / 2 * 1e-3 / max(one_copy / 6e12 * n_graph, 1e-6)))):
            graph.replay()
        t.cuda.synchronize()
        ga, gb = self.event_pair()
        replays = max(1, args.steps // n_graph)
        ga.record()
        for _ in range(replays):
            graph.replay()
        gb.record()
        t.cuda.synchronize()
        extra["graph_replay_ms_per_step"] = round(ga.elapsed_time(gb) / (replays * n_graph), 5)
        assert la.lean_attn_workspace_status(ws) == 0, "a host workgroup timed out waiting for a peer (graph replay)"
        del graph, captured

        # Streaming-read ceiling of this machine (context only): the same contiguous-share pattern
        # without arithmetic, with non-temporal loads (what the decode kernels use) and with default loads.
        sink = t.zeros(64, dtype=t.int32, device=self.dev)
        n_probe = min(copies, 2)

        def probe(mode: int) -> float:
            best = 0.0
            for grid in (256, 512):   # one or two workgroups per unit: whichever streams faster
                for _ in range(2):
                    la.lean_attn_read_probe(ks[0].view(-1), sink, grid, mode)
                t.cuda.synchronize()
                ps, pe = self.event_pair()
                reps = max(2, min(10, int(0.05 / (one_copy / 6e12))))
                ps.record()
                for r in range(reps):
                    la.lean_attn_read_probe(ks[r % n_probe].view(-1), sink, grid, mode)
                    la.lean_attn_read_probe(vs[r % n_probe].view(-1), sink, grid, mode)
                pe.record()
                t.cuda.synchronize()
                best = max(best, one_copy * reps / (ps.elapsed_time(pe) * 1e-3) / 1e9)
            return best

        extra["stream_read_probe_GBps"] = {"non_temporal_loads": round(probe(2), 1), "default_loads": round(probe(0), 1)}

        if args.calibrate_copy:
            # A plain copy of known size: reads 1 GiB, writes 1 GiB.  Profiler counter runs scale their
            # FETCH_SIZE / WRITE_SIZE readings by what the same counters report for this kernel.
            src = t.empty(1 << 30, dtype=t.uint8, device=self.dev)
            dst = t.empty_like(src)
            for _ in range(3):
                dst.copy_(src)
            t.cuda.synchronize()
            del src, dst

        if not args.no_cpu_baseline:
            extra["cpu_baseline"] = self.cpu_baseline(w, inp)
        return extra

    def cpu_baseline(self, w, inp):
        """The fp64 oracle on the host cores, on a bounded sample of the same workload."""
        import oracle

        workloads, args = self.workloads, self.args
        group = w.Hq // w.Hkv

        # the first `hs` KV heads (all their query heads, every sequence), sized from a one-head trial
        def sample(hs: int):
            if w.kv_layout == workloads.KV_PADDED:
                k_s, v_s = inp.k[:, :hs].contiguous().cpu(), inp.v[:, :hs].contiguous().cpu()
            else:
                k_s, v_s = inp.k[:hs].contiguous().cpu(), inp.v[:hs].contiguous().cpu()
            q_s = inp.q.view(w.B, w.N_q, w.Hq, w.D)[:, :, :hs * group].contiguous().cpu()
            t0 = time.perf_counter()
            _o, _l, threads = oracle.attention(q_s, k_s, v_s, inp.seqlens, N_q=w.N_q, Hq=hs * group, Hkv=hs, D=w.D,
                                               scale=w.scale, causal=w.causal, kv_layout=w.kv_layout,
                                               n_stride=w.n_stride, return_threads=True)
            return time.perf_counter() - t0, threads

        t1, threads = sample(1)
        hs = max(1, min(w.Hkv, int(args.cpu_seconds / max(t1, 1e-3))))
        t_s, threads = sample(hs) if hs > 1 else (t1, threads)
        repeats = 1
        if t_s < 2.0:   # the whole sample takes a fraction of a second: repeat it for a steadier clock
            repeats = min(50, int(2.0 / max(t_s, 1e-3)) + 1)
            t_s = sum(sample(hs)[0] for _ in range(repeats)) / repeats
        sample_bytes = 2 * hs * w.total_tokens * w.D * 2
        return {"value": round(sample_bytes / t_s / 1e9, 4), "unit": "GB/s", "cores": int(threads), "kind": "oracle",
                "seconds": round(t_s, 3), "repeats": repeats,
                "sample": f"first {hs} of {w.Hkv} KV heads of {w.name} (all sequences, {hs * group} query heads), "
                          f"fp64 two-pass oracle, OpenMP; mean of {repeats} run(s), host copy of the inputs not timed"}

    # ---- the context range of the target --------------------------------------------------------
    def context_sweep(self):
        """Streaming rate at contexts 4k .. 256k (D = 128, bf16; MHA 32 heads and GQA 64/8; batch 1 and 4).

        Per point: prepared calls, steps back to back under one event pair, median of 3 rounds, cache
        copies rotated so that no point is served from the last-level cache; next to it a read probe
        without arithmetic or reduction over the same bytes (K and V of a copy are two halves of
        one buffer), launched the same way with one workgroup per compute unit."""
        t, la, workloads = self.torch, self.la, self.workloads
        sink = t.zeros(64, dtype=t.int32, device=self.dev)
        sweep = []
        for (B_s, Hq_s, Hkv_s) in ((1, 32, 32), (1, 64, 8), (4, 32, 32), (4, 64, 8)):
            for ctx in (4096, 8192, 16384, 32768, 65536, 131072, 262144):
                w = workloads.Workload(f"sweep_b{B_s}_h{Hq_s}_{Hkv_s}_n{ctx}", B_s, Hq_s, Hkv_s, 128, "bf16",
                                       (ctx,) * B_s, workloads.KV_PADDED, seed=7)
                if w.kv_bytes > (4 << 30):
                    continue
                n_copies = max(2, min(32, -(-2 * LLC_BYTES // w.kv_bytes) + 1))
                inp = workloads.generate(w, device=self.dev)
                kv = []
                for _ in range(n_copies):
                    buf = t.empty((2,) + tuple(inp.k.shape), dtype=inp.k.dtype, device=self.dev)
                    buf[0].copy_(inp.k)
                    buf[1].copy_(inp.v)
                    kv.append(buf)
                out = t.empty(B_s, Hq_s, 128, dtype=t.float32, device=self.dev)
                wsp = t.empty(la.lean_attn_workspace_size(B_s, Hq_s, Hkv_s, 128, la.BF16), dtype=t.uint8, device=self.dev)
                la.lean_attn_workspace_init(wsp)
                calls = [la.lean_attn_decode(inp.q, kv[j][0], kv[j][1], inp.seqlens, out, wsp, Hkv=Hkv_s,
                                             kv_layout=w.kv_layout, kv_seq_stride=w.n_stride, scale=w.scale,
                                             prepare_only=True) for j in range(n_copies)]
                plan = la.lean_attn_schedule(list(w.seqlens), Hq_s, Hkv_s, 128, la.BF16, w.kv_layout)
                lib_probe = la.binding._load().lean_attn_read_probe
                stream = t.cuda.current_stream().cuda_stream

                def probe_call(j):
                    args_ = (kv[j].data_ptr(), w.kv_bytes, sink.data_ptr(), 256, 2, stream)
                    return lambda: lib_probe(*args_)

                probes = [probe_call(j) for j in range(n_copies)]
                reps = max(20, min(200, int(0.03 / (w.kv_bytes / 6e12))))
                self.ramp(calls)
                ms = self.back_to_back_ms(calls, reps, rounds=3)
                self.ramp(probes, RAMP_MS / 2)
                probe_ms = self.back_to_back_ms(probes, reps, rounds=3)
                assert la.lean_attn_workspace_status(wsp) == 0
                sweep.append({"B": B_s, "Hq": Hq_s, "Hkv": Hkv_s, "context": ctx, "kv_bytes": w.kv_bytes,
                              "grid": int(plan.grid), "us_per_step": round(ms * 1e3, 2),
                              "GBps": round(w.kv_bytes / ms / 1e6, 1),
                              "frac": round(w.kv_bytes / ms / 1e6 / HBM_PEAK_GBPS, 4),
                              "read_probe_us_per_step": round(probe_ms * 1e3, 2),
                              "over_probe_us": round((ms - probe_ms) * 1e3, 2)})
                del inp, kv, calls, probes     # kept in torch's cache: see measure()
        return sweep

    # ---- LeanTile sweep (Section 4.2: the tile size is chosen per architecture by a sweep) -----------
    def tile_sweep(self):
        """Every compiled tile shape x one or two workgroups per unit, per (head dim, dtype, rows per tile).

        Interleaved rounds in one process (boxes of the pool differ by a few percent, so only
        figures from one process are comparable); median microseconds per step, back to back."""
        t, la, workloads = self.torch, self.la, self.workloads
        cases = []
        for D in (64, 128, 256):
            for dtype in ("bf16", "f16"):
                for rows in (1, 8, 16, 32):
                    if D == 256 and rows > 16:
                        continue
                    cases.append((D, dtype, rows))
        result = []
        for (D, dtype, rows) in cases:
            Hkv = 8
            ctx = (1 << 30) // (Hkv * D * 2 * 2)       # 1 GiB of KV per call: the long-context regime of the metric
            w = workloads.Workload(f"tiles_d{D}_{dtype}_r{rows}", 1, Hkv * rows, Hkv, D, dtype, (ctx,),
                                   workloads.KV_PADDED, seed=9)
            code = la.F16 if dtype == "f16" else la.BF16
            inp = workloads.generate(w, device=self.dev)
            n_copies = 2                               # each call reads more than the last-level cache holds
            ks = [inp.k] + [inp.k.clone() for _ in range(n_copies - 1)]
            vs = [inp.v] + [inp.v.clone() for _ in range(n_copies - 1)]
            out = t.empty(1, w.Hq, D, dtype=t.float32, device=self.dev)
            wsp = t.empty(la.lean_attn_workspace_size(1, w.Hq, Hkv, D, code), dtype=t.uint8, device=self.dev)
            la.lean_attn_workspace_init(wsp)
            variants = []
            for shape in range(1, la.NUM_TILE_SHAPES + 1):
                grid_one = 0
                for per_cu in (1, 2):
                    tn = la.Tuning(tile_shape=shape, ctas_per_cu=per_cu)
                    try:
                        plan = la.lean_attn_schedule(list(w.seqlens), w.Hq, Hkv, D, code, w.kv_layout, tn)
                    except la.LeanAttnError as e:
                        if e.status != la.binding.ERR_UNSUPPORTED:
                            raise
                        break             # this shape is not built for the core / head dim
                    if per_cu == 1:
                        grid_one = int(plan.grid)
                    elif int(plan.grid) == grid_one:
                        continue          # the kernel does not fit twice on a unit: same launch as per_cu = 1
                    calls = [la.lean_attn_decode(inp.q, ks[j], vs[j], inp.seqlens, out, wsp, Hkv=Hkv,
                                                 kv_layout=w.kv_layout, kv_seq_stride=w.n_stride, scale=w.scale,
                                                 tuning=tn, prepare_only=True) for j in range(n_copies)]
                    variants.append({"shape": shape, "ctas_per_cu": per_cu, "grid": int(plan.grid),
                                     "lean_tile": int(plan.T_n), "threads": int(plan.block_threads), "calls": calls,
                                     "ms": []})
            for v in variants:
                for i in range(8):
                    v["calls"][i % n_copies]()
            t.cuda.synchronize()
            for _ in range(5):                      # interleaved rounds
                for v in variants:
                    v["ms"].append(self.back_to_back_ms(v["calls"], 8))
            assert la.lean_attn_workspace_status(wsp) == 0
            default_plan = la.lean_attn_schedule(list(w.seqlens), w.Hq, Hkv, D, code, w.kv_layout)
            rowset = []
            for v in variants:
                med = sorted(v["ms"])[len(v["ms"]) // 2]
                rowset.append({"shape": v["shape"], "ctas_per_cu": v["ctas_per_cu"], "grid": v["grid"],
                               "lean_tile": v["lean_tile"], "threads": v["threads"], "us": round(med * 1e3, 2),
                               "frac": round(w.kv_bytes / med / 1e6 / HBM_PEAK_GBPS, 4)})
            best = min(rowset, key=lambda r: r["us"])
            result.append({"D": D, "dtype": dtype, "rows_per_tile": rows, "kv_bytes": w.kv_bytes,
                           "default": {"shape": int(default_plan.tile_shape), "lean_tile": int(default_plan.T_n),
                                       "grid": int(default_plan.grid), "threads": int(default_plan.block_threads)},
                           "best": {k: best[k] for k in ("shape", "ctas_per_cu", "lean_tile", "us")},
                           "variants": rowset})
            print(f"tile sweep D={D} {dtype} rows={rows}: best shape {best['shape']} x{best['ctas_per_cu']} "
                  f"T_n={best['lean_tile']} {best['us']} us", file=sys.stderr, flush=True)
            del inp, ks, vs, variants           # kept in torch's cache: see measure()
        return result


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", type=int, default=0,
                    help="0 (default): the five named configurations, headline = configuration 4; 1..5: only that "
                         "one (6..8: widened shapes)")
    ap.add_argument("--ctas-per-cu", type=int, default=0)
    ap.add_argument("--grid", type=int, default=0)
    ap.add_argument("--tile-shape", type=int, default=0, help="compiled LeanTile shape 1..9 (0: the library default for the shape of the problem)")
    ap.add_argument("--ramp-ms", type=float, default=RAMP_MS,
                    help="untimed sustained launches before every timed region (0 for profiler counter runs, "
                         "where every launch is serialised and the clocks do not matter)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-schedule-comparison", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="target CPU time of the oracle sample")
    ap.add_argument("--context-sweep", action="store_true", help="time contexts 4k..256k (on by default without --workload)")
    ap.add_argument("--no-context-sweep", action="store_true")
    ap.add_argument("--tile-sweep", action="store_true",
                    help="time every compiled LeanTile shape per (head dim, dtype, rows per tile) and report "
                         "them under \"tile_sweep\" (several minutes)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus must be 1 (multi-GPU sharding is design-only)",
              file=sys.stderr)
        return 2

    import torch

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    torch.cuda.set_device(0)
    props = torch.cuda.get_device_properties(0)
    bench = Bench(args)
    settle_ms, settle_rate, settle_first = bench.settle() if args.ramp_ms > 0 else (0.0, None, None)

    per_config = []
    if args.workload == 0:
        order = [1, 2, 3, 5, HEADLINE]
        head = None
        for idx in order:
            res, config, extra, w = bench.measure(idx, full=(idx == HEADLINE))
            per_config.append(res)
            print(f"{res['workload']}: {res['launch_duration_us_avg']} us/step, {res['GBps']} GB/s, "
                  f"frac {res['frac']}", file=sys.stderr, flush=True)
            if idx == HEADLINE:
                head = (res, config, extra, w)
        per_config.sort(key=lambda r: r["workload"])
    else:
        head = bench.measure(args.workload, full=True)
    res, config, extra, w = head

    result = {
        "metric": "decode-attention KV-cache HBM GB/s (latency in ms_per_step / latency_us)",
        "value": res["value_GBps"],
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "clock_ramp_ms": args.ramp_ms,
        "settle": {"waited_ms": settle_ms, "read_probe_GBps": settle_rate, "read_probe_GBps_at_start": settle_first,
                   "note": "before the first configuration: read probe over 1 GiB until the rate is steady (memory freed "
                           "by an earlier process is wiped in the background and slows all traffic meanwhile)"},   # untimed sustained launches before the W warm-up steps of every timed region
        "ms_per_step": res["ms_per_step"],
        "latency_us": res["latency_us"],
        "launch_duration_us_avg": res["launch_duration_us_avg"],
        "graph_replay_ms_per_step": extra.get("graph_replay_ms_per_step"),
        "warm_cache_latency_us_median": extra.get("warm_cache_latency_us_median"),
        "pct_of_hbm_peak": round(100.0 * res["frac"], 2),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,            # element type of Q/K/V; products and sums accumulate in f32
        "accumulate": "f32",
        "data": "synthetic",
        "config": config,
        "roofline": {"bound": "hbm", "achieved": res["GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": res["frac"], "traffic": res["traffic"], "traffic_source": res["traffic_source"],
                     "traffic_note": "HBM bytes per launch read from the committed rocprofv3 --pmc summary named in "
                                     "traffic_source (FETCH_SIZE + WRITE_SIZE, scaled by a 1 GiB copy); not measured "
                                     "by this run"},
        "device": {"name": props.name, "compute_units": props.multi_processor_count,
                   "hbm_bytes": props.total_memory},
        "stream_read_probe_GBps": extra.get("stream_read_probe_GBps"),
        "schedule_comparison": res["schedule_comparison"],
        "span_balance": res["span_balance"],
        "paper_context": "LeanAttention reports speedups over FlashDecoding only (avg 1.73x, up to 2.18x at 256k, "
                         "A100-80GB, FP16->FP32); no absolute number for this metric",
    }
    if per_config:
        result["per_config"] = per_config
    if (args.workload == 0 and not args.no_context_sweep) or args.context_sweep:
        result["context_sweep"] = bench.context_sweep()
    if args.tile_sweep:
        result["tile_sweep"] = bench.tile_sweep()
    if "cpu_baseline" in extra:
        result["cpu_baseline"] = extra["cpu_baseline"]
    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
