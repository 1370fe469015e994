#!/usr/bin/env python3
"""Benchmark of the resharding hot path on one MI355X.

One step = one pass of the whole path over one workload: the repack kernels,
swap-out of the training-side buffers (device-to-host, on the library's side
stream), release of the training copy, re-allocation, swap-in (host-to-device).
Inputs are synthetic and already resident in HBM when the timed region starts.

The headline workload (default C2, the largest that is a task config with the full
swap) gets `--warmup` + `--steps` such steps, timed; in them the swap-out is queued
behind the repack, so that the kernel time in the record is the kernel alone and a
rocprofv3 trace of the same command agrees with it.  After the timed region the same
workload runs a few steps with the swap-out queued BEFORE the repack (the two overlap:
both only read the sources), and the other task workloads (C1, C3, C3P, C4) each run
a few steps of their own, each in a fresh child process started once this one has given its
buffers back; all of that goes into the same record.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C2] [--others C1,C3,C3P,C4]
"""

from __future__ import annotations

import argparse
import ctypes
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E bandwidth
clock = time.perf_counter


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="C2", help="headline workload: C0, C1, C1R, C2, C3, C3P, C3E or C4")
    ap.add_argument("--others", default="C1,C3,C3P,C4",
                    help="workloads measured after the headline one, a few steps each, into `workloads` ('' = none)")
    ap.add_argument("--other-steps", type=int, default=2, help="full steps per workload of --others (after one warm-up)")
    ap.add_argument("--no-swap", action="store_true", help="time the repack alone (not a valid headline run)")
    ap.add_argument("--overlap-steps", type=int, default=3,
                    help="steps with the swap-out queued before the repack, after the timed region (0 = none; use 0 under "
                         "rocprofv3, which makes the runtime copy with shader kernels that starve a concurrent repack)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--verbose", action="store_true", help="progress and per-step timings on stderr")
    ap.add_argument("--framework-baseline", action="store_true",
                    help="also time the same plan as one torch strided copy per descriptor (a GPU-side comparison)")
    ap.add_argument("--streaming", action="store_true",
                    help="after the timed steps, also run the streaming flow once (one source buffer resident at a "
                         "time) and report its peak HBM")
    ap.add_argument("--no-link-probe", action="store_true")
    ap.add_argument("--tuning", default="", help="e.g. tile_bytes=65536,unroll=8 (default 32768, 2)")
    ap.add_argument("--ablate", default="",
                    help="design ablation instead of the benchmark: tunings separated by ';' (e.g. "
                         "'flags=31;flags=23;tile_bytes=65536,unroll=8'), one plan each on the SAME buffers, executed in "
                         "turn for --ablate-rounds rounds (so that all variants see the same physical placement); "
                         "prints one JSON line with the event-timed kernel time of each")
    ap.add_argument("--ablate-rounds", type=int, default=10)
    ap.add_argument("--ablate-repeat", type=int, default=1,
                    help="executes of one variant in a row inside a round, all timed (shows what depends on the execute before "
                         "being the same plan's, e.g. table_copies=1)")
    ap.add_argument("--as-entry", action="store_true",
                    help="(used by the bench itself for --others) measure --workload alone and print it as one entry of `workloads`")
    ap.add_argument("--link", default="", help="(with --as-entry) the link probe's d2h,h2d GB/s from the parent run")
    return ap.parse_args()


def say(a, *msg, detail=False):
    """Progress on stderr: one line per phase always, per-step lines with --verbose."""
    if a.verbose or not detail:
        print("[bench %.1fs]" % (clock() - T_START), *msg, file=sys.stderr, flush=True)


T_START = clock()


def host_info():
    """What the CPU baseline ran on: logical CPUs, the share this process may use, model, RAM."""
    model, mem_kb, avail_kb = None, None, None
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                model = line.split(":", 1)[1].strip()
                break
        for line in open("/proc/meminfo"):
            if line.startswith("MemTotal"):
                mem_kb = int(line.split()[1])
            if line.startswith("MemAvailable"):
                avail_kb = int(line.split()[1])
    except OSError:
        pass
    return {"nproc": os.cpu_count(), "usable_cpus": len(os.sched_getaffinity(0)), "cpu_model": model,
            "host_ram_GB": None if mem_kb is None else round(mem_kb * 1024 / 1e9, 1),
            "host_ram_available_GB": None if avail_kb is None else round(avail_kb * 1024 / 1e9, 1),
            "OMP_NUM_THREADS": os.environ.get("OMP_NUM_THREADS")}


def pinned_view(plan, index, nbytes):
    """The plan's pinned host copy of one source buffer as an int16 numpy array (no copy)."""
    import numpy as np

    raw = (ctypes.c_int16 * (nbytes // 2)).from_address(plan.host_copy(index))
    return np.frombuffer(raw, dtype=np.int16)


def cpu_baseline(wl, host_src, whole):
    """The loop oracle, as it stands, on the host cores.  whole: every destination buffer of the
    workload, at all threads and at one thread; otherwise a bounded sample (destination rank 0 of
    each kind) at all threads.  Sources are the pinned swap copies (no extra host copy)."""
    import numpy as np

    from oracle import fast

    info = host_info()
    dst_lay = dict(wl["dst"])
    sample = "whole workload, all destination buffers in one call"
    sizes, used = fast.buffer_sizes(wl["spec"], dst_lay), fast.buffers_used(wl["spec"], dst_lay)
    need = sum(n for n, u in zip(sizes, used) if u)
    avail = (info["host_ram_available_GB"] or 0) * 1e9
    if not whole or avail < need + 16e9:
        if dst_lay["tp"] > 1 and dst_lay["tp_filter"] < 0:
            dst_lay["tp_filter"] = 0
        if dst_lay["ep"] > 1 and dst_lay["ep_filter"] < 0:
            dst_lay["ep_filter"] = 0
        sample = "destination rank 0 only" + ("" if not whole else " (host RAM too small for every destination buffer at once)")
        sizes, used = fast.buffer_sizes(wl["spec"], dst_lay), fast.buffers_used(wl["spec"], dst_lay)
    dst = [np.empty(n // 2, dtype=np.int16) if u else None for n, u in zip(sizes, used)]
    threads = fast.max_threads()
    t0 = clock()
    fast.reshard(wl["spec"], wl["src"], dst_lay, host_src, dst, threads=threads)  # touches the destination pages
    first = clock() - t0
    # bounded: about half a minute of wall time at most (element-wise transposes run at a tenth of the copies' rate)
    runs = (3 if first < 4.0 else 1) if whole else 1
    dt = None
    for _ in range(runs):
        t0 = clock()
        nbytes = fast.reshard(wl["spec"], wl["src"], dst_lay, host_src, dst, threads=threads)
        dt = min(dt or 1e30, clock() - t0)
    dt1 = None
    if whole and dt * threads * 0.5 < 30.0:  # one core: skipped where it would take too long
        t0 = clock()
        fast.reshard(wl["spec"], wl["src"], dst_lay, host_src, dst, threads=1)
        dt1 = clock() - t0
    out = {
        "value": round(2 * nbytes / dt / 1e9, 3), "unit": "GB/s (read+write)", "cores": threads, "kind": "oracle",
        "sample": "%s, %s: %.2f GB written per run, best of %d after a page-touching run" % (wl["name"], sample, nbytes / 1e9, runs),
    }
    if whole:
        out["one_core_value"] = round(2 * nbytes / dt1 / 1e9, 3) if dt1 else None
        out["host"] = info
    return out


def link_probe(nbytes=1 << 30):
    """Best of plain pinned hipMemcpyAsync D2H / H2D (torch copies), GB/s each way."""
    import torch

    dev = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    host = torch.empty(nbytes, dtype=torch.uint8, pin_memory=True)
    best = {"d2h": 0.0, "h2d": 0.0}
    for _ in range(4):
        for name, (a, b) in (("d2h", (host, dev)), ("h2d", (dev, host))):
            torch.cuda.synchronize()
            t0 = clock()
            a.copy_(b, non_blocking=True)
            torch.cuda.synchronize()
            best[name] = max(best[name], nbytes / (clock() - t0) / 1e9)
    del dev, host
    return best


def source_hash():
    """Hash of the kernel and plan sources: recorded counter figures are tied to it."""
    h = hashlib.sha256()
    for f in ("repack.hip", "plan.cpp", "internal.h"):
        h.update(open(os.path.join(ROOT, "paper_2507_19017_amd", "csrc", f), "rb").read())
    return h.hexdigest()[:16]


class Run:
    """One workload on the device: plan, seeded sources, destinations, and the measurements."""

    def __init__(self, a, name, tuning):
        import torch

        from paper_2507_19017_amd import Plan
        from synth_inputs import BF16_ONE, WORKLOADS, fill_buffer

        self.a, self.torch = a, torch
        self.wl = wl = WORKLOADS[name]
        self.plan = plan = Plan(wl["spec"], wl["src"], wl["dst"], tuning=tuning or None)
        self.info = plan.info()
        self.sizes_s, self.used_s = plan.buf_bytes(0), plan.buf_used(0)
        self.sizes_d, self.used_d = plan.buf_bytes(1), plan.buf_used(1)
        self.src = [fill_buffer(n, wl["seed"] * 1000 + i, "cuda") if u else None
                    for i, (n, u) in enumerate(zip(self.sizes_s, self.used_s))]
        for t in plan.tensors(0):  # norm vectors are ones
            if (t["name"].endswith("ln") or t["name"] in ("ln1", "ln2")) and self.src[t["buffer"]] is not None:
                self.src[t["buffer"]][t["offset"] // 2:(t["offset"] + t["bytes"]) // 2] = BF16_ONE
        self.dst = [torch.empty(n // 2, dtype=torch.int16, device="cuda") if u else None
                    for n, u in zip(self.sizes_d, self.used_d)]
        self.stream = torch.cuda.current_stream()
        self.h = self.stream.cuda_stream
        self.src_bytes = sum(n for n, u in zip(self.sizes_s, self.used_s) if u)
        self.first_used = self.used_s.index(True)
        plan.bind_src(self.ptrs(self.src))
        if not a.no_swap:
            plan.reserve_host()  # pin the host pages outside every timed region
        torch.cuda.synchronize()
        torch.cuda.reset_peak_memory_stats()
        self.kernel_ms, self.out_s, self.in_s, self.first_s, self.freed = [], [], [], [], []

    @staticmethod
    def ptrs(bufs):
        return [0 if b is None else b.data_ptr() for b in bufs]

    def alloc_src(self):
        torch = self.torch
        return [torch.empty(n // 2, dtype=torch.int16, device="cuda") if u else None for n, u in zip(self.sizes_s, self.used_s)]

    def events(self):
        return self.torch.cuda.Event(enable_timing=True), self.torch.cuda.Event(enable_timing=True)

    def step(self, record):
        """Repack, then swap-out behind it, release, re-allocation, swap-in."""
        a, plan, torch, h = self.a, self.plan, self.torch, self.h
        e0, e1 = self.events()
        t0 = clock()
        e0.record(self.stream)
        plan.execute(self.ptrs(self.src), self.ptrs(self.dst), h)
        e1.record(self.stream)
        if not a.no_swap:
            plan.swap_out(h)            # D2H starts when the repack queued above has finished
            plan.swap_wait()
            t1 = clock()
            plan.mark_src_released()
            before = torch.cuda.memory_allocated()
            self.src = None             # the training copy goes back to the allocator
            after = torch.cuda.memory_allocated()
            self.src = self.alloc_src()  # "before the next update": a device home again
            plan.bind_src(self.ptrs(self.src))
            t2 = clock()
            plan.swap_in(h)
            plan.swap_wait_buffer(self.first_used)   # the first stage's weights are usable from here on
            t2b = clock()
            plan.swap_wait()
            t3 = clock()
        torch.cuda.synchronize()
        if record:
            self.kernel_ms.append(e0.elapsed_time(e1))
            if not a.no_swap:
                self.out_s.append(t1 - t0)
                self.in_s.append(t3 - t2)
                self.first_s.append(t2b - t2)
                self.freed.append(before - after)
                say(a, "%s step: kernel %.3f ms, swap-out %.1f GB/s, swap-in %.1f GB/s" % (
                    self.wl["name"], self.kernel_ms[-1], self.src_bytes / (t1 - t0) / 1e9, self.src_bytes / (t3 - t2) / 1e9), detail=True)

    def repack_only(self, n):
        """n more executes back to back, event-timed one by one (no swap in between)."""
        evs = []
        for _ in range(n):
            e0, e1 = self.events()
            e0.record(self.stream)
            self.plan.execute(self.ptrs(self.src), self.ptrs(self.dst), self.h)
            e1.record(self.stream)
            evs.append((e0, e1))
        self.torch.cuda.synchronize()
        return [x.elapsed_time(y) for x, y in evs]

    def overlap(self, n):
        """Steps with the swap-out queued BEFORE the repack: the device-to-host copies run on the
        side stream while the kernel runs.  Evidence that they do: the first buffer's copy ends
        about (its bytes / link rate) after it was queued, and the kernel has started and ended
        inside that window."""
        plan, h, torch = self.plan, self.h, self.torch
        k_ms, out_s, first_ms, kdone_ms, state_at_kernel_end = [], [], [], [], []
        for _ in range(n):
            e0, e1 = self.events()
            torch.cuda.synchronize()
            time.sleep(0.3)             # untimed: the copy engines go idle after the swap-in just before
            t0 = clock()
            plan.swap_out(h)            # D2H starts now on the side stream
            e0.record(self.stream)
            plan.execute(self.ptrs(self.src), self.ptrs(self.dst), h)
            e1.record(self.stream)
            e1.synchronize()
            t_k = clock()
            state_at_kernel_end.append(plan.src_buffer_state(self.first_used))
            plan.swap_wait_buffer(self.first_used)
            t_b = clock()
            plan.swap_wait()
            t1 = clock()
            k_ms.append(e0.elapsed_time(e1))
            out_s.append(t1 - t0)
            first_ms.append((t_b - t0) * 1e3)
            kdone_ms.append((t_k - t0) * 1e3)
            # back to RESIDENT without moving anything: the device copy was never dropped
            plan.mark_src_released()
            plan.bind_src(self.ptrs(self.src))
            plan.swap_in(h)
            plan.swap_wait()
        k = sum(k_ms) / len(k_ms) / 1e3
        so = sum(out_s) / len(out_s)
        return {
            "steps": n, "order": "swap_out queued first, execute second, same caller stream",
            "repack_GBps": round(2 * self.info["bytes_moved"] / k / 1e9, 1), "repack_kernel_ms_avg": round(k * 1e3, 4),
            "repack_frac_of_peak": round(2 * self.info["bytes_moved"] / k / 1e9 / HBM_PEAK_GBPS, 4),
            "swap_out_GBps": round(self.src_bytes / so / 1e9, 2),
            "swap_out_GBps_best_step": round(self.src_bytes / min(out_s) / 1e9, 2),
            "concurrency_evidence": {
                "kernel_done_ms_after_swap_out_was_queued": round(sum(kdone_ms) / n, 3),
                "first_buffer_copy_done_ms_after_swap_out_was_queued": round(sum(first_ms) / n, 3),
                "first_buffer_bytes": self.sizes_s[self.first_used],
                "first_buffer_state_when_the_kernel_ended": sorted(set(state_at_kernel_end)),
            },
        }

    def driver_free_check(self):
        """Untimed: the same release all the way back to the driver, to show the HBM really becomes
        free (a fresh allocation is slow on first touch, which is why the timed steps recycle the
        allocator's blocks instead), and a strided checksum across the round trip."""
        plan, torch, h = self.plan, self.torch, self.h
        check = [None if s is None else int(s[::4099].to(torch.int64).sum()) for s in self.src]
        plan.swap_out(h)
        plan.swap_wait()
        plan.mark_src_released()
        free0 = torch.cuda.mem_get_info()[0]
        self.src = None
        torch.cuda.empty_cache()
        driver_freed = torch.cuda.mem_get_info()[0] - free0
        self.src = self.alloc_src()
        plan.bind_src(self.ptrs(self.src))
        plan.swap_in(h)
        plan.swap_wait()
        torch.cuda.synchronize()
        assert check == [None if s is None else int(s[::4099].to(torch.int64).sum()) for s in self.src], "swap round trip changed the weights"
        return driver_freed

    def probes(self):
        """Plain copy and one-way rates with the copy kernel's tile and launch shape, on this
        workload's largest buffers: a copy moves equal bytes both ways over the same memory, so
        2 / (1/R + 1/W) bounds it."""
        from paper_2507_19017_amd import copy_baseline, read_baseline, write_baseline

        torch, h = self.torch, self.h
        big_s = max((s for s in self.src if s is not None), key=lambda t: t.numel())
        big_d = max((d for d in self.dst if d is not None), key=lambda t: t.numel())
        cp_n = min(big_s.numel() * 2, big_d.numel() * 2, 8 << 30) // 32768 * 32768

        def best_ms(fn):
            evs = []
            for _ in range(6):
                e0, e1 = self.events()
                e0.record(self.stream)
                fn()
                e1.record(self.stream)
                evs.append((e0, e1))
            torch.cuda.synchronize()
            return min(x.elapsed_time(y) for x, y in evs[1:])

        if cp_n <= 0:
            return None
        plain = 2 * cp_n / (best_ms(lambda: copy_baseline(big_d.data_ptr(), big_s.data_ptr(), cp_n, h)) / 1e3) / 1e9
        rd = cp_n / (best_ms(lambda: read_baseline(big_s.data_ptr(), cp_n, h)) / 1e3) / 1e9
        wr = cp_n / (best_ms(lambda: write_baseline(big_d.data_ptr(), cp_n, h)) / 1e3) / 1e9
        return {"plain_copy_GBps": round(plain, 1), "read_only_GBps": round(rd, 1), "write_only_GBps": round(wr, 1),
                "mixed_bound_GBps": round(2.0 / (1.0 / rd + 1.0 / wr), 1)}

    def host_sources(self):
        """Pinned host copies of the sources (a swap-out; the device copies stay) for the oracle."""
        self.plan.swap_out(self.h)
        self.plan.swap_wait()
        return [pinned_view(self.plan, i, n) if u else None for i, (n, u) in enumerate(zip(self.sizes_s, self.used_s))]

    def close(self):
        self.src = self.dst = None
        self.plan.destroy()
        self.torch.cuda.synchronize()
        self.torch.cuda.empty_cache()

    def summary(self, link):
        """Figures every workload reports."""
        moved = self.info["bytes_moved"]
        k_avg = sum(self.kernel_ms) / len(self.kernel_ms) / 1e3
        gbps = 2 * moved / k_avg / 1e9
        out = {"workload": "%s: %s" % (self.wl["name"], self.wl["note"]), "bytes_moved_one_way": moved,
               "kernel_ms_avg": round(k_avg * 1e3, 4), "kernel_ms_min": round(min(self.kernel_ms), 4),
               "kernel_samples": len(self.kernel_ms), "GBps": round(gbps, 1), "frac": round(gbps / HBM_PEAK_GBPS, 4),
               "ledger_peak_device": self.plan.mem_stats()["peak_device"],
               "torch_max_allocated": self.torch.cuda.max_memory_allocated()}
        if self.out_s:
            so, si = sum(self.out_s) / len(self.out_s), sum(self.in_s) / len(self.in_s)
            out["swap"] = {"bytes_each_way": self.src_bytes, "out_GBps": round(self.src_bytes / so / 1e9, 2),
                           "in_GBps": round(self.src_bytes / si / 1e9, 2),
                           "out_GBps_best_step": round(self.src_bytes / min(self.out_s) / 1e9, 2),
                           "in_GBps_best_step": round(self.src_bytes / min(self.in_s) / 1e9, 2),
                           "in_first_buffer_ms": round(sum(self.first_s) / len(self.first_s) * 1e3, 2),
                           "in_all_buffers_ms": round(si * 1e3, 2)}
            if link:
                out["swap"]["out_frac_of_link"] = round(self.src_bytes / so / 1e9 / link["d2h"], 3)
                out["swap"]["in_frac_of_link"] = round(self.src_bytes / si / 1e9 / link["h2d"], 3)
        return out


def framework_baseline(run):
    """What the slice selection and copy looks like with framework tensor operations: one strided
    tensor copy per descriptor of the same plan (torch.as_strided views of the flat buffers,
    Tensor.copy_), on the same buffers.  A GPU-side comparison only: the product path never runs it."""
    torch, plan, src, dst = run.torch, run.plan, run.src, run.dst
    assert run.wl["spec"]["elem_bytes"] == 2, "the framework baseline views the buffers as 16-bit words"
    views = []
    for d in plan.descs():
        sb, db = src[d["src_buf"]], dst[d["dst_buf"]]
        cols = d["row_bytes"] // 2
        sv = torch.as_strided(sb, (d["rows"], cols), (d["src_stride"] // 2, 1), d["src_off"] // 2)
        if d["kind"] == 0:
            dv = torch.as_strided(db, (d["rows"], cols), (d["dst_stride"] // 2, 1), d["dst_off"] // 2)
        else:  # transposing: element (i, k) lands at row k, column i
            dv = torch.as_strided(db, (d["rows"], cols), (1, d["dst_stride"] // 2), d["dst_off"] // 2)
        views.append((dv, sv))
    ref = [None if t is None else t.clone() for t in dst]
    for t in dst:
        if t is not None:
            t.zero_()

    def run_views():
        for dv, sv in views:
            dv.copy_(sv)

    run_views()
    torch.cuda.synchronize()
    same = all((x is None and y is None) or torch.equal(x, y) for x, y in zip(ref, dst))
    del ref
    times = []
    for _ in range(3):
        torch.cuda.synchronize()
        t0 = clock()
        run_views()
        torch.cuda.synchronize()
        times.append(clock() - t0)
    best = min(times)
    return {"kind": "one torch strided copy_ per descriptor", "copies": len(views), "ms": round(best * 1e3, 3),
            "GBps": round(2 * run.info["bytes_moved"] / best / 1e9, 1), "same_bits_as_the_library": same}


def streaming_flow(run, tuning):
    """The gathered shards "arrive" one buffer at a time: repack what reads it, swap it out, drop it."""
    from paper_2507_19017_amd import Plan

    torch, wl, h = run.torch, run.wl, run.h
    run.plan.release_host()
    run.src = None
    torch.cuda.empty_cache()
    splan = Plan(wl["spec"], wl["src"], wl["dst"], tuning=tuning or None)
    splan.prepare()
    splan.reserve_host()  # pin the host pages outside the timed region
    base = torch.cuda.memory_allocated()
    torch.cuda.reset_peak_memory_stats()
    torch.cuda.synchronize()
    t0 = clock()
    in_flight = []  # (index, tensor): at most two source buffers are resident at any time
    host_ms = {"alloc": 0.0, "execute": 0.0, "swap_queue": 0.0, "wait": 0.0}
    for i, (n, u) in enumerate(zip(run.sizes_s, run.used_s)):
        if not u:
            continue
        c0 = clock()
        buf = torch.empty(n // 2, dtype=torch.int16, device="cuda")
        c1 = clock()
        splan.execute_source(i, buf.data_ptr(), run.ptrs(run.dst), h)
        c2 = clock()
        splan.swap_out_source(i, h)      # its copy runs while the next buffer is repacked
        c3 = clock()
        in_flight.append((i, buf))
        if len(in_flight) == 2:
            j, old = in_flight.pop(0)
            splan.swap_wait_buffer(j)
            splan.mark_src_buffer_released(j)
            del old
        c4 = clock()
        for k, v in zip(host_ms, (c1 - c0, c2 - c1, c3 - c2, c4 - c3)):
            host_ms[k] += v * 1e3
    for j, old in in_flight:
        splan.swap_wait_buffer(j)
        splan.mark_src_buffer_released(j)
    del in_flight, buf, old
    torch.cuda.synchronize()
    t1 = clock()
    sst = splan.mem_stats()
    out = {"total_ms": round((t1 - t0) * 1e3, 2), "ledger_peak_device": sst["peak_device"],
           "torch_peak_allocated": torch.cuda.max_memory_allocated(), "dst_bytes": sst["dst_live"],
           "largest_src_buffer": max(n for n, u in zip(run.sizes_s, run.used_s) if u), "buffers_in_flight": 2,
           "host_ms": {k: round(v, 1) for k, v in host_ms.items()}, "state": sst["state"],
           "one_shot_peak_device": run.plan.mem_stats()["peak_device"], "allocated_before": base}
    run.src = run.alloc_src()  # a device home again, and the weights back, so the rest of the run goes on
    splan.bind_src(run.ptrs(run.src))
    splan.swap_in(h)
    splan.swap_wait()
    splan.destroy()
    run.plan.bind_src(run.ptrs(run.src))
    return out


def ablation(a, run):
    """The repack under several tunings on the same source and destination buffers, in turn.
    Dispatch order (for reading a kernel trace of this run): one warm-up execute per variant in
    the order given, then `rounds` rounds of: one untimed execute of the last variant, one timed
    execute per variant in the order given."""
    from paper_2507_19017_amd import Plan

    wl, torch = run.wl, run.torch
    variants = [v for v in a.ablate.split(";") if v]
    plans = []
    for v in variants:
        tn = {k: int(x) for k, x in (kv.split("=") for kv in v.split(","))}
        p = Plan(wl["spec"], wl["src"], wl["dst"], tuning=tn)
        p.prepare()
        plans.append(p)
    for p in plans:
        p.execute(run.ptrs(run.src), run.ptrs(run.dst), run.h)
    torch.cuda.synchronize()
    times = [[] for _ in plans]
    for _ in range(a.ablate_rounds):
        evs = []
        plans[-1].execute(run.ptrs(run.src), run.ptrs(run.dst), run.h)  # untimed: the first launch after a host wait runs slow
        for i, p in enumerate(plans):
            for _ in range(max(1, a.ablate_repeat)):
                e0, e1 = run.events()
                e0.record(run.stream)
                p.execute(run.ptrs(run.src), run.ptrs(run.dst), run.h)
                e1.record(run.stream)
                evs.append((i, e0, e1))
        torch.cuda.synchronize()
        for i, e0, e1 in evs:
            times[i].append(e0.elapsed_time(e1))
    moved = run.info["bytes_moved"]
    base = sum(times[0]) / len(times[0])
    out = []
    for v, p, t in zip(variants, plans, times):
        avg = sum(t) / len(t)
        out.append({"tuning": v, "tiles": p.info()["num_tiles"], "kernel_ms_avg": round(avg, 4), "kernel_ms_min": round(min(t), 4),
                    "GBps": round(2 * moved / avg / 1e6, 1), "frac": round(2 * moved / avg / 1e6 / HBM_PEAK_GBPS, 4),
                    "vs_first_pct": round(100 * (base / avg - 1), 2)})
        rep = max(1, a.ablate_repeat)
        if rep > 1:  # the first execute of a row follows another plan's, the later ones this plan's own
            lead, rest = t[0::rep], [x for i, x in enumerate(t) if i % rep]
            out[-1]["GBps_first_in_row"] = round(2 * moved / (sum(lead) / len(lead)) / 1e6, 1)
            out[-1]["GBps_later_in_row"] = round(2 * moved / (sum(rest) / len(rest)) / 1e6, 1)
            out[-1]["table_copies"] = p.get_tuning()["table_copies"]
        p.destroy()
    return {"ablation": out, "workload": "%s: %s" % (wl["name"], wl["note"]), "bytes_moved_one_way": moved,
            "rounds": a.ablate_rounds, "repeat": max(1, a.ablate_repeat),
            "order": "one warm-up execute per variant, then rounds of (one untimed execute of the last variant, `repeat` timed "
                     "executes in a row per variant in the order given)"}


def entry_of(a, run):
    """One entry of the record's `workloads` array: a warm-up step and a few full steps, more executes of the
    repack alone, the overlapped order, and the CPU oracle on a bounded sample."""
    link = None
    if a.link:
        d2h, h2d = (float(x) for x in a.link.split(","))
        link = {"d2h": d2h, "h2d": h2d}
    for _ in range(a.warmup):
        run.step(False)
    for _ in range(a.steps):
        run.step(True)
    run.kernel_ms += run.repack_only(6)[1:]  # more samples of the kernel alone, back to back
    entry = run.summary(link)
    if a.overlap_steps > 0 and not a.no_swap:
        ov = run.overlap(a.overlap_steps)
        say(a, run.wl["name"], "overlap:", json.dumps(ov), detail=True)
        entry["overlap"] = {k: ov[k] for k in ("repack_GBps", "repack_frac_of_peak", "swap_out_GBps", "swap_out_GBps_best_step")}
    if not a.no_cpu_baseline and not a.no_swap:
        entry["cpu_baseline"] = cpu_baseline(run.wl, run.host_sources(), whole=False)
    run.close()
    return entry


def recorded_traffic(name, tuning_now):
    """HBM bytes per execute from earlier rocprofv3 --pmc runs (FETCH_SIZE and WRITE_SIZE, each scaled
    by the same counter's reading for a plain copy of known size), kept in profiles/.  A recorded
    figure, not one this run measured: it is dropped when the kernel sources or the tuning have
    changed since it was taken."""
    path = os.path.join(ROOT, "profiles", "repack_hbm_traffic.json")
    if not os.path.exists(path):
        return None, None
    entry = json.load(open(path)).get(name)
    if not entry:
        return None, None
    entry = dict(entry, recorded=True)
    stale = []
    if entry.get("csrc_sha") != source_hash():
        stale.append("kernel or plan sources changed since the counters were read")
    if entry.get("tuning") and {k: entry["tuning"].get(k) for k in ("tile_bytes", "block_threads", "blocks_per_cu", "unroll", "flags")} != \
            {k: tuning_now.get(k) for k in ("tile_bytes", "block_threads", "blocks_per_cu", "unroll", "flags")}:
        stale.append("tuning differs from the recorded run's")
    if stale:
        entry["stale"] = stale
        return None, entry
    return entry["total_bytes"], entry


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    import torch

    from paper_2507_19017_amd.build import ensure_built

    ensure_built()  # compiles only if no library is there
    from synth_inputs import WORKLOADS

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    tuning = {k: int(v) for k, v in (kv.split("=") for kv in a.tuning.split(","))} if a.tuning else {}
    assert a.workload in WORKLOADS, a.workload
    others = [w for w in a.others.split(",") if w and w != a.workload]
    for w in others:
        assert w in WORKLOADS, w

    # ------------------------------------------------------------ headline workload ----
    say(a, "filling", a.workload)
    if a.ablate:
        a.no_swap = True
    run = Run(a, a.workload, tuning)
    if a.ablate:
        print(json.dumps(ablation(a, run)))
        return
    if a.as_entry:
        print(json.dumps(entry_of(a, run)))
        return
    say(a, "warm-up")
    for _ in range(a.warmup):
        run.step(False)
    torch.cuda.synchronize()
    t_begin = clock()
    for _ in range(a.steps):
        run.step(True)
    torch.cuda.synchronize()
    total_s = clock() - t_begin
    say(a, "timed region done: %.2f s" % total_s)

    # the overlapped order comes before anything gives memory back to the driver: for some seconds after tens of
    # GB were freed (the driver clears them) host copies on this machine run at half rate now and then
    overlap = run.overlap(a.overlap_steps) if (a.overlap_steps > 0 and not a.no_swap) else None
    say(a, "overlap done")
    # the same kernel with nothing between the executes: in a step it starts after seconds of link copies during
    # which the shader engines sat idle
    b2b = run.repack_only(7)[1:]
    link = None if a.no_link_probe or a.no_swap else link_probe()
    head = run.summary(link)
    driver_freed = None if a.no_swap else run.driver_free_check()
    framework = framework_baseline(run) if a.framework_baseline else None
    streaming = streaming_flow(run, tuning) if a.streaming else None
    probes = run.probes()
    plan_tuning = run.plan.get_tuning()
    traffic, traffic_detail = recorded_traffic(a.workload, plan_tuning)
    cpu = None
    if not a.no_cpu_baseline:
        say(a, "cpu baseline")
        if a.no_swap:
            host_src = [None if s is None else s.cpu().numpy() for s in run.src]
            cpu = cpu_baseline(run.wl, host_src, whole=True)
        else:
            cpu = cpu_baseline(run.wl, run.host_sources(), whole=True)
    stats = run.plan.mem_stats()
    moved, info = head["bytes_moved_one_way"], run.info
    config = {"workload": head["workload"], "bytes_moved_one_way": moved,
              "src_buffers": sum(run.used_s), "dst_buffers": sum(run.used_d),
              "descriptors": info["num_descs"], "tiles": info["num_tiles"], "tuning": plan_tuning,
              "swap_overlaps_repack": False,
              "step": "repack, swap-out behind it, release, re-allocation, swap-in; the overlapped order is measured "
                      "after the timed region (`overlap`)"}
    freed = run.freed
    run.close()
    say(a, "headline workload done")

    # ------------------------------------------------------------ the other task workloads ----
    # Each in a process of its own, one after the other (this one holds no buffers any more): the same conditions
    # as the headline workload had, and nothing one workload frees disturbs the next one's copies.
    import subprocess

    workloads = [dict(head, swap_overlaps_repack=False)]
    for name in others:
        say(a, "workload", name)
        cmd = [sys.executable, os.path.abspath(__file__), "--as-entry", "--workload", name, "--steps", str(max(1, a.other_steps)),
               "--warmup", "1", "--overlap-steps", str(min(2, a.overlap_steps))]
        cmd += ["--tuning", a.tuning] if a.tuning else []
        cmd += [flag for flag, on in (("--no-swap", a.no_swap), ("--no-cpu-baseline", a.no_cpu_baseline), ("--verbose", a.verbose)) if on]
        if link:
            cmd += ["--link", "%.3f,%.3f" % (link["d2h"], link["h2d"])]
        res = subprocess.run(cmd, stdout=subprocess.PIPE, text=True)  # its progress lines go to this process's stderr
        if res.returncode != 0:
            raise SystemExit("bench.py: the run of workload %s failed with exit code %d" % (name, res.returncode))
        workloads.append(json.loads(res.stdout.strip().splitlines()[-1]))

    out = {
        "metric": "reshard repack GB/s (read+write)",
        "value": head["GBps"],
        "unit": "GB/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": round(total_s / a.steps * 1e3, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u16", "data": "synthetic",
        "config": config,
        "roofline": dict({"bound": "hbm", "achieved": head["GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                          "frac": head["frac"], "traffic": traffic, "algorithmic_bytes": 2 * moved,
                          "traffic_detail": traffic_detail,
                          "kernel_ms_avg": head["kernel_ms_avg"], "kernel_ms_min": head["kernel_ms_min"]},
                         **(probes or {})),
        "pct_hbm_peak": round(100 * head["frac"], 2),
        "peak_hbm_bytes": {"ledger": stats["peak_device"], "torch_max_allocated": head["torch_max_allocated"],
                           "plan_tile_tables": plan_tuning["table_copies"] * (info["table_bytes"] + 256),
                           "freed_after_swap_out": (sum(freed) // len(freed)) if freed else None,
                           "returned_to_driver_after_swap_out": driver_freed},
    }
    if probes:
        out["roofline"]["frac_of_mixed_bound"] = round(head["GBps"] / probes["mixed_bound_GBps"], 4)
    b2b_s = sum(b2b) / len(b2b) / 1e3
    out["roofline"]["back_to_back"] = {"what": "executes queued back to back after the timed region, event-timed one by one (not `value`)",
                                       "samples": len(b2b), "kernel_ms_avg": round(b2b_s * 1e3, 4),
                                       "GBps": round(2 * moved / b2b_s / 1e9, 1), "frac": round(2 * moved / b2b_s / 1e9 / HBM_PEAK_GBPS, 4)}
    if "swap" in head:
        out["swap"] = dict(head["swap"], link_probe_GBps=None if link is None else {k: round(v, 2) for k, v in link.items()})
    if overlap:
        out["overlap"] = overlap
    if streaming:
        out["streaming"] = streaming
    if framework:
        out["framework_baseline"] = framework
    if cpu:
        out["cpu_baseline"] = cpu
    out["workloads"] = workloads
    print(json.dumps(out))


if __name__ == "__main__":
    main()
