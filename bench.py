#!/usr/bin/env python3
"""Benchmark of the resharding hot path on one MI355X.

One step = one pass of the whole path over one workload: the repack kernel,
swap-out of the training-side buffers (device-to-host, on the library's side
stream; --overlap queues it before the repack so the two run concurrently),
release of the training copy, re-allocation, swap-in (host-to-device).  Inputs are synthetic and already resident in HBM when the
timed region starts.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C1]
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

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E bandwidth


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="C1", help="C0, C1, C1R, C2, C3, C3P or C4")
    ap.add_argument("--no-swap", action="store_true", help="time the repack alone (not a valid headline run)")
    ap.add_argument("--overlap", action="store_true",
                    help="queue the swap-out before the repack so the two overlap (under rocprofv3 the runtime "
                         "copies with shader kernels instead of the DMA engines, which starves the repack)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--verbose", action="store_true", help="per-step timings on stderr")
    ap.add_argument("--framework-baseline", action="store_true",
                    help="also time the same plan as one torch strided copy per descriptor (a GPU-side comparison)")
    ap.add_argument("--streaming", action="store_true",
                    help="after the timed steps, also run the streaming flow once (one source buffer resident at a "
                         "time) and report its peak HBM")
    ap.add_argument("--no-link-probe", action="store_true")
    ap.add_argument("--tuning", default="", help="e.g. tile_bytes=65536,unroll=8 (default 32768, 2)")
    return ap.parse_args()


def cpu_baseline(wl, plan, src):
    """The loop oracle, as it stands, on the host cores, on a bounded sample:
    destination tensor rank 0 (and expert rank 0) of the same workload."""
    import numpy as np

    from oracle import fast
    from paper_2507_19017_amd import Plan

    only = dict(wl["dst"])
    if only["tp"] > 1:
        only["tp_filter"] = 0
    if only["ep"] > 1 and only["ep_filter"] < 0:
        only["ep_filter"] = 0
    sub = Plan(wl["spec"], wl["src"], only)
    used_src = sub.buf_used(0)
    host_src = [s.cpu().numpy() if (u and s is not None) else None for s, u in zip(src, used_src)]
    sizes, used = fast.buffer_sizes(wl["spec"], only), fast.buffers_used(wl["spec"], only)
    dst = [np.zeros(n // 2, dtype=np.int16) if u else None for n, u in zip(sizes, used)]
    threads = min(fast.max_threads(), 16)
    fast.reshard(wl["spec"], wl["src"], only, host_src, dst, threads=threads)  # warm the pages
    dt = None
    for _ in range(3):  # best of three: the runs are short
        t0 = time.perf_counter()
        nbytes = fast.reshard(wl["spec"], wl["src"], only, host_src, dst, threads=threads)
        dt = min(dt or 1e30, time.perf_counter() - t0)
    dt1 = None
    if dt * threads < 40.0:  # keep the default run short: skipped where one core would need longer
        t0 = time.perf_counter()
        fast.reshard(wl["spec"], wl["src"], only, host_src, dst, threads=1)
        dt1 = time.perf_counter() - t0
    return {
        "value": round(2 * nbytes / dt / 1e9, 3), "unit": "GB/s (read+write)", "cores": threads,
        "kind": "oracle", "one_core_value": round(2 * nbytes / dt1 / 1e9, 3) if dt1 else None,
        "sample": "%s, destination rank 0 only: %.2f GB written, best of three runs after a page-warming run" % (wl["name"], nbytes / 1e9),
    }


def link_probe(nbytes=1 << 30):
    """Best of plain pinned hipMemcpyAsync D2H / H2D (torch copies), GB/s each way."""
    import torch

    dev = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    host = torch.empty(nbytes, dtype=torch.uint8, pin_memory=True)
    best = {"d2h": 0.0, "h2d": 0.0}
    for _ in range(4):
        for name, (a, b) in (("d2h", (host, dev)), ("h2d", (dev, host))):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            a.copy_(b, non_blocking=True)
            torch.cuda.synchronize()
            best[name] = max(best[name], nbytes / (time.perf_counter() - t0) / 1e9)
    del dev, host
    return best


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    import torch

    from paper_2507_19017_amd.build import ensure_built

    ensure_built()  # compiles only if no library is there
    from paper_2507_19017_amd import Plan, copy_baseline, get_tuning, read_baseline, set_tuning, write_baseline
    from synth_inputs import BF16_ONE, WORKLOADS, fill_buffer

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if a.tuning:
        set_tuning(**{k: int(v) for k, v in (kv.split("=") for kv in a.tuning.split(","))})
    wl = WORKLOADS[a.workload]
    plan = Plan(wl["spec"], wl["src"], wl["dst"])
    info = plan.info()
    sizes_s, used_s = plan.buf_bytes(0), plan.buf_used(0)
    sizes_d, used_d = plan.buf_bytes(1), plan.buf_used(1)

    def alloc_src(fill):
        out = []
        for i, (n, u) in enumerate(zip(sizes_s, used_s)):
            if not u:
                out.append(None)
            elif fill:
                out.append(fill_buffer(n, wl["seed"] * 1000 + i, "cuda"))
            else:
                out.append(torch.empty(n // 2, dtype=torch.int16, device="cuda"))
        return out

    src = alloc_src(True)
    for t in plan.tensors(0):  # norm vectors are ones
        if (t["name"].endswith("ln") or t["name"] in ("ln1", "ln2")) and src[t["buffer"]] is not None:
            src[t["buffer"]][t["offset"] // 2:(t["offset"] + t["bytes"]) // 2] = BF16_ONE
    dst = [torch.empty(n // 2, dtype=torch.int16, device="cuda") if u else None for n, u in zip(sizes_d, used_d)]
    ptrs = lambda bufs: [0 if b is None else b.data_ptr() for b in bufs]
    stream = torch.cuda.current_stream()
    h = stream.cuda_stream
    src_bytes = sum(n for n, u in zip(sizes_s, used_s) if u)
    plan.bind_src(ptrs(src))
    torch.cuda.reset_peak_memory_stats()

    kernel_ms, out_s, in_s, first_s, freed = [], [], [], [], []
    first_used = used_s.index(True)

    def step(record):
        nonlocal src
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        if a.overlap and not a.no_swap:
            plan.swap_out(h)            # D2H starts now on the side stream and overlaps the repack
        e0.record(stream)
        plan.execute(ptrs(src), ptrs(dst), h)
        e1.record(stream)
        if not a.no_swap:
            if not a.overlap:
                plan.swap_out(h)        # D2H starts when the repack queued above has finished
            plan.swap_wait()
            t1 = time.perf_counter()
            plan.mark_src_released()
            before = torch.cuda.memory_allocated()
            src = None                  # the training copy goes back to the allocator
            after = torch.cuda.memory_allocated()
            src = alloc_src(False)      # "before the next update": a device home again
            plan.bind_src(ptrs(src))
            t2 = time.perf_counter()
            plan.swap_in(h)
            plan.swap_wait_buffer(first_used)   # the first stage's weights are usable from here on
            t2b = time.perf_counter()
            plan.swap_wait()
            t3 = time.perf_counter()
        torch.cuda.synchronize()
        if record:
            kernel_ms.append(e0.elapsed_time(e1))
            if not a.no_swap:
                out_s.append(t1 - t0)
                in_s.append(t3 - t2)
                first_s.append(t2b - t2)
                freed.append(before - after)
                if a.verbose:
                    print("step: kernel %.3f ms, swap-out %.1f GB/s, swap-in %.1f GB/s" % (
                        kernel_ms[-1], src_bytes / (t1 - t0) / 1e9, src_bytes / (t3 - t2) / 1e9), file=sys.stderr)

    for _ in range(a.warmup):
        step(False)
    torch.cuda.synchronize()
    t_begin = time.perf_counter()
    for _ in range(a.steps):
        step(True)
    torch.cuda.synchronize()
    total_s = time.perf_counter() - t_begin

    # untimed: the same release, this time all the way back to the driver, to show the
    # HBM really becomes free (a fresh allocation is slow on first touch, which is
    # why the timed steps above recycle the allocator's blocks instead)
    driver_freed = None
    if not a.no_swap:
        check = [None if s is None else int(s[::4099].to(torch.int64).sum()) for s in src]
        plan.swap_out(h)
        plan.swap_wait()
        plan.mark_src_released()
        free0 = torch.cuda.mem_get_info()[0]
        src = None
        torch.cuda.empty_cache()
        driver_freed = torch.cuda.mem_get_info()[0] - free0
        src = alloc_src(False)
        plan.bind_src(ptrs(src))
        plan.swap_in(h)
        plan.swap_wait()
        torch.cuda.synchronize()
        assert check == [None if s is None else int(s[::4099].to(torch.int64).sum()) for s in src], "swap round trip changed the weights"

    framework = None
    if a.framework_baseline:
        # What the slice selection and copy looks like with framework tensor operations: one strided
        # tensor copy per descriptor of the same plan (torch.as_strided views of the flat
        # buffers, Tensor.copy_), on the same buffers.  A GPU-side comparison only: the
        # product path never runs it.
        eb = wl["spec"]["elem_bytes"]
        assert eb == 2, "the framework baseline views the buffers as 16-bit words"
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
            t0 = time.perf_counter()
            run_views()
            torch.cuda.synchronize()
            times.append(time.perf_counter() - t0)
        best = min(times)
        framework = {"kind": "one torch strided copy_ per descriptor", "copies": len(views), "ms": round(best * 1e3, 3),
                     "GBps": round(2 * info["bytes_moved"] / best / 1e9, 1), "same_bits_as_the_library": same}

    streaming = None
    if a.streaming:
        # the gathered shards "arrive" one buffer at a time: repack what reads it, swap it out, drop it
        plan.release_host()
        src = None
        torch.cuda.empty_cache()
        splan = Plan(wl["spec"], wl["src"], wl["dst"])
        splan.prepare()
        splan.reserve_host()  # pin the host pages outside the timed region
        base = torch.cuda.memory_allocated()
        torch.cuda.reset_peak_memory_stats()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        in_flight = []  # (index, tensor): at most two source buffers are resident at any time
        host_ms = {"alloc": 0.0, "execute": 0.0, "swap_queue": 0.0, "wait": 0.0}
        clock = time.perf_counter
        for i, (n, u) in enumerate(zip(sizes_s, used_s)):
            if not u:
                continue
            c0 = clock()
            buf = torch.empty(n // 2, dtype=torch.int16, device="cuda")
            c1 = clock()
            splan.execute_source(i, buf.data_ptr(), ptrs(dst), h)
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
        t1 = time.perf_counter()
        sst = splan.mem_stats()
        streaming = {"total_ms": round((t1 - t0) * 1e3, 2), "ledger_peak_device": sst["peak_device"],
                     "torch_peak_allocated": torch.cuda.max_memory_allocated(), "dst_bytes": sst["dst_live"],
                     "largest_src_buffer": max(n for n, u in zip(sizes_s, used_s) if u), "buffers_in_flight": 2,
                     "host_ms": {k: round(v, 1) for k, v in host_ms.items()}, "state": sst["state"],
                     "one_shot_peak_device": plan.mem_stats()["peak_device"], "allocated_before": base}
        src = alloc_src(False)  # a device home again, and the weights back, so the rest of the run goes on
        splan.bind_src(ptrs(src))
        splan.swap_in(h)
        splan.swap_wait()
        splan.release_host()

    moved = info["bytes_moved"]
    k_avg = sum(kernel_ms) / len(kernel_ms) / 1e3
    repack_gbps = 2 * moved / k_avg / 1e9
    stats = plan.mem_stats()
    peak_torch = torch.cuda.max_memory_allocated()

    # plain copy of the same byte count class, same load/store code: the ceiling next to it
    big_s = max((s for s in src if s is not None), key=lambda t: t.numel())
    big_d = max((d for d in dst if d is not None), key=lambda t: t.numel())
    cp_n = min(big_s.numel() * 2, big_d.numel() * 2, 8 << 30) // 4096 * 4096
    evs = []
    for _ in range(6):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        copy_baseline(big_d.data_ptr(), big_s.data_ptr(), cp_n, h)
        e1.record(stream)
        evs.append((e0, e1))
    torch.cuda.synchronize()
    plain_gbps = 2 * cp_n / (min(x.elapsed_time(y) for x, y in evs[1:]) / 1e3) / 1e9
    # one-way rates of the same buffers with the same tile shape: a copy moves equal bytes both ways
    # over the same memory, so 2 / (1/R + 1/W) bounds it (the destination is rewritten by every repack)
    one_way = {}
    pr_n = cp_n // 32768 * 32768
    for key, fn in (("read", lambda: read_baseline(big_s.data_ptr(), pr_n, h)), ("write", lambda: write_baseline(big_d.data_ptr(), pr_n, h))):
        evs = []
        for _ in range(6):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            fn()
            e1.record(stream)
            evs.append((e0, e1))
        torch.cuda.synchronize()
        one_way[key] = pr_n / (min(x.elapsed_time(y) for x, y in evs[1:]) / 1e3) / 1e9
    mixed_bound = 2.0 / (1.0 / one_way["read"] + 1.0 / one_way["write"])

    traffic, traffic_detail = None, None
    tpath = os.path.join(ROOT, "profiles", "repack_hbm_traffic.json")  # from rocprofv3 --pmc runs
    if os.path.exists(tpath):
        traffic_detail = json.load(open(tpath)).get(a.workload)
        if traffic_detail:
            traffic = traffic_detail["total_bytes"]  # HBM bytes per execute, fetch + write, counter-based

    link = None if a.no_link_probe or a.no_swap else link_probe()
    out = {
        "metric": "reshard repack GB/s (read+write)",
        "value": round(repack_gbps, 1),
        "unit": "GB/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": round(total_s / a.steps * 1e3, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u16", "data": "synthetic",
        "config": {"workload": "%s: %s" % (wl["name"], wl["note"]), "bytes_moved_one_way": moved,
                   "src_buffers": sum(used_s), "dst_buffers": sum(used_d),
                   "descriptors": info["num_descs"], "tiles": info["num_tiles"], "tuning": get_tuning(),
                   "swap_overlaps_repack": bool(a.overlap and not a.no_swap)},
        "roofline": {"bound": "hbm", "achieved": round(repack_gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(repack_gbps / HBM_PEAK_GBPS, 4), "traffic": traffic,
                     "algorithmic_bytes": 2 * moved, "traffic_detail": traffic_detail,
                     "kernel_ms_avg": round(k_avg * 1e3, 4), "kernel_ms_min": round(min(kernel_ms), 4),
                     "plain_copy_GBps": round(plain_gbps, 1), "read_only_GBps": round(one_way["read"], 1),
                     "write_only_GBps": round(one_way["write"], 1), "mixed_bound_GBps": round(mixed_bound, 1),
                     "frac_of_mixed_bound": round(2 * moved / k_avg / 1e9 / mixed_bound, 4)},
        "pct_hbm_peak": round(100 * repack_gbps / HBM_PEAK_GBPS, 2),
        "peak_hbm_bytes": {"ledger": stats["peak_device"], "torch_max_allocated": peak_torch,
                           "freed_after_swap_out": (sum(freed) // len(freed)) if freed else None,
                           "returned_to_driver_after_swap_out": driver_freed},
    }
    if not a.no_swap:
        so, si = sum(out_s) / len(out_s), sum(in_s) / len(in_s)
        out["swap"] = {"bytes_each_way": src_bytes, "out_GBps": round(src_bytes / so / 1e9, 2),
                       "in_GBps": round(src_bytes / si / 1e9, 2),
                       "in_first_buffer_ms": round(sum(first_s) / len(first_s) * 1e3, 2), "in_all_buffers_ms": round(si * 1e3, 2),
                       "link_probe_GBps": None if link is None else {k: round(v, 2) for k, v in link.items()}}
        if link:
            out["swap"]["out_frac_of_link"] = round(src_bytes / so / 1e9 / link["d2h"], 3)
            out["swap"]["in_frac_of_link"] = round(src_bytes / si / 1e9 / link["h2d"], 3)
    if streaming:
        out["streaming"] = streaming
    if framework:
        out["framework_baseline"] = framework
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, plan, src)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
