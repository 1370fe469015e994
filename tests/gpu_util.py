"""Helpers for the GPU parity tests: seeded device buffers, oracle runs on the host."""

from __future__ import annotations

import numpy as np
import torch

from oracle import fast
from synth_inputs import BF16_ONE, fill_buffer

SENT16 = -23131  # 0xA5A5 as int16


def stream_handle() -> int:
    return torch.cuda.current_stream().cuda_stream


def device_sources(plan, wl, mode="normal", device="cuda"):
    """One int16 device tensor per used source buffer (None otherwise), seeded fill,
    norm vectors overwritten with bf16 ones (normal mode only)."""
    sizes, used = plan.buf_bytes(0), plan.buf_used(0)
    bufs = [fill_buffer(n, wl["seed"] * 1000 + i, device, mode) if u else None
            for i, (n, u) in enumerate(zip(sizes, used))]
    if mode == "normal" and wl["spec"]["elem_bytes"] == 2:
        for t in plan.tensors(0):
            if t["name"].endswith("ln") or t["name"] in ("ln1", "ln2"):
                b = bufs[t["buffer"]]
                if b is not None:
                    b[t["offset"] // 2:(t["offset"] + t["bytes"]) // 2] = BF16_ONE
    return bufs


def device_destinations(plan, device="cuda"):
    sizes, used = plan.buf_bytes(1), plan.buf_used(1)
    return [torch.full((n // 2,), SENT16, dtype=torch.int16, device=device) if u else None
            for n, u in zip(sizes, used)]


def ptrs(bufs):
    return [0 if b is None else b.data_ptr() for b in bufs]


def oracle_destinations(wl, src_host, threads=16, dst_lay=None, src_lay=None):
    """Loop oracle on host copies of the sources, from sentinel-filled destinations."""
    spec = wl["spec"]
    dst_lay = dst_lay or wl["dst"]
    src_lay = src_lay or wl["src"]
    sizes = fast.buffer_sizes(spec, dst_lay)
    used = fast.buffers_used(spec, dst_lay)
    dst = [np.full(n // 2, SENT16, dtype=np.int16) if u else None for n, u in zip(sizes, used)]
    fast.reshard(spec, src_lay, dst_lay, src_host, dst, threads=threads)
    return dst


def host_copy_view(plan, index):
    """The plan's pinned host copy of one source buffer as an int16 numpy array (no copy)."""
    import ctypes

    n = plan.buf_bytes(0)[index] // 2
    raw = (ctypes.c_int16 * n).from_address(plan.host_copy(index))
    return np.frombuffer(raw, dtype=np.int16)


def to_host(bufs):
    return [None if b is None else b.cpu().numpy() for b in bufs]


def assert_equal_buffers(got_dev, want_host, what=""):
    for i, (g, w) in enumerate(zip(got_dev, want_host)):
        if w is None:
            assert g is None
            continue
        gh = g.cpu().numpy()
        if not np.array_equal(gh, w):
            bad = np.flatnonzero(gh != w)
            raise AssertionError(f"{what} buffer {i}: {bad.size} words differ, first at word {bad[0]}")


def gather_check(src_dev, dst_dev, pairs, eb=2):
    """Compare sampled (source element, destination element) pairs on the device."""
    sb, so, db, do = pairs
    bad = 0
    for a in np.unique(sb):
        for b in np.unique(db[sb == a]):
            m = (sb == a) & (db == b)
            si = torch.from_numpy(so[m] // eb).to(src_dev[a].device)
            di = torch.from_numpy(do[m] // eb).to(src_dev[a].device)
            bad += int((src_dev[a][si] != dst_dev[b][di]).sum())
    return bad
