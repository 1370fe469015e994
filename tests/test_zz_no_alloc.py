"""The entry point that allocates nothing (reshard_execute_noalloc: the tile table lives in a
static device array shared by every plan on the GPU) against reshard_execute, bit for bit."""

import numpy as np
import pytest
import torch

import gpu_util as G
from paper_2507_19017_amd import Plan, ReshardError, binding
from synth_inputs import TINY, WORKLOADS, random_case

pytestmark = pytest.mark.gpu


def both_ways(plan, wl, seed_shift=0):
    """Destinations of the static-array entry point and of the ordinary one on the same inputs
    (sentinel-filled first, so untouched gaps count too), plus the oracle's."""
    w = dict(wl, seed=wl["seed"] + seed_shift)
    src = G.device_sources(plan, w, "raw16")
    a, b = G.device_destinations(plan), G.device_destinations(plan)
    h = G.stream_handle()
    allocated = torch.cuda.memory_allocated()
    plan.execute_noalloc(G.ptrs(src), G.ptrs(a), h)
    assert torch.cuda.memory_allocated() == allocated
    plan.execute(G.ptrs(src), G.ptrs(b), h)
    torch.cuda.synchronize()
    for x, y in zip(a, b):
        assert (x is None and y is None) or torch.equal(x, y)
    G.assert_equal_buffers(a, G.oracle_destinations(w, G.to_host(src), 4), wl["name"])


def test_static_table_entry_point_matches_execute_on_calls_in_a_row():
    """Two calls in a row, the second on a smaller plan (its table replaces the start of the larger
    one's in the shared array), then the first plan again (its table has to come back) and once more
    (now launches only); every result equals reshard_execute's and the oracle's."""
    big_wl, small_wl = random_case(5, 16), TINY["mid_moe_grouped"]
    print("case no-alloc", big_wl["name"], "then", small_wl["name"], flush=True)
    big = Plan(big_wl["spec"], big_wl["src"], big_wl["dst"], tuning=dict(tile_bytes=4096))
    small = Plan(small_wl["spec"], small_wl["src"], small_wl["dst"])
    assert big.info()["num_tiles"] > 4 * small.info()["num_tiles"] > 0
    assert big.info()["table_bytes"] <= 32 << 20
    both_ways(big, big_wl)
    both_ways(small, small_wl)
    both_ways(big, big_wl, 1)
    both_ways(big, big_wl, 2)
    both_ways(small, small_wl, 3)


def test_static_table_entry_point_at_c0_and_full_c1_size():
    for name in ("C0", "C1"):
        wl = WORKLOADS[name]
        print("case no-alloc", name, flush=True)
        plan = Plan(wl["spec"], wl["src"], wl["dst"])
        src = G.device_sources(plan, wl, "raw16")
        a, b = G.device_destinations(plan), G.device_destinations(plan)
        plan.execute_noalloc(G.ptrs(src), G.ptrs(a), G.stream_handle())
        plan.execute(G.ptrs(src), G.ptrs(b), G.stream_handle())
        torch.cuda.synchronize()
        for x, y in zip(a, b):
            assert torch.equal(x, y)
        assert plan.mem_stats()["state"] == "resident"


def test_a_table_beyond_the_static_array_is_refused_with_a_clear_error():
    wl = WORKLOADS["C1"]
    plan = Plan(wl["spec"], wl["src"], wl["dst"], tuning=dict(tile_bytes=16384))  # twice the tiles: 46 MB of table
    assert plan.info()["table_bytes"] > 32 << 20
    src = G.device_sources(plan, wl, "raw16")
    dst = G.device_destinations(plan)
    with pytest.raises(ReshardError) as e:
        plan.execute_noalloc(G.ptrs(src), G.ptrs(dst), G.stream_handle())
    assert e.value.code == binding.ERR_UNSUPPORTED and "static device array" in str(e.value)
    assert plan.mem_stats()["state"] == "unbound"
    torch.cuda.synchronize()
    assert all(bool((d == G.SENT16).all()) for d in dst)  # nothing was launched
