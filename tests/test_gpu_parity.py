"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle,
bit for bit, on the same seeded inputs."""

import numpy as np
import pytest
import torch

import gpu_util as G
from oracle import fast, locate
from paper_2507_19017_amd import Plan, ReshardError, binding, copy_baseline, read_baseline, set_tuning, write_baseline
from synth_inputs import MID, TINY, WORKLOADS, fill_buffer, make_layout, make_spec, random_case

pytestmark = pytest.mark.gpu


def with_eb(wl, eb):
    w = dict(wl)
    w["spec"] = dict(wl["spec"], elem_bytes=eb)
    return w


def run_case(wl, mode="normal", src_lay=None, dst_lay=None, threads=16, via_swap=False, tuning=None):
    src_lay = src_lay or wl["src"]
    dst_lay = dst_lay or wl["dst"]
    plan = Plan(wl["spec"], src_lay, dst_lay, tuning=tuning)
    src = G.device_sources(plan, wl, mode)
    dst = G.device_destinations(plan)
    plan.execute(G.ptrs(src), G.ptrs(dst), G.stream_handle())
    torch.cuda.synchronize()
    if via_swap:
        # the oracle reads the library's own pinned swap copies (a 57 GB/s copy instead of a pageable
        # one), which also holds the swap-out to the same bar: a wrong byte there shows in the result
        plan.swap_out(G.stream_handle())
        plan.swap_wait()
        host_src = [None if s is None else G.host_copy_view(plan, i) for i, s in enumerate(src)]
    else:
        host_src = [None if s is None else s.cpu().numpy() for s in src]
    # the oracle needs every source buffer it reads; unused ones may stay None
    want = G.oracle_destinations(wl, host_src, threads, dst_lay, src_lay)
    G.assert_equal_buffers(dst, want, wl["name"])
    return plan, src, dst


@pytest.mark.parametrize("eb", [2, 1, 4, 8])
@pytest.mark.parametrize("name", sorted(TINY))
def test_tiny_models_all_element_sizes(name, eb):
    print("case", name, eb, flush=True)
    run_case(with_eb(TINY[name], eb), mode="raw16")


@pytest.mark.parametrize("first", range(0, 160, 20))
def test_random_small_workloads(first):
    """Random shapes, degrees and layout options (the cases the CPU tests hold against the
    numpy constructions), twenty per test."""
    for seed in range(first, first + 20):
        print("case random", seed, flush=True)
        run_case(random_case(seed), mode="raw16", threads=2)


@pytest.mark.parametrize("first", range(0, 64, 16))
def test_random_midsize_workloads(first):
    """The random generator with widths scaled by 16: tensors of many tiles with ragged ends,
    3 MB to 1 GB per case, every element size, transposing descriptors on the register path."""
    for seed in range(first, first + 16):
        print("case random x16", seed, flush=True)
        run_case(random_case(seed, 16), mode="raw16", threads=8)


@pytest.mark.parametrize("mode", ["normal", "raw16"])
def test_toy_config_c0(mode):
    print("case C0", mode, flush=True)
    run_case(WORKLOADS["C0"], mode)


@pytest.mark.parametrize("name", sorted(TINY) + ["C0"])
def test_identity_and_round_trip_on_device(name):
    print("case", name, flush=True)
    wl = {**TINY, **WORKLOADS}[name]
    train = wl["src"]
    gen = dict(wl["dst"], tp_filter=-1, ep_filter=-1)
    # identity: equal layouts copy every stored tensor in place
    run_case(wl, "raw16", train, train)
    # train -> gen -> train returns the input bit for bit when replicas agree
    p1 = Plan(wl["spec"], train, gen)
    p2 = Plan(wl["spec"], gen, train)
    src = G.device_sources(p1, wl, "raw16")
    # make replicas agree: run the identity first so rank 0's common weights reach every rank
    p0 = Plan(wl["spec"], train, train)
    src_eq = G.device_destinations(p0)
    p0.execute(G.ptrs(src), G.ptrs(src_eq), G.stream_handle())
    mid = G.device_destinations(p1)
    p1.execute(G.ptrs(src_eq), G.ptrs(mid), G.stream_handle())
    back = G.device_destinations(p2)
    p2.execute(G.ptrs(mid), G.ptrs(back), G.stream_handle())
    torch.cuda.synchronize()
    for a, b in zip(src_eq, back):
        assert torch.equal(a, b)


TUNINGS = [
    dict(tile_bytes=4096, block_threads=64, unroll=1, flags=-1),
    dict(tile_bytes=8192, block_threads=128, unroll=2, flags=1),
    dict(tile_bytes=32768, block_threads=512, unroll=2, flags=2),
    dict(tile_bytes=16384, block_threads=256, unroll=2, flags=4),
    dict(tile_bytes=16384, block_threads=256, unroll=2, flags=5),
    dict(tile_bytes=16384, block_threads=1024, unroll=2, flags=6),
    dict(tile_bytes=524288, block_threads=1024, unroll=4, blocks_per_cu=1),
    dict(tile_bytes=65536, block_threads=256, unroll=8, blocks_per_cu=16, flags=7),
    dict(tile_bytes=65536, block_threads=1024, unroll=2, blocks_per_cu=2, flags=4),
    dict(tile_bytes=131072, block_threads=1024, unroll=8, flags=7),
    dict(tile_bytes=262144, block_threads=1024, unroll=2, flags=11),
    dict(tile_bytes=65536, block_threads=1024, unroll=8, flags=31),
    dict(tile_bytes=32768, block_threads=1024, unroll=2, flags=23),
    dict(tile_bytes=32768, block_threads=1024, unroll=2, flags=27),
    dict(tile_bytes=32768, block_threads=1024, unroll=2, flags=28),
    dict(tile_bytes=16384, block_threads=1024, unroll=1, flags=31),
    dict(tile_bytes=65536, block_threads=1024, unroll=4, flags=15),
    dict(tile_bytes=4096, block_threads=256, unroll=2, flags=8),
    dict(tile_bytes=4096, flags=31, tail_pool_percent=25, tail_chunk_tiles=3),   # the shared tail pool: ragged last chunks
    dict(tile_bytes=8192, flags=31, tail_pool_percent=50, tail_chunk_tiles=1),
    dict(flags=31, tail_pool_percent=10),
    dict(flags=63),                                         # the woven order (XCDs share every group of 8 tiles)
    dict(flags=127, tile_bytes=16384),                      # with gathered tiles where the plan has them
    dict(flags=36, tile_bytes=4096),
    dict(flags=35, tile_bytes=131072),
    dict(flags=39, tile_bytes=8192),
]


@pytest.mark.parametrize("tuning", TUNINGS)
def test_every_launch_shape_gives_the_same_bits(tuning):
    print("tuning", tuning, flush=True)
    for name in ("tiny_dense", "tiny_moe_grouped"):
        run_case(TINY[name], "raw16", tuning=tuning)
    run_case(WORKLOADS["C0"], "raw16", tuning=tuning)


GATHER_TUNINGS = [None, dict(flags=127, tile_bytes=4096), dict(flags=100, tile_bytes=8192), dict(flags=99, tile_bytes=131072),
                  dict(flags=103, tile_bytes=524288), dict(flags=63), dict(flags=31), dict(flags=95), dict(flags=127, block_threads=512),
                  dict(flags=127, blocks_per_cu=2)]


@pytest.mark.parametrize("name", sorted(MID))
def test_side_by_side_merges_as_gathered_tiles(name):
    """Row-parallel shards with rows of 64 and 88 vectors, merged 2, 4 and 8 abreast or packed out
    of a wider source: in the woven order these bytes go out as gathered tiles (one contiguous
    stream of the destination fed by the sources in turn), in every other launch shape as row
    blocks.  Every shape gives the oracle's bits, so does the one-source-at-a-time path (row
    blocks only) and the entry point that reads the table from the static array; and the counting
    build shows every byte written exactly once in the woven order."""
    wl = MID[name]
    for tuning in GATHER_TUNINGS:
        print("case", name, tuning, flush=True)
        plan, src, dst = run_case(wl, "raw16", tuning=tuning)
        if tuning is None:
            assert plan.get_tuning()["flags"] == 127
            tiles = plan.tiles()
            assert any(t["kind"] == 2 for t in tiles) and any(t["order"] == 1 for t in tiles)
            again = G.device_destinations(plan)
            plan.execute_noalloc(G.ptrs(src), G.ptrs(again), G.stream_handle())
            torch.cuda.synchronize()
            for a, b in zip(dst, again):
                assert (a is None and b is None) or torch.equal(a, b)
            by_source = G.device_destinations(plan)
            for i, buf in enumerate(src):
                if buf is not None:
                    plan.execute_source(i, buf.data_ptr(), G.ptrs(by_source), G.stream_handle())
            torch.cuda.synchronize()
            for a, b in zip(dst, by_source):
                assert (a is None and b is None) or torch.equal(a, b)
            # the same plan switched between its two forms from one execute to the next
            for flags in (63, 127, 31, 127):
                plan.set_tuning(flags=flags)
                other = G.device_destinations(plan)
                plan.execute(G.ptrs(src), G.ptrs(other), G.stream_handle())
                torch.cuda.synchronize()
                for a, b in zip(dst, other):
                    assert (a is None and b is None) or torch.equal(a, b), flags
    for tuning in (None, dict(flags=127, tile_bytes=4096)):
        counts, D = _count_writes_on_device(wl, tuning)
        for b, c in enumerate(counts):
            if c is None:
                continue
            want = np.zeros(D.buf_bytes[b], dtype=np.uint8)
            for off, nb in D.owned(b):
                want[off:off + nb] = 1
            assert np.array_equal(c, want), f"{name} buffer {b}: {int((c != want).sum())} bytes not written exactly once"


def test_successive_executes_rotate_through_the_copies_of_the_tile_table():
    """A plan keeps several copies of its tile table on the device and every execute reads the next
    one (so that the records are not still in the memory-side cache from the execute before).  Every
    copy gives the oracle's bits; the count is what the tuning says, or chosen from the table size
    (one for a small table), and is fixed once the table is on the device."""
    wl = MID["mid_merge2"]
    plan, src, dst = run_case(wl, "raw16", tuning=dict(table_copies=3))
    assert plan.get_tuning()["table_copies"] == 3
    plan.set_tuning(table_copies=7, flags=127)  # the launch shape changes, the copies stay
    assert plan.get_tuning()["table_copies"] == 3 and plan.get_tuning()["flags"] == 127
    for n in range(7):
        again = G.device_destinations(plan)
        plan.execute(G.ptrs(src), G.ptrs(again), G.stream_handle())
        torch.cuda.synchronize()
        for a, b in zip(dst, again):
            assert (a is None and b is None) or torch.equal(a, b), n
    small = Plan(WORKLOADS["C0"]["spec"], WORKLOADS["C0"]["src"], WORKLOADS["C0"]["dst"])
    assert small.get_tuning()["table_copies"] == 0
    small.prepare()
    assert small.get_tuning()["table_copies"] == 1
    big = Plan(WORKLOADS["C1"]["spec"], WORKLOADS["C1"]["src"], WORKLOADS["C1"]["dst"])
    big.prepare()  # 29.9 MB of table: 18 copies make 512 MiB
    assert big.get_tuning()["table_copies"] == 18
    before = torch.cuda.mem_get_info()[0]
    big.destroy()
    assert torch.cuda.mem_get_info()[0] - before >= 18 * big_table_bytes(wl=WORKLOADS["C1"]) - (64 << 20)


def big_table_bytes(wl):
    return Plan(wl["spec"], wl["src"], wl["dst"]).info()["table_bytes"]


def test_two_plans_with_different_tunings_interleave():
    """Tuning belongs to the plan: two plans of one workload cut into different tile sizes and launched
    with different shapes run alternately on one stream, one of them changes its launch shape in
    between, and every result equals the oracle's."""
    wl = WORKLOADS["C0"]
    print("case two tunings", flush=True)
    small = Plan(wl["spec"], wl["src"], wl["dst"], tuning=dict(tile_bytes=4096, unroll=1, block_threads=256, flags=7))
    big = Plan(wl["spec"], wl["src"], wl["dst"], tuning=dict(tile_bytes=131072, unroll=8))
    assert small.info()["num_tiles"] > 8 * big.info()["num_tiles"]
    src = G.device_sources(small, wl, "raw16")
    want = G.oracle_destinations(wl, G.to_host(src), 4)
    h = G.stream_handle()
    outs = []
    for round_ in range(3):
        for plan in (small, big):
            dst = G.device_destinations(plan)
            plan.execute(G.ptrs(src), G.ptrs(dst), h)
            outs.append(dst)
        small.set_tuning(unroll=2, flags=(23, 31)[round_ % 2], blocks_per_cu=round_)
        assert small.get_tuning()["tile_bytes"] == 4096 and big.get_tuning()["tile_bytes"] == 131072
    torch.cuda.synchronize()
    for dst in outs:
        G.assert_equal_buffers(dst, want, "two tunings")


def _transpose_shapes():
    """Every (element size, tile shape) the register-transpose kernel is built for."""
    out = []
    for eb in (2, 1, 4, 8):
        for ti in (64, 128, 256, 512):
            for tk in (64, 128, 256, 512):
                fits = ti * tk * eb <= 131072
                if fits and ((ti >= 128 and tk >= 128) if eb == 1 else max(ti, tk) <= 256):
                    out.append((eb, ti, tk))
    return out + [(2, 256, 192), (2, 192, 256), (2, 192, 192)]


@pytest.mark.parametrize("eb,ti,tk", _transpose_shapes())
def test_register_transpose_tile_shapes(eb, ti, tk):
    """Grouped (transposing) experts at sizes with full tiles and ragged edges, every element size
    and tile shape; plus a shape whose expert dimensions are exact multiples of every tile shape."""
    print("transpose shape", eb, ti, tk, flush=True)
    exact = dict(TINY["mid_moe_grouped"])
    exact["spec"] = dict(exact["spec"], H=512, Ie=256)
    shape = dict(transpose_rows=ti, transpose_cols=tk)
    for wl in (TINY["mid_moe_grouped"], TINY["big_moe_grouped"], exact):
        wl = with_eb(wl, eb)
        plan, _, _ = run_case(wl, "raw16", tuning=shape)
        # way back: generation [out][in] -> grouped [in][out] is a transpose as well
        gen = dict(wl["dst"])
        run_case(wl, "raw16", gen, wl["src"], tuning=shape)
        classes = {t["tile_class"] for t in plan.tiles()}
        if wl["name"] == "big_moe_grouped":
            assert 1 in classes and 3 in classes, "full tiles and ragged strips both present"
    assert plan.info()["num_transpose_tiles"] > 0


DEGENERATE = [
    # the smallest model the shape rules allow: one head, one layer, 16-byte rows, nothing to split
    ("one_head", make_spec(family="dense_gqa", L=1, H=8, nq=1, nkv=1, d=8, I=8, V=8),
     make_layout(kind="train"), make_layout(kind="gen")),
    # no embeddings at all and a single stage on both sides: only the fused-QKV permutation moves data
    ("qkv_only_moves", make_spec(family="dense_gqa", L=3, H=64, nq=8, nkv=4, d=8, I=32, V=0, has_embeddings=0),
     make_layout(kind="train", tp=1), make_layout(kind="gen", tp=1)),
    # generation -> generation with equal degrees: a pure copy, pads skipped
    ("gen_identity", make_spec(family="moe_gqa", L=2, H=32, nq=4, nkv=2, d=8, V=48, E=4, Ie=24, n_shared=1),
     make_layout(kind="gen", tp=2, ep=2), make_layout(kind="gen", tp=2, ep=2)),
    # a destination filter that keeps one dense rank and one expert rank of many
    ("one_rank_of_each", make_spec(family="moe_gqa", L=2, H=32, nq=4, nkv=4, d=8, V=64, E=8, Ie=16),
     make_layout(kind="train", tp=2, pp=2, ep=4), make_layout(kind="gen", tp=4, ep=8, tp_filter=3, ep_filter=5)),
    # odd byte counts: 1-byte elements and widths that are not multiples of anything
    ("odd_bytes", make_spec(family="dense_gqa", L=2, H=7, nq=3, nkv=3, d=5, I=9, V=6, qkv_bias=1, elem_bytes=1),
     make_layout(kind="train", tp=3), make_layout(kind="gen", tp=1)),
]


@pytest.mark.parametrize("case", DEGENERATE, ids=[c[0] for c in DEGENERATE])
def test_degenerate_and_ragged_shapes(case):
    """Edge shapes: nothing to split, a pure copy, single-rank filters, 1-byte ragged rows.
    (An empty plan does not exist: every valid model has at least one layer.)"""
    name, spec, src, dst = case
    print("degenerate", name, flush=True)
    wl = dict(name=name, spec=spec, src=src, dst=dst, seed=4000)
    plan, s, d = run_case(wl, "raw16")
    assert plan.info()["bytes_moved"] > 0


def _count_writes_on_device(wl, tuning=None):
    """Runs the plan's real kernels from the counting build on zeroed shadow destinations and
    returns (per-byte write counts, the definition oracle's layout of the destination)."""
    import contextlib

    from paper_2507_19017_amd.build import COUNT_LIB

    @contextlib.contextmanager
    def counting_library():
        keep = (binding._lib, binding._LIB_PATH)
        binding._lib, binding._LIB_PATH = None, COUNT_LIB
        try:
            yield
        finally:
            binding._lib, binding._LIB_PATH = keep

    with counting_library():
        plan = Plan(wl["spec"], wl["src"], wl["dst"], tuning=tuning)
        try:
            src = G.device_sources(plan, wl, "raw16")
            shadow = [torch.zeros(n // 2, dtype=torch.int16, device="cuda") if u else None
                      for n, u in zip(plan.buf_bytes(1), plan.buf_used(1))]
            plan.execute(G.ptrs(src), G.ptrs(shadow), G.stream_handle())
            torch.cuda.synchronize()
            counts = [None if s_ is None else s_.cpu().numpy().view(np.uint8) for s_ in shadow]
        finally:
            plan.destroy()  # by the library that made it
    return counts, locate.Layout(wl["spec"], wl["dst"])


@pytest.mark.parametrize("name", sorted(TINY) + ["C0"])
def test_every_destination_byte_is_written_exactly_once_on_the_device(name):
    """The kernels themselves, built with counting stores: every byte of every stored destination
    tensor is written exactly once by the device code, and no byte of a gap or of vocabulary padding
    is written at all.  Checked for the default tuning and for small tiles with the shared tail pool."""
    wl = {**TINY, **WORKLOADS}[name]
    print("case exactly once", name, flush=True)
    for tuning in (None, dict(tile_bytes=4096, transpose_rows=64, transpose_cols=64, flags=31, tail_pool_percent=20, tail_chunk_tiles=2)):
        counts, D = _count_writes_on_device(wl, tuning)
        for b, c in enumerate(counts):
            if c is None:
                continue
            want = np.zeros(D.buf_bytes[b], dtype=np.uint8)
            for off, nb in D.owned(b):
                want[off:off + nb] = 1
            assert np.array_equal(c, want), f"{name} buffer {b}: {int((c != want).sum())} bytes not written exactly once"


def test_exactly_once_on_the_device_for_random_midsize_workloads():
    """The same check on the random generator's workloads with widths scaled by 16 (every element
    size, ragged ends, transposing tiles of several shapes)."""
    for seed in range(0, 24):
        wl = random_case(seed, 16)
        print("case exactly once random x16", seed, flush=True)
        counts, D = _count_writes_on_device(wl)
        for b, c in enumerate(counts):
            if c is None:
                continue
            want = np.zeros(D.buf_bytes[b], dtype=np.uint8)
            for off, nb in D.owned(b):
                want[off:off + nb] = 1
            assert np.array_equal(c, want), f"seed {seed} buffer {b}"


def test_copy_baseline_matches_memcpy():
    n = 64 * 1024 * 1024 + 4096 + 16
    a = fill_buffer(n, 7, "cuda", "raw16")
    b = torch.zeros_like(a)
    copy_baseline(b.data_ptr(), a.data_ptr(), n, G.stream_handle())
    torch.cuda.synchronize()
    assert torch.equal(a, b)
    with pytest.raises(ReshardError):
        copy_baseline(b.data_ptr() + 2, a.data_ptr(), 32)


def test_unused_source_buffers_may_be_null_and_are_never_read():
    wl = TINY["tiny_mla"]
    plan, src, dst = run_case(wl, "raw16")
    assert src.count(None) == 4 and dst.count(None) == 1


def test_execute_on_a_side_stream_and_inside_a_hip_graph():
    """After prepare() an execute is launches only, so it can run on any stream and be
    recorded into a graph; each replay is compared with an eager run on fresh inputs."""
    wl = TINY["mid_moe_grouped"]
    plan = Plan(wl["spec"], wl["src"], wl["dst"])
    plan.prepare()
    src = G.device_sources(plan, wl, "raw16")
    dst = G.device_destinations(plan)
    eager = G.device_destinations(plan)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        plan.execute(G.ptrs(src), G.ptrs(eager), side.cuda_stream)
    side.synchronize()
    want = G.oracle_destinations(wl, G.to_host(src), 4)
    G.assert_equal_buffers(eager, want, "side stream")
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        plan.execute(G.ptrs(src), G.ptrs(dst), torch.cuda.current_stream().cuda_stream)
    for replay in range(3):
        for i, s_ in enumerate(src):  # new contents in the same buffers
            s_.copy_(fill_buffer(s_.numel() * 2, 77 + 10 * replay + i, "cuda", "raw16"))
        for d_ in dst:
            d_.fill_(G.SENT16)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        plan.execute(G.ptrs(src), G.ptrs(eager), G.stream_handle())
        torch.cuda.synchronize()
        for a, b in zip(dst, eager):
            assert torch.equal(a, b), f"replay {replay}"
        G.assert_equal_buffers(dst, G.oracle_destinations(wl, G.to_host(src), 4), f"replay {replay}")


def test_one_way_bandwidth_probes():
    """The read probe leaves its buffer alone, the write probe fills exactly the bytes it was given
    (each 16-byte unit holds its tile, its lane, a constant and the tile's complement), and both
    refuse sizes that are not whole tiles."""
    n = 5 * 32768
    buf = torch.arange(n // 2 + 64, dtype=torch.int16, device="cuda")
    keep = buf.clone()
    read_baseline(buf.data_ptr(), n, G.stream_handle())
    torch.cuda.synchronize()
    assert torch.equal(buf, keep)
    write_baseline(buf.data_ptr(), n, G.stream_handle())
    torch.cuda.synchronize()
    got = buf[:n // 2].view(torch.int32).view(-1, 4).cpu().numpy().view(np.uint32).reshape(5, 2, 1024, 4)
    tile = np.arange(5, dtype=np.uint32)[:, None, None]
    lane = np.arange(1024, dtype=np.uint32)[None, None, :]
    assert np.array_equal(got[..., 0], np.broadcast_to(tile, (5, 2, 1024)))
    assert np.array_equal(got[..., 1], np.broadcast_to(lane, (5, 2, 1024)))
    assert np.all(got[..., 2] == 0x9E3779B9) and np.array_equal(got[..., 3], np.broadcast_to(~tile, (5, 2, 1024)))
    assert torch.equal(buf[n // 2:], keep[n // 2:])  # nothing past the end
    for bad in (n + 16, 0):
        with pytest.raises(ReshardError):
            write_baseline(buf.data_ptr(), bad, G.stream_handle())
        with pytest.raises(ReshardError):
            read_baseline(buf.data_ptr(), bad, G.stream_handle())


def test_a_plain_c_program_drives_the_library_on_the_gpu(tmp_path):
    """No Python and no tensor framework in the client: a C99 program allocates device memory with
    the HIP runtime, reshards the toy workload, swaps the sources out, frees them, allocates new
    ones and swaps back in.  Its destination buffer must equal the oracle's on the same inputs and
    the sources must return bit for bit."""
    import os
    import subprocess

    exe = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c_abi_gpu_client")
    assert os.path.exists(exe), "tests/c_abi_gpu_client is missing: run __graft_entry__.build() first"
    out = str(tmp_path / "c_client.bin")
    res = subprocess.run([exe, out], capture_output=True, text=True, timeout=120)
    assert res.returncode == 0, res.stdout + res.stderr
    wl = WORKLOADS["C0"]
    sizes_s, sizes_d = fast.buffer_sizes(wl["spec"], wl["src"]), fast.buffer_sizes(wl["spec"], wl["dst"])
    assert res.stdout.split() == ["ok", str(sizes_d[0]), str(sizes_s[0]), str(sizes_s[1])]
    src = [(((np.arange(n // 2, dtype=np.uint64) * np.uint64(2654435761) + np.uint64(b * 40503)) >> np.uint64(9))
            & np.uint64(0xFFFF)).astype(np.uint16).view(np.int16) for b, n in enumerate(sizes_s)]
    want = [np.full(sizes_d[0] // 2, G.SENT16, dtype=np.int16)]
    fast.reshard(wl["spec"], wl["src"], wl["dst"], src, want, threads=2)
    got = np.fromfile(out, dtype=np.int16)
    nd = sizes_d[0] // 2
    assert got.size == nd + sum(sizes_s) // 2
    assert np.array_equal(got[:nd], want[0])
    assert np.array_equal(got[nd:nd + sizes_s[0] // 2], src[0]) and np.array_equal(got[nd + sizes_s[0] // 2:], src[1])


# ------------------------------------------------------------- streaming ----
@pytest.mark.parametrize("name", sorted(TINY) + ["C0"])
def test_streaming_one_source_buffer_at_a_time(name):
    """The gathered shards arrive one buffer at a time, are repacked, swapped out and dropped:
    the destination equals the oracle's, only one source buffer is ever live, and the swapped
    copies come back bit for bit."""
    wl = {**TINY, **WORKLOADS}[name]
    print("streaming", name, flush=True)
    plan = Plan(wl["spec"], wl["src"], wl["dst"])
    sizes, used = plan.buf_bytes(0), plan.buf_used(0)
    dst = G.device_destinations(plan)
    h = G.stream_handle()
    keep = {}
    order = [i for i, u in enumerate(used) if u][::-1]  # any order works; take the last buffer first
    for n, i in enumerate(order):
        buf = fill_buffer(sizes[i], wl["seed"] * 1000 + i, "cuda", "raw16")  # this buffer "arrives"
        keep[i] = buf.cpu().numpy()
        plan.execute_source(i, buf.data_ptr(), G.ptrs(dst), h)
        assert plan.src_buffer_state(i) == "resident"
        assert plan.mem_stats()["src_live"] == sizes[i]
        plan.swap_out_source(i, h)
        with pytest.raises(ReshardError) as e:
            plan.execute_source(i, buf.data_ptr(), G.ptrs(dst), h)
        assert e.value.code == binding.ERR_BAD_STATE
        with pytest.raises(ReshardError) as e:
            plan.mark_src_buffer_released(i)  # its copy has not been waited for
        assert e.value.code == binding.ERR_BAD_STATE
        plan.swap_wait_buffer(i)
        assert plan.src_buffer_state(i) == "on_host"
        plan.mark_src_buffer_released(i)
        del buf
        want_state = "released" if n == len(order) - 1 else "mixed"
        assert plan.mem_stats()["state"] == want_state
    torch.cuda.synchronize()
    st = plan.mem_stats()
    ndst = sum(b for b, u in zip(plan.buf_bytes(1), plan.buf_used(1)) if u)
    assert st["src_live"] == 0 and st["released"] == sum(sizes[i] for i in order)
    assert st["peak_device"] == ndst + max(sizes[i] for i in order)  # never more than one source buffer
    host_src = [keep.get(i) for i in range(len(sizes))]
    G.assert_equal_buffers(dst, G.oracle_destinations(wl, host_src, 4), name)
    # before the next update: bind a fresh device home and swap everything back in
    fresh = [torch.zeros(n // 2, dtype=torch.int16, device="cuda") if u else None for n, u in zip(sizes, used)]
    plan.bind_src(G.ptrs(fresh))
    assert plan.mem_stats()["state"] == "on_host"
    plan.swap_in(h)
    plan.swap_wait()
    torch.cuda.synchronize()
    for i in order:
        assert np.array_equal(fresh[i].cpu().numpy(), keep[i])
    # the same way back one buffer at a time: out again, released, then each buffer to a new home
    plan.swap_out(h)
    plan.swap_wait()
    plan.mark_src_released()
    del fresh
    with pytest.raises(ReshardError) as e:
        plan.swap_in_source(order[0], 0, h)  # released: a new device pointer is needed
    assert e.value.code == binding.ERR_BAD_STATE
    homes = {}
    for n, i in enumerate(order):
        homes[i] = torch.zeros(sizes[i] // 2, dtype=torch.int16, device="cuda")
        plan.swap_in_source(i, homes[i].data_ptr(), h)
        assert plan.src_buffer_state(i) == "swapping_in"
        with pytest.raises(ReshardError) as e:
            plan.swap_in_source(i, homes[i].data_ptr(), h)  # already on its way
        assert e.value.code == binding.ERR_BAD_STATE
        assert plan.mem_stats()["src_live"] == sum(sizes[j] for j in order[:n + 1])
        # the caller's stream waits for the copy: work queued on it now sees the weights
        assert np.array_equal(homes[i].cpu().numpy(), keep[i])
        plan.swap_wait_buffer(i)
        assert plan.src_buffer_state(i) == "resident"
        assert plan.mem_stats()["state"] == ("resident" if n == len(order) - 1 else "mixed")
    # and the plan carries on as after an ordinary swap-in
    again = G.device_destinations(plan)
    plan.execute(G.ptrs([homes.get(i) for i in range(len(sizes))]), G.ptrs(again), h)
    torch.cuda.synchronize()
    for a, b in zip(dst, again):
        assert (a is None and b is None) or torch.equal(a, b)


@pytest.mark.parametrize("name", ["C1", "C3E"])
def test_streaming_equals_one_shot_at_full_size(name):
    wl = WORKLOADS[name]
    print("streaming full size", name, flush=True)
    plan = Plan(wl["spec"], wl["src"], wl["dst"])
    src = G.device_sources(plan, wl)
    one = G.device_destinations(plan)
    h = G.stream_handle()
    plan.execute(G.ptrs(src), G.ptrs(one), h)
    stream_plan = Plan(wl["spec"], wl["src"], wl["dst"])
    two = G.device_destinations(stream_plan)
    for i, s_ in enumerate(src):
        if s_ is not None:
            stream_plan.execute_source(i, s_.data_ptr(), G.ptrs(two), h)
    torch.cuda.synchronize()
    for a, b in zip(one, two):
        assert (a is None and b is None) or torch.equal(a, b)
    assert stream_plan.mem_stats()["state"] == "resident"


# ------------------------------------------------------------------ swap ----
def test_swap_round_trip_ledger_and_rebinding():
    wl = WORKLOADS["C0"]
    plan = Plan(wl["spec"], wl["src"], wl["dst"])
    src = G.device_sources(plan, wl)
    dst = G.device_destinations(plan)
    keep = [s.clone() for s in src]
    nsrc, ndst = sum(plan.buf_bytes(0)), sum(plan.buf_bytes(1))
    h = G.stream_handle()
    plan.execute(G.ptrs(src), G.ptrs(dst), h)
    st = plan.mem_stats()
    assert (st["src_live"], st["dst_live"], st["peak_device"], st["state"]) == (nsrc, ndst, nsrc + ndst, "resident")
    plan.swap_out(h)
    assert plan.mem_stats()["state"] == "swapping_out"
    # a repack may run while the copies are in flight: both only read the sources
    dst_b = G.device_destinations(plan)
    plan.execute(G.ptrs(src), G.ptrs(dst_b), h)
    assert plan.mem_stats()["state"] == "swapping_out"
    with pytest.raises(ReshardError) as e:
        plan.execute(G.ptrs(keep), G.ptrs(dst_b), h)  # other pointers than the ones in flight
    assert e.value.code == binding.ERR_BAD_STATE
    plan.swap_wait()
    torch.cuda.synchronize()
    assert torch.equal(dst[0], dst_b[0])
    st = plan.mem_stats()
    assert st["state"] == "on_host" and st["host_pinned"] == nsrc
    # the pinned copy holds the source bytes
    import ctypes
    for i, s in enumerate(keep):
        raw = (ctypes.c_int16 * s.numel()).from_address(plan.host_copy(i))
        assert np.array_equal(np.frombuffer(raw, dtype=np.int16), s.cpu().numpy())
    with pytest.raises(ReshardError):
        plan.swap_out(h)  # already out
    plan.mark_src_released()
    st = plan.mem_stats()
    assert (st["src_live"], st["released"], st["state"], st["peak_device"]) == (0, nsrc, "released", nsrc + ndst)
    # the allocator agrees with the ledger: dropping the training copy frees exactly those bytes
    before = torch.cuda.memory_allocated()
    del src
    assert before - torch.cuda.memory_allocated() == st["released"]
    with pytest.raises(ReshardError) as e:
        plan.swap_in(h)  # no device home yet
    assert e.value.code == binding.ERR_BAD_STATE
    # the caller re-allocates at new addresses and binds them
    fresh = [torch.zeros_like(k) for k in keep]
    plan.bind_src(G.ptrs(fresh))
    assert plan.mem_stats()["state"] == "on_host"
    plan.swap_in(h)
    assert plan.mem_stats()["state"] == "swapping_in"
    torch.cuda.current_stream().synchronize()  # `stream` waits for the copies
    for a, b in zip(fresh, keep):
        assert torch.equal(a, b)
    plan.swap_wait()
    st = plan.mem_stats()
    assert st["state"] == "resident" and st["src_live"] == nsrc
    # and the repack still matches after the round trip
    dst2 = G.device_destinations(plan)
    plan.execute(G.ptrs(fresh), G.ptrs(dst2), h)
    torch.cuda.synchronize()
    assert torch.equal(dst[0], dst2[0])
    plan.release_host()
    assert plan.mem_stats()["host_pinned"] == 0


def test_swap_in_overlaps_other_work_on_the_callers_stream():
    """The host-to-device copies run on the plan's side stream: kernels already queued on
    the caller's stream proceed meanwhile, and work queued after swap_in sees the weights."""
    wl = WORKLOADS["C0"]
    plan = Plan(wl["spec"], wl["src"], wl["dst"])
    src = G.device_sources(plan, wl, "raw16")
    keep = [s.clone() for s in src]
    h = G.stream_handle()
    plan.bind_src(G.ptrs(src))
    plan.swap_out(h)
    plan.swap_wait()
    for s in src:
        s.zero_()
    busy = torch.ones(1 << 24, device="cuda")
    for _ in range(20):  # unrelated work in flight on the caller's stream
        busy = busy * 1.0001
    plan.swap_in(h)
    after = [s.clone() for s in src]  # queued after swap_in on the same stream: must see the weights
    torch.cuda.synchronize()
    for a, k in zip(after, keep):
        assert torch.equal(a, k)
    assert abs(float(busy[0]) - 1.0001 ** 20) < 1e-3
    plan.swap_wait()
    assert plan.mem_stats()["state"] == "resident"


def test_buffers_of_a_swap_in_can_be_consumed_one_by_one():
    """Per-buffer waits: a consumer stream that waits for buffer i alone sees buffer i."""
    wl = TINY["tiny_dense"]  # 8 source buffers
    plan = Plan(wl["spec"], wl["src"], wl["dst"])
    src = G.device_sources(plan, wl, "raw16")
    keep = [s.clone() for s in src]
    h = G.stream_handle()
    plan.bind_src(G.ptrs(src))
    plan.swap_out(h)
    plan.swap_wait_buffer(0)           # host wait for the first buffer's copy
    plan.swap_wait()
    for s in src:
        s.zero_()
    torch.cuda.synchronize()
    plan.swap_in(h)
    consumer = torch.cuda.Stream()
    seen = []
    for i in range(len(src)):
        plan.swap_wait_buffer(i, consumer.cuda_stream, host_wait=False)
        with torch.cuda.stream(consumer):
            seen.append(src[i].clone())
    consumer.synchronize()
    for a, k in zip(seen, keep):
        assert torch.equal(a, k)
    plan.swap_wait()
    assert plan.mem_stats()["state"] == "resident"


def test_pinned_allocation_failure_leaves_the_ledger_unchanged():
    wl = WORKLOADS["C0"]
    plan = Plan(wl["spec"], wl["src"], wl["dst"])
    src = G.device_sources(plan, wl)
    plan.bind_src(G.ptrs(src))
    before = plan.mem_stats()
    try:
        binding.set_host_limit(1 << 20)
        with pytest.raises(ReshardError) as e:
            plan.swap_out(G.stream_handle())
        assert e.value.code == binding.ERR_HOST_OOM
        assert plan.mem_stats() == before
    finally:
        binding.set_host_limit(-1)
    plan.reserve_host()  # allocation ahead of the first swap-out
    assert plan.mem_stats()["host_pinned"] == sum(plan.buf_bytes(0)) and plan.host_copy(0) != 0
    plan.swap_out(G.stream_handle())
    plan.swap_wait()
    assert plan.mem_stats()["state"] == "on_host"


# ------------------------------------------------------------- full sizes ----
def sampled(wl, plan, src, dst, per_tensor, max_tensors, seed):
    rng = np.random.default_rng(seed)
    pairs = locate.sample_pairs(wl["spec"], wl["src"], wl["dst"], per_tensor, rng, max_tensors)
    assert G.gather_check(src, dst, pairs) == 0
    return pairs[0].size


def pads_untouched(plan, dst):
    """Every gap between stored tensors still holds the sentinel."""
    by_buf = {}
    for t in plan.tensors(1):
        by_buf.setdefault(t["buffer"], []).append((t["offset"], t["bytes"]))
    for b, d in enumerate(dst):
        if d is None:
            continue
        end = 0
        for off, nb in sorted(by_buf[b]):
            if off > end:
                assert bool((d[end // 2:off // 2] == G.SENT16).all())
            end = off + nb
        assert bool((d[end // 2:] == G.SENT16).all())


def test_c1_qwen25_7b_shape_whole_output_against_the_oracle():
    print("case C1 full", flush=True)
    plan, src, dst = run_case(WORKLOADS["C1"], "normal")
    pads_untouched(plan, dst)


def test_c1_one_destination_rank_only():
    """A plan for one destination rank (what a single device of the generation side would run):
    only its buffer is written, and it equals the same rank of the unfiltered result."""
    wl = WORKLOADS["C1"]
    print("case C1 rank filter", flush=True)
    only = dict(wl["dst"], tp_filter=1)
    plan, src, dst = run_case(wl, "normal", dst_lay=only)
    assert dst[0] is None and plan.buf_used(1) == [False, True]
    assert plan.info()["bytes_moved"] < 0.51 * Plan(wl["spec"], wl["src"], wl["dst"]).info()["bytes_moved"]
    pads_untouched(plan, dst)


@pytest.mark.parametrize("name", ["C1", "C3"])
def test_full_size_round_trip_returns_the_training_shards_bit_for_bit(name):
    """A property that needs no oracle at any size: train -> gen -> train is the identity on
    every stored tensor (replicated tensors compared on the rank that is read)."""
    wl = WORKLOADS[name]
    print("round trip", name, flush=True)
    train, gen = wl["src"], wl["dst"]
    fwd, back = Plan(wl["spec"], train, gen), Plan(wl["spec"], gen, train)
    src = G.device_sources(fwd, wl, "raw16")
    mid = G.device_destinations(fwd)
    fwd.execute(G.ptrs(src), G.ptrs(mid), G.stream_handle())
    out = G.device_destinations(back)
    back.execute(G.ptrs(mid), G.ptrs(out), G.stream_handle())
    torch.cuda.synchronize()
    del mid
    read_ranks = {t["buffer"] for t in fwd.tensors(0) if t["replicated"]}
    first_rank_of_stage = {b for b in read_ranks if b % train["tp"] == 0}
    for t in fwd.tensors(0):
        if t["replicated"] and t["buffer"] not in first_rank_of_stage:
            continue  # other ranks' copies of common weights are overwritten with rank 0's
        a = src[t["buffer"]][t["offset"] // 2:(t["offset"] + t["bytes"]) // 2]
        b = out[t["buffer"]][t["offset"] // 2:(t["offset"] + t["bytes"]) // 2]
        assert torch.equal(a, b), (t["name"], t["layer"], t["buffer"])
    pads_untouched(back, out)


def test_c1r_kv_replication_and_interleaved_stages_at_full_size():
    print("case C1R full", flush=True)
    plan, src, dst = run_case(WORKLOADS["C1R"], "normal")
    pads_untouched(plan, dst)


@pytest.mark.parametrize("name", ["C2", "C3", "C3P", "C3E"])
def test_largest_shapes_whole_output_and_sampled_pairs(name):
    """The 61-65 GB workloads: every destination byte against the loop oracle (run on host copies
    of the sources), sampled element pairs from every tensor against the definition oracle, pads
    untouched."""
    wl = WORKLOADS[name]
    print("case", name, "full", flush=True)
    plan, src, dst = run_case(wl, "normal", via_swap=True)
    n = sampled(wl, plan, src, dst, 48, 3000, 22)
    print(name, "sampled pairs", n, flush=True)
    pads_untouched(plan, dst)
    assert (plan.info()["num_transpose_tiles"] > 0) == (wl["src"]["expert_layout"] == "grouped")
    if name != "C2":
        return
    # "... and back": the device copy is dropped, the caller allocates new buffers, and the swap-in
    # returns every source byte (compared with the pinned copies and with the seeded fill made again)
    print(name, "swap-in at full size", flush=True)
    del dst
    nsrc = sum(b for b, u in zip(plan.buf_bytes(0), plan.buf_used(0)) if u)
    assert plan.mem_stats()["state"] == "on_host"
    plan.mark_src_released()
    before = torch.cuda.memory_allocated()
    del src
    assert before - torch.cuda.memory_allocated() == nsrc == plan.mem_stats()["released"]
    fresh = [torch.zeros(b // 2, dtype=torch.int16, device="cuda") if u else None
             for b, u in zip(plan.buf_bytes(0), plan.buf_used(0))]
    plan.bind_src(G.ptrs(fresh))
    plan.swap_in(G.stream_handle())
    plan.swap_wait()
    torch.cuda.synchronize()
    assert plan.mem_stats()["state"] == "resident" and plan.mem_stats()["src_live"] == nsrc
    for i, f in enumerate(fresh):
        if f is not None:
            assert np.array_equal(f.cpu().numpy(), G.host_copy_view(plan, i)), f"source buffer {i} differs from its pinned copy"
    again = G.device_sources(plan, wl, "normal")
    for i, (f, g) in enumerate(zip(fresh, again)):
        assert (f is None and g is None) or torch.equal(f, g), f"source buffer {i} differs from the seeded fill"


@pytest.mark.parametrize("name", ["C1", "C4"])
def test_repack_while_the_swap_out_is_in_flight_at_full_size(name):
    """The overlapped order: the swap-out is queued first, the repack is launched while the
    device-to-host copies run (both only read the sources).  The destination must equal the loop
    oracle's, the pinned copies must equal the device sources, and once reshard_swap_wait has
    returned the repack has finished reading them, so they may be dropped at once."""
    wl = WORKLOADS[name]
    print("case", name, "overlapped swap-out and repack", flush=True)
    plan = Plan(wl["spec"], wl["src"], wl["dst"])
    plan.prepare()
    plan.reserve_host()
    src = G.device_sources(plan, wl, "raw16")
    dst = G.device_destinations(plan)
    h = G.stream_handle()
    plan.bind_src(G.ptrs(src))
    torch.cuda.synchronize()
    plan.swap_out(h)
    assert plan.mem_stats()["state"] == "swapping_out"
    plan.execute(G.ptrs(src), G.ptrs(dst), h)
    first = plan.buf_used(0).index(True)
    assert plan.src_buffer_state(first) == "swapping_out"
    plan.swap_wait()
    assert plan.mem_stats()["state"] == "on_host"
    # no synchronisation of the caller's stream here: swap_wait vouches for the repack as well
    plan.mark_src_released()
    keep = [None if s is None else G.host_copy_view(plan, i) for i, s in enumerate(src)]
    for i, s in enumerate(src):
        if s is not None:
            assert np.array_equal(s.cpu().numpy(), keep[i]), f"pinned copy of source buffer {i} differs"
    del src
    torch.cuda.synchronize()
    want = G.oracle_destinations(wl, keep, 16)
    G.assert_equal_buffers(dst, want, name + " overlapped")
    pads_untouched(plan, dst)


def test_swap_wait_also_waits_for_a_repack_launched_during_the_swap_out():
    """On a small plan the copies end before the kernel does.  reshard_swap_wait must not return
    (and the sources must not count as free to go) before a repack launched during the swap-out has
    read them: right after it returns another stream overwrites the sources, and the destination
    must still hold the original weights' repack."""
    wl = WORKLOADS["C0"]
    plan = Plan(wl["spec"], wl["src"], wl["dst"])
    plan.prepare()
    plan.reserve_host()
    h = G.stream_handle()
    other = torch.cuda.Stream()
    for rep in range(20):
        src = G.device_sources(plan, wl, "raw16")
        keep = G.to_host(src)
        dst = G.device_destinations(plan)
        plan.bind_src(G.ptrs(src))
        torch.cuda.synchronize()
        plan.swap_out(h)
        plan.execute(G.ptrs(src), G.ptrs(dst), h)
        plan.swap_wait()
        with torch.cuda.stream(other):  # not ordered after the caller's stream in any way
            for s_ in src:
                s_.fill_(0x5A5A)
        torch.cuda.synchronize()
        G.assert_equal_buffers(dst, G.oracle_destinations(wl, keep, 2), f"rep {rep}")
        plan.mark_src_released()
        plan.bind_src(G.ptrs(src))
        plan.swap_in(h)
        plan.swap_wait()
        torch.cuda.synchronize()
        for s_, k in zip(src, keep):
            assert np.array_equal(s_.cpu().numpy(), k)


def test_shared_tail_pool_at_full_size():
    """The copy kernel's optional tail pool (the end of every XCD's share of the table is handed out
    in chunks to whichever workgroups get there first) on the 15 GB plan: same bits as the default
    launch, also on the second execute (the pool's counters are cleared by every launch)."""
    wl = WORKLOADS["C1"]
    print("case C1 tail pool", flush=True)
    plan = Plan(wl["spec"], wl["src"], wl["dst"])
    src = G.device_sources(plan, wl, "raw16")
    one = G.device_destinations(plan)
    plan.execute(G.ptrs(src), G.ptrs(one), G.stream_handle())
    for pct, chunk in ((6, 16), (6, 16), (33, 5)):
        plan.set_tuning(flags=31, tail_pool_percent=pct, tail_chunk_tiles=chunk)
        two = G.device_destinations(plan)
        plan.execute(G.ptrs(src), G.ptrs(two), G.stream_handle())
        torch.cuda.synchronize()
        for a, b in zip(one, two):
            assert torch.equal(a, b), (pct, chunk)
        del two


def test_a_table_too_long_for_one_launch_goes_out_in_slices():
    """4 KiB tiles on the 26 GB plan: 6.4 million workgroups of 1024 lanes, more lanes than one
    launch can have, so the copy class is launched in two slices; same bits as the default plan."""
    wl = WORKLOADS["C4"]
    print("case C4 sliced launches", flush=True)
    plan = Plan(wl["spec"], wl["src"], wl["dst"])
    src = G.device_sources(plan, wl, "raw16")
    one = G.device_destinations(plan)
    plan.execute(G.ptrs(src), G.ptrs(one), G.stream_handle())
    small = Plan(wl["spec"], wl["src"], wl["dst"], tuning=dict(tile_bytes=4096))
    assert small.info()["num_tiles"] * 1024 > 1 << 32
    two = G.device_destinations(small)
    small.execute(G.ptrs(src), G.ptrs(two), G.stream_handle())
    torch.cuda.synchronize()
    for a, b in zip(one, two):
        assert (a is None and b is None) or torch.equal(a, b)


def test_c4_deepseek_shape_share_whole_output():
    print("case C4 full", flush=True)
    plan, src, dst = run_case(WORKLOADS["C4"], "normal")
    assert sum(s is not None for s in src) == 9
    pads_untouched(plan, dst)
