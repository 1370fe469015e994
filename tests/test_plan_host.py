"""Host logic of the library, checked without a GPU.

The plan builder's output (buffer tables, tensor tables, copy descriptors) is
interpreted here by a few lines of numpy and compared with the CPU oracles.
Nothing in this file launches a kernel; the interpreter below lives in the
tests only and is not a product path.
"""

import ctypes as C
import os
import re
import subprocess

import numpy as np
import pytest

import np_pack
from oracle import fast, locate
from paper_2507_19017_amd import Plan, ReshardError, binding, get_tuning, set_tuning
from synth_inputs import MID, TINY, WORKLOADS, make_layout, make_spec

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SENT = 0xA5


def with_eb(spec, eb):
    s = dict(spec)
    s["elem_bytes"] = eb
    return s


def run_descs(descs, src, dst, counts=None):
    """Interpret the descriptor table on byte arrays, exactly as reshard.h words it."""
    for d in descs:
        s, t = src[d["src_buf"]], dst[d["dst_buf"]]
        eb = d["elem_bytes"]
        if d["kind"] == 0:
            for i in range(d["rows"]):
                a, b = d["src_off"] + i * d["src_stride"], d["dst_off"] + i * d["dst_stride"]
                t[b:b + d["row_bytes"]] = s[a:a + d["row_bytes"]]
                if counts is not None:
                    counts[d["dst_buf"]][b:b + d["row_bytes"]] += 1
        else:
            cols = d["row_bytes"] // eb
            i, k, e = np.meshgrid(np.arange(d["rows"]), np.arange(cols), np.arange(eb), indexing="ij")
            a = (d["src_off"] + i * d["src_stride"] + k * eb + e).ravel()
            b = (d["dst_off"] + k * d["dst_stride"] + i * eb + e).ravel()
            t[b] = s[a]
            if counts is not None:
                np.add.at(counts[d["dst_buf"]], b, 1)


def run_tiles(tiles, src, dst, counts, woven=True):
    """Interpret the device tile table on byte arrays, as reshard.h words it: the tiles every
    execute launches plus those of the one order (woven or not)."""
    for t in tiles:
        if t["order"] == (1 if woven else 2):
            continue
        s, d = src[t["src_buf"]], dst[t["dst_buf"]]
        v = t["vec_bytes"]
        if t["kind"] == 2:
            w = t["phase"] + np.arange(t["rows"])
            seg, c = w // t["row_units"], w % t["row_units"]
            j, r = seg % t["sources"], seg // t["sources"]
            a0 = t["src_off"] + r * t["src_stride"] + c * v
            e = np.arange(v)
            b = (t["dst_off"] + np.arange(t["rows"])[:, None] * v + e).ravel()
            vals = np.empty((t["rows"], v), dtype=np.uint8)
            for jj in np.unique(j):
                m = j == jj
                vals[m] = src[t["src_buf"] + int(jj)][(a0[m][:, None] + e)]
            d[b] = vals.ravel()
            np.add.at(counts[t["dst_buf"]], b, 1)
            continue
        if t["kind"] == 0:
            i, u, e = np.meshgrid(np.arange(t["rows"]), np.arange(t["row_units"]), np.arange(v), indexing="ij")
            a = (t["src_off"] + i * t["src_stride"] + u * v + e).ravel()
            b = (t["dst_off"] + i * t["dst_stride"] + u * v + e).ravel()
        else:
            i, k, e = np.meshgrid(np.arange(t["rows"]), np.arange(t["row_units"]), np.arange(v), indexing="ij")
            a = (t["src_off"] + i * t["src_stride"] + k * v + e).ravel()
            b = (t["dst_off"] + k * t["dst_stride"] + i * v + e).ravel()
        d[b] = s[a]
        np.add.at(counts[t["dst_buf"]], b, 1)


TILE_TUNINGS = [dict(), dict(tile_bytes=4096, transpose_rows=64, transpose_cols=128),
                dict(tile_bytes=8192, transpose_rows=128, transpose_cols=64), dict(transpose_rows=64, transpose_cols=64)]
TILE_CASES = [(n, 2, t) for n in ["tiny_dense", "tiny_moe_grouped", "mid_moe_grouped", "tiny_kvrep", "tiny_vocabpad",
                                  "tiny_etp", "C0"] for t in TILE_TUNINGS]
# transposing tiles at the other element sizes: the default shape of each, and the longest tiles
TILE_CASES += [("big_moe_grouped", eb, t) for eb, t in [
    (1, dict()), (1, dict(transpose_rows=512, transpose_cols=256)), (1, dict(transpose_rows=128, transpose_cols=512)),
    (2, dict()), (4, dict()), (4, dict(transpose_rows=256, transpose_cols=64)), (8, dict()),
    (8, dict(transpose_rows=64, transpose_cols=256))]]
TILE_CASES += [("mid_moe_grouped", eb, dict()) for eb in (1, 4, 8)]
# side-by-side merges that also exist as gathered tiles, at several tile sizes (rows of 64 and 88 vectors)
TILE_CASES += [(n, MID[n]["spec"]["elem_bytes"], t) for n in sorted(MID)
               for t in (dict(), dict(tile_bytes=4096), dict(tile_bytes=8192), dict(tile_bytes=131072))]


def transpose_shape(eb, tuning):
    """Tile shape the library documents for an element size: the tuning's if it fits 128 KiB
    (and is one it builds), else the default of that size."""
    default = {1: (512, 256), 2: (256, 256), 4: (128, 256), 8: (128, 128)}[eb]
    ti, tk = tuning.get("transpose_rows", 0), tuning.get("transpose_cols", 0)
    ok = ti and tk and ti * tk * eb <= 131072 and (ti >= 128 and tk >= 128 if eb == 1 else max(ti, tk) <= 256)
    if 192 in (ti, tk):  # built for 2-byte elements only, with 192 or 256 on the other side
        ok = ok and eb == 2 and min(ti, tk) >= 192
    return (ti, tk) if ok else default


@pytest.mark.parametrize("name,eb,tuning", TILE_CASES)
def test_tile_table_reproduces_the_oracle_and_writes_every_byte_once(name, eb, tuning):
    """The cut into device tiles (rows per tile, runs of long rows, vector width, the three
    levels of transposing tiles) moves exactly what the descriptors say."""
    w = {**TINY, **MID, **WORKLOADS}[name]
    spec = with_eb(w["spec"], eb)
    try:
        set_tuning(**tuning)
        plan = Plan(spec, w["src"], w["dst"])
    finally:
        set_tuning()
    S, D = locate.Layout(spec, w["src"]), locate.Layout(spec, w["dst"])
    rng = np.random.default_rng(17)
    src = [rng.integers(0, 256, size=n, dtype=np.uint8) for n in S.buf_bytes]
    dst = [np.full(n, SENT, dtype=np.uint8) for n in D.buf_bytes]
    cnt = [np.zeros(n, dtype=np.int32) for n in D.buf_bytes]
    tiles = plan.tiles()
    assert len(tiles) == plan.info()["num_tiles"]
    want = [np.full(n, SENT, dtype=np.uint8) for n in D.buf_bytes]
    fast.reshard(spec, w["src"], w["dst"], [x.view(np.uint16) for x in src], [x.view(np.uint16) for x in want])
    for woven in (True, False):  # the table holds some bytes cut two ways; either order is the whole work
        for b in range(D.nbufs):
            dst[b][:] = SENT
            cnt[b][:] = 0
        run_tiles(tiles, src, dst, cnt, woven)
        for b in range(D.nbufs):
            assert np.array_equal(dst[b], want[b]), f"buffer {b}"
            owned = np.zeros(D.buf_bytes[b], dtype=bool)
            for off, nb in D.owned(b):
                owned[off:off + nb] = True
            assert np.all(cnt[b][owned] == 1) and np.all(cnt[b][~owned] == 0)
    assert sum(t["order"] == 1 for t in tiles) > 0 or all(t["order"] == 0 for t in tiles)
    shape = transpose_shape(eb, tuning)
    for t in tiles:
        units = t["rows"] * t["row_units"]
        assert units >= 1 and t["vec_bytes"] in (1, 2, 4, 8, 16)
        if t["kind"] == 2:
            assert t["tile_class"] == 0 and t["order"] == 2 and t["vec_bytes"] == 16 and 1 <= t["rows"] <= 32768
            assert 64 <= t["row_units"] and t["sources"] in (1, 2, 4, 8, 16, 32, 64, 128, 256)
            assert 0 <= t["phase"] < t["sources"] * t["row_units"]
            assert (t["src_off"] | t["dst_off"] | t["src_stride"]) % 16 == 0 and t["src_stride"] >= 16 * t["row_units"]
        elif t["kind"] == 0:
            assert t["tile_class"] == 0 and units <= 32768
            assert (t["src_off"] | t["dst_off"]) % t["vec_bytes"] == 0
            if t["rows"] > 1:
                assert (t["src_stride"] | t["dst_stride"]) % t["vec_bytes"] == 0
        else:
            assert t["tile_class"] in (1, 2, 3)
            if t["tile_class"] in (1, 2):  # register path: whole tiles of a built shape, 16-byte accesses
                assert (t["src_off"] | t["dst_off"] | t["src_stride"] | t["dst_stride"]) % 16 == 0
                got = (t["rows"], t["row_units"])
                assert (got == shape) == (t["tile_class"] == 1)
                assert transpose_shape(eb, dict(transpose_rows=got[0], transpose_cols=got[1])) == got
                assert t["vec_bytes"] == eb
            else:
                assert t["rows"] <= 64 and t["row_units"] <= 64
    classes = {t["tile_class"] for t in tiles}
    if name in MID:  # the gathered form exists exactly where a tile holds more than one segment of a row
        gathered = sum(t["rows"] * 16 for t in tiles if t["kind"] == 2)
        assert gathered == sum(t["rows"] * t["row_units"] * 16 for t in tiles if t["order"] == 1)
        assert gathered > 0
        assert {t["sources"] for t in tiles if t["kind"] == 2} <= {{"mid_merge2": 2, "mid_merge4": 4, "mid_merge8": 8, "mid_split": 1}[name]}
    if name == "mid_moe_grouped" and eb == 2:  # 320 x 200 and 200 x 320 matrices: register path and ragged rest
        assert 0 in classes and 3 in classes and classes & {1, 2}
    if name == "big_moe_grouped":  # the preferred shape, smaller shapes on the strips, a ragged rest
        assert classes == {0, 1, 2, 3}


CASES = [(n, eb) for n in sorted(TINY) for eb in (1, 2, 4, 8)]


@pytest.mark.parametrize("name,eb", CASES)
def test_descriptors_reproduce_the_oracle_on_tiny_models(name, eb):
    w = TINY[name]
    spec = with_eb(w["spec"], eb)
    plan = Plan(spec, w["src"], w["dst"])
    S = locate.Layout(spec, w["src"])
    D = locate.Layout(spec, w["dst"])
    assert plan.buf_bytes(0) == S.buf_bytes and plan.buf_bytes(1) == D.buf_bytes
    assert plan.buf_used(1) == [D.buffer_used(b) for b in range(D.nbufs)]
    rng = np.random.default_rng(w["seed"] + eb)
    src = [rng.integers(0, 256, size=n, dtype=np.uint8) for n in S.buf_bytes]
    dst = [np.full(n, SENT, dtype=np.uint8) for n in D.buf_bytes]
    cnt = [np.zeros(n, dtype=np.int32) for n in D.buf_bytes]
    run_descs(plan.descs(), src, dst, cnt)
    dt = {1: np.uint8, 2: np.uint16, 4: np.uint32, 8: np.uint64}[eb]
    want = [np.full(n, SENT, dtype=np.uint8) if D.buffer_used(b) else None for b, n in enumerate(D.buf_bytes)]
    read = locate.reshard_definition(spec, w["src"], w["dst"], [s.view(dt) for s in src],
                                     [x.view(dt) if x is not None else None for x in want])
    total = 0
    for b in range(D.nbufs):
        if want[b] is None:
            assert np.all(dst[b] == SENT) and not cnt[b].any()
            continue
        assert np.array_equal(dst[b], want[b]), f"buffer {b}"
        owned = np.zeros(D.buf_bytes[b], dtype=bool)
        for off, nb in D.owned(b):
            owned[off:off + nb] = True
        assert np.all(cnt[b][owned] == 1) and np.all(cnt[b][~owned] == 0)  # exactly once, pads never
        total += int(owned.sum())
    assert plan.info()["bytes_moved"] == total
    assert {i for i, u in enumerate(plan.buf_used(0)) if u} == read


def test_degenerate_shapes_through_the_descriptor_interpreter():
    cases = [
        (make_spec(family="dense_gqa", L=1, H=8, nq=1, nkv=1, d=8, I=8, V=8), make_layout(kind="train"), make_layout(kind="gen")),
        (make_spec(family="dense_gqa", L=3, H=64, nq=8, nkv=4, d=8, I=32, V=0, has_embeddings=0),
         make_layout(kind="train", tp=1), make_layout(kind="gen", tp=1)),
        (make_spec(family="moe_gqa", L=2, H=32, nq=4, nkv=2, d=8, V=48, E=4, Ie=24, n_shared=1),
         make_layout(kind="gen", tp=2, ep=2), make_layout(kind="gen", tp=2, ep=2)),
        (make_spec(family="moe_gqa", L=2, H=32, nq=4, nkv=4, d=8, V=64, E=8, Ie=16),
         make_layout(kind="train", tp=2, pp=2, ep=4), make_layout(kind="gen", tp=4, ep=8, tp_filter=3, ep_filter=5)),
        (make_spec(family="dense_gqa", L=2, H=7, nq=3, nkv=3, d=5, I=9, V=6, qkv_bias=1, elem_bytes=1),
         make_layout(kind="train", tp=3), make_layout(kind="gen", tp=1)),
    ]
    for spec, a, b in cases:
        eb = spec["elem_bytes"]
        plan = Plan(spec, a, b)
        A, B = locate.Layout(spec, a), locate.Layout(spec, b)
        assert plan.buf_bytes(0) == A.buf_bytes and plan.buf_bytes(1) == B.buf_bytes
        rng = np.random.default_rng(5)
        src = [rng.integers(0, 256, size=n, dtype=np.uint8) for n in A.buf_bytes]
        dst = [np.full(n, SENT, dtype=np.uint8) for n in B.buf_bytes]
        run_descs(plan.descs(), src, dst)
        dt = {1: np.uint8, 2: np.uint16}[eb]
        want = [np.full(n, SENT, dtype=np.uint8) if B.buffer_used(i) else None for i, n in enumerate(B.buf_bytes)]
        fast.reshard(spec, a, b, [x.view(dt) for x in src], [x.view(dt) if x is not None else None for x in want])
        for i, wnt in enumerate(want):
            assert np.array_equal(dst[i], wnt if wnt is not None else np.full(B.buf_bytes[i], SENT, dtype=np.uint8))


@pytest.mark.parametrize("pair", ["identity", "back"])
@pytest.mark.parametrize("name", sorted(TINY))
def test_identity_and_way_back_plans(name, pair):
    w = TINY[name]
    spec = with_eb(w["spec"], 2)
    train = w["src"]
    gen = dict(w["dst"], tp_filter=-1, ep_filter=-1)
    a, b = (train, train) if pair == "identity" else (gen, train)
    plan = Plan(spec, a, b)
    A, B = locate.Layout(spec, a), locate.Layout(spec, b)
    rng = np.random.default_rng(3)
    lg = np_pack.make_logical(spec, locate.logical_tensors(spec), rng, np.uint16)
    src = [x.view(np.uint8) for x in np_pack.pack(spec, a, lg, np.uint16, 0xA5A5)]
    want = [x.view(np.uint8) for x in np_pack.pack(spec, b, lg, np.uint16, 0xA5A5)]
    dst = [np.full(n, SENT, dtype=np.uint8) for n in B.buf_bytes]
    run_descs(plan.descs(), src, dst)
    for x, y in zip(dst, want):
        assert np.array_equal(x, y)
    if pair == "identity":
        # one contiguous run per stored tensor at most: nothing is cut finer than a tensor
        assert all(d["kind"] == 0 for d in plan.descs())


def test_tensor_table_matches_the_oracle_layout():
    for w in list(TINY.values()) + [WORKLOADS["C0"], WORKLOADS["C1"], WORKLOADS["C4"]]:
        plan = Plan(w["spec"], w["src"], w["dst"])
        for side, lay in ((0, w["src"]), (1, w["dst"])):
            L = locate.Layout(w["spec"], lay)
            got = [(t["buffer"], t["name"], t["layer"], t["offset"], t["bytes"]) for t in plan.tensors(side)]
            want = [(b, n, l, off, nb) for b in range(L.nbufs) for (n, l, j, off, nb) in L.stored[b]]
            assert got == want
            for t in plan.tensors(side):
                assert t["replicated"] == (t["name"] in locate.REPLICATED or t["name"] == "emb_tied")
                assert t["offset"] % 256 == 0


@pytest.mark.parametrize("name", ["C0", "C1", "C1R", "C2", "C3", "C3P", "C4"])
def test_full_size_plans_cover_every_destination_byte_once(name):
    """Interval analysis at the benchmark shapes: the destination intervals of all
    descriptor rows are pairwise disjoint and their union is exactly the stored
    tensors of the used buffers (so pads are never written and no byte twice);
    source rows stay inside their buffers."""
    w = WORKLOADS[name]
    plan = Plan(w["spec"], w["src"], w["dst"])
    D = locate.Layout(w["spec"], w["dst"])
    S = locate.Layout(w["spec"], w["src"])
    assert plan.buf_bytes(0) == S.buf_bytes and plan.buf_bytes(1) == D.buf_bytes
    starts, ends = {}, {}
    moved = 0
    for d in plan.descs():
        moved += d["rows"] * d["row_bytes"]
        eb = d["elem_bytes"]
        if d["kind"] == 0:
            n, nb, st = d["rows"], d["row_bytes"], d["dst_stride"]
        else:  # destination side of a transposing descriptor: one row per source column
            n, nb, st = d["row_bytes"] // eb, d["rows"] * eb, d["dst_stride"]
        shi = d["src_off"] + (d["rows"] - 1) * d["src_stride"] + d["row_bytes"]
        assert 0 <= d["src_off"] and shi <= S.buf_bytes[d["src_buf"]]
        assert n >= 1 and nb >= 1 and (n == 1 or st >= nb)
        if n > 1 and st == nb:
            n, nb = 1, n * nb
        a = d["dst_off"] + st * np.arange(n, dtype=np.int64)
        starts.setdefault(d["dst_buf"], []).append(a)
        ends.setdefault(d["dst_buf"], []).append(a + nb)
    assert moved == plan.info()["bytes_moved"]
    total = 0
    for b in range(D.nbufs):
        if not D.buffer_used(b):
            assert b not in starts
            continue
        a = np.concatenate(starts[b])
        e = np.concatenate(ends[b])
        order = np.argsort(a, kind="stable")
        a, e = a[order], e[order]
        assert np.all(a[1:] >= e[:-1]), "two descriptor rows overlap"
        # union of the written intervals, merged where they touch
        brk = np.flatnonzero(a[1:] != e[:-1])
        ua = np.concatenate([a[:1], a[brk + 1]])
        ue = np.concatenate([e[brk], e[-1:]])
        # union of the stored tensors, merged where they touch
        ta = np.array([off for off, nb in D.owned(b)], dtype=np.int64)
        te = ta + np.array([nb for off, nb in D.owned(b)], dtype=np.int64)
        tb = np.flatnonzero(ta[1:] != te[:-1])
        wa = np.concatenate([ta[:1], ta[tb + 1]])
        we = np.concatenate([te[tb], te[-1:]])
        assert np.array_equal(ua, wa) and np.array_equal(ue, we)
        total += int((te - ta).sum())
    assert moved == total


def test_sampled_descriptor_rows_agree_with_the_definition_oracle_at_full_size():
    """For C1 and C3: pick random logical elements, find the descriptor row that writes
    their destination byte, and check it reads the oracle's source byte."""
    rng = np.random.default_rng(9)
    for name in ("C1", "C3"):
        w = WORKLOADS[name]
        plan = Plan(w["spec"], w["src"], w["dst"])
        descs = plan.descs()
        sb, so, db, do = locate.sample_pairs(w["spec"], w["src"], w["dst"], 6, rng, max_tensors=400)
        by_buf = {}
        for d in descs:
            by_buf.setdefault(d["dst_buf"], []).append(d)
        for b in by_buf:
            by_buf[b].sort(key=lambda d: d["dst_off"])
        for a, ao, b, bo in zip(sb, so, db, do):
            hit = None
            for d in by_buf[int(b)]:
                eb = d["elem_bytes"]
                if d["kind"] == 0:
                    span = (d["rows"] - 1) * d["dst_stride"] + d["row_bytes"]
                    if not (d["dst_off"] <= bo < d["dst_off"] + span):
                        continue
                    i, rem = divmod(int(bo) - d["dst_off"], d["dst_stride"])
                    if rem < d["row_bytes"]:
                        hit = (d["src_buf"], d["src_off"] + i * d["src_stride"] + rem)
                        break
                else:
                    cols = d["row_bytes"] // eb
                    span = (cols - 1) * d["dst_stride"] + d["rows"] * eb
                    if not (d["dst_off"] <= bo < d["dst_off"] + span):
                        continue
                    k, rem = divmod(int(bo) - d["dst_off"], d["dst_stride"])
                    if rem < d["rows"] * eb:
                        i = rem // eb
                        hit = (d["src_buf"], d["src_off"] + i * d["src_stride"] + k * eb)
                        break
            assert hit == (int(a), int(ao)), (name, int(b), int(bo))


def test_weight_classes_and_the_redundant_memory_formula():
    """Classes T / E / C of the paper's redundant-memory example, and Eq. (3) on them."""
    from paper_2507_19017_amd import redundant_memory_bytes
    w = WORKLOADS["C3"]
    plan = Plan(w["spec"], w["src"], w["dst"])
    src = plan.class_bytes(0)
    # source TP1: experts 57.98 GB, replicated norms + routers, the rest tensor-parallel class
    assert src["E"] == 57_982_058_496
    assert src["T"] + src["C"] + src["E"] == 61_064_220_672
    common = sum(R * C for n, *_, R, C in locate.logical_tensors(w["spec"]) if n in locate.REPLICATED) * 2
    assert src["C"] == common
    dst = plan.class_bytes(1)
    assert dst["E"] == src["E"] and dst["T"] == src["T"] and dst["C"] == 2 * common  # TP2: two copies
    for t in plan.tensors(0):
        assert t["weight_class"] == ("E" if t["buffer"] >= 2 else "C" if t["name"] in locate.REPLICATED else "T")
    # Eq. (3) with TW = T + C bytes and EW = E bytes: the paper's "more than 60 GB"
    tw, ew = src["T"] + src["C"], src["E"]
    r = redundant_memory_bytes(4, tw, 4, ew, 4)
    assert r == 4 * (tw / 4 + ew / 4) and r / 1e9 > 60
    assert redundant_memory_bytes(0, tw, 4, ew, 4) == -1.0


def test_invalid_requests_return_error_codes():
    spec = dict(WORKLOADS["C0"]["spec"])
    gen = make_layout(kind="gen", tp=1)
    cases = [
        (spec, make_layout(kind="train", tp=3), gen, binding.ERR_UNSUPPORTED),   # heads % tp
        (dict(spec, nq=12, nkv=4, H=768), make_layout(kind="train", tp=6), gen, binding.ERR_UNSUPPORTED),  # 6 vs 4 KV heads
        (spec, make_layout(kind="train", tp=2, pp=2, vpp=2, first_stage_layers=1, last_stage_layers=1), gen, binding.ERR_UNSUPPORTED),
        (spec, make_layout(kind="train", tp=2, pp=2, vpp=3), gen, binding.ERR_UNSUPPORTED),
        (spec, make_layout(kind="train", tp=2, pp=2, first_stage_layers=1, last_stage_layers=2), gen, binding.ERR_UNSUPPORTED),
        (spec, make_layout(kind="train", tp=2, pp=1, first_stage_layers=1, last_stage_layers=1), gen, binding.ERR_UNSUPPORTED),
        (spec, make_layout(kind="train", tp=2, vpp=-1), gen, binding.ERR_INVALID_ARG),
        (spec, make_layout(kind="train", tp=2, pp=3), gen, binding.ERR_UNSUPPORTED),
        (spec, make_layout(kind="train", tp=2), make_layout(kind="gen", tp=1, pp=2), binding.ERR_UNSUPPORTED),
        (spec, make_layout(kind="train", tp=2, ep=2), gen, binding.ERR_UNSUPPORTED),
        (spec, make_layout(kind="train", tp=2, tp_filter=0), gen, binding.ERR_INVALID_ARG),
        (spec, make_layout(kind="train", tp=2), make_layout(kind="gen", tp=1, tp_filter=1), binding.ERR_INVALID_ARG),
        (dict(spec, elem_bytes=3), make_layout(kind="train", tp=2), gen, binding.ERR_INVALID_ARG),
        (dict(spec, V=1023), make_layout(kind="train", tp=2), gen, binding.ERR_UNSUPPORTED),
        (TINY["tiny_etp"]["spec"], make_layout(kind="train", tp=4, ep=2, etp=2), make_layout(kind="gen", ep=1), binding.ERR_UNSUPPORTED),
        (spec, make_layout(kind="train", tp=2, vocab_padded=1000), gen, binding.ERR_INVALID_ARG),   # below V
        (spec, make_layout(kind="train", tp=2, vocab_padded=1025), gen, binding.ERR_UNSUPPORTED),   # not divisible
        (dict(spec, L=0), make_layout(kind="train", tp=2), gen, binding.ERR_INVALID_ARG),
    ]
    for s, a, b, code in cases:
        with pytest.raises(ReshardError) as e:
            Plan(s, a, b)
        assert e.value.code == code, (a, b, e.value)
        assert binding.last_error()
    # too many buffers
    big = make_spec(family="moe_gqa", L=4, H=64, nq=4, nkv=4, d=8, V=64, E=512, Ie=8)
    with pytest.raises(ReshardError) as e:
        Plan(big, make_layout(kind="train", ep=512), make_layout(kind="gen", ep=1))
    assert e.value.code == binding.ERR_UNSUPPORTED
    # struct_size mismatch and NULLs through the raw ABI
    l = binding.lib()
    s, a, b = binding.make_spec(spec), binding.make_layout(make_layout(kind="train", tp=2)), binding.make_layout(gen)
    out = C.c_void_p()
    s.struct_size = 4
    assert l.reshard_plan_create(C.byref(s), C.byref(a), C.byref(b), C.byref(out)) == binding.ERR_INVALID_ARG
    assert l.reshard_plan_create(None, C.byref(a), C.byref(b), C.byref(out)) == binding.ERR_INVALID_ARG
    assert l.reshard_plan_destroy(None) == 0


def test_state_machine_errors_without_a_device():
    """Calls that need bound pointers are refused before any HIP call is made."""
    w = WORKLOADS["C0"]
    plan = Plan(w["spec"], w["src"], w["dst"])
    assert plan.mem_stats() == dict(src_live=0, dst_live=0, host_pinned=0, peak_device=0, released=0, state="unbound")
    for call in (plan.swap_out, plan.swap_in, plan.mark_src_released):
        with pytest.raises(ReshardError) as e:
            call()
        assert e.value.code == binding.ERR_BAD_STATE
    with pytest.raises(ReshardError) as e:
        plan.execute([0, 0], [0])
    assert e.value.code == binding.ERR_INVALID_ARG  # NULL pointers for used buffers
    with pytest.raises(ReshardError) as e:
        plan.execute([256, 512 + 8], [4096])
    assert e.value.code == binding.ERR_INVALID_ARG  # misaligned
    with pytest.raises(ReshardError) as e:
        plan.execute([1 << 20, 1 << 30], [(1 << 20) + 256])
    assert e.value.code == binding.ERR_INVALID_ARG  # overlap
    plan.swap_wait()  # no-op
    with pytest.raises(ReshardError) as e:
        plan.swap_wait_buffer(0)
    assert e.value.code == binding.ERR_BAD_STATE
    with pytest.raises(ReshardError) as e:
        plan.swap_in_source(0, 256)  # nothing was swapped out
    assert e.value.code == binding.ERR_BAD_STATE
    with pytest.raises(ReshardError) as e:
        plan.swap_in_source(9, 256)
    assert e.value.code == binding.ERR_INVALID_ARG
    with pytest.raises(ReshardError) as e:
        plan.swap_wait_buffer(7)
    assert e.value.code == binding.ERR_INVALID_ARG
    plan.release_host()
    assert plan.host_copy(0) == 0


def test_tuning_is_validated():
    set_tuning()
    base = get_tuning()
    assert base == dict(tile_bytes=32768, block_threads=1024, blocks_per_cu=0, unroll=2, flags=127, transpose_rows=0,
                        transpose_cols=0, tail_pool_percent=0, tail_chunk_tiles=16, table_copies=0)
    set_tuning(tile_bytes=8192, unroll=4)
    assert get_tuning()["tile_bytes"] == 8192 and get_tuning()["unroll"] == 4
    w = WORKLOADS["C1"]
    n8 = Plan(w["spec"], w["src"], w["dst"]).info()["num_tiles"]
    set_tuning()
    n32 = Plan(w["spec"], w["src"], w["dst"]).info()["num_tiles"]
    assert n8 > 3.5 * n32
    for bad in (dict(tile_bytes=1000), dict(block_threads=96), dict(unroll=3), dict(unroll=16), dict(blocks_per_cu=100),
                dict(unroll=8, flags=5), dict(flags=128), dict(table_copies=65), dict(table_copies=-1)):
        with pytest.raises(ReshardError):
            set_tuning(**bad)
    assert get_tuning() == base


def test_every_plan_keeps_its_own_tuning():
    """The process-wide tuning is only what new plans start from: a plan keeps the tile size it was
    cut with and its own launch shape whatever is set afterwards, and two plans may differ."""
    w = WORKLOADS["C0"]
    set_tuning()
    a = Plan(w["spec"], w["src"], w["dst"], tuning=dict(tile_bytes=4096, unroll=1, block_threads=256))
    b = Plan(w["spec"], w["src"], w["dst"])
    try:
        set_tuning(tile_bytes=8192, unroll=4, flags=7)
        c = Plan(w["spec"], w["src"], w["dst"])
    finally:
        set_tuning()
    assert a.get_tuning() == dict(tile_bytes=4096, block_threads=256, blocks_per_cu=0, unroll=1, flags=127,
                                  transpose_rows=0, transpose_cols=0, tail_pool_percent=0, tail_chunk_tiles=16, table_copies=0)
    assert b.get_tuning()["tile_bytes"] == 32768 and b.get_tuning()["unroll"] == 2
    assert c.get_tuning()["tile_bytes"] == 8192 and c.get_tuning()["unroll"] == 4 and c.get_tuning()["flags"] == 7
    assert a.info()["num_tiles"] > c.info()["num_tiles"] >= b.info()["num_tiles"]
    # the launch shape of an existing plan may change, what cut its tiles may not
    a.set_tuning(unroll=2, flags=23, blocks_per_cu=2)
    t = a.get_tuning()
    assert (t["tile_bytes"], t["unroll"], t["flags"], t["blocks_per_cu"], t["block_threads"]) == (4096, 2, 23, 2, 1024)
    a.set_tuning(tile_bytes=4096, block_threads=128)  # naming the plan's own tile size is fine
    assert a.get_tuning()["block_threads"] == 128 and a.get_tuning()["unroll"] == 2
    for bad in (dict(tile_bytes=8192), dict(transpose_rows=64), dict(unroll=3)):
        with pytest.raises(ReshardError) as e:
            a.set_tuning(**bad)
        assert e.value.code == binding.ERR_INVALID_ARG
    assert a.get_tuning()["block_threads"] == 128
    with pytest.raises(ReshardError):
        Plan(w["spec"], w["src"], w["dst"], tuning=dict(tile_bytes=5000))
    assert b.get_tuning()["tile_bytes"] == 32768 and get_tuning()["tile_bytes"] == 32768


def test_library_exports_every_symbol_the_header_declares():
    text = open(os.path.join(ROOT, "include", "reshard.h")).read()
    declared = set(re.findall(r"\b(reshard_[a-z_0-9]+)\s*\(", text))
    assert declared == set(binding.EXPORTS)
    l = binding.lib()
    for name in sorted(declared):
        assert getattr(l, name) is not None


def test_a_plain_c_client_sees_what_the_binding_sees(tmp_path):
    """reshard.h is C99, and a C program that uses nothing but the header gets the same
    answers as the ctypes binding (host-side calls only)."""
    libdir = os.path.join(ROOT, "paper_2507_19017_amd")
    exe = str(tmp_path / "c_abi_client")
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I" + os.path.join(ROOT, "include"),
                           os.path.join(ROOT, "tests", "c_abi_client.c"), "-o", exe, "-L" + libdir, "-l:libreshard.so",
                           "-Wl,-rpath," + libdir])
    out = subprocess.run([exe], check=True, capture_output=True, text=True).stdout
    got = {}
    for line in out.splitlines():
        k, *v = line.split()
        got.setdefault(k, []).append(v)
    w = WORKLOADS["C0"]
    plan = Plan(w["spec"], w["src"], w["dst"])
    info = plan.info()
    assert got["create_null_out"] == [[str(binding.ERR_INVALID_ARG), "1"]]
    assert got["create_tp3"] == [[str(binding.ERR_UNSUPPORTED), "1"]]
    assert got["create_bad_size"] == [[str(binding.ERR_INVALID_ARG)]]
    assert got["create"] == [["0"]] and got["destroy"] == [["0"]]
    assert got["num_bufs"] == [["0", "2"], ["1", "1"]]
    want_bufs = [[str(s), str(b), str(n), str(int(u))] for s in (0, 1)
                 for b, (n, u) in enumerate(zip(plan.buf_bytes(s), plan.buf_used(s)))]
    assert got["buf"] == want_bufs
    assert got["info"] == [["0", str(info["num_descs"]), str(info["num_tiles"]), str(info["bytes_moved"])]]
    d0 = plan.descs()[0]
    assert got["desc0"] == [["0"] + [str(d0[k]) for k in ("src_buf", "dst_buf", "src_off", "dst_off", "rows", "row_bytes")]]
    assert got["desc_out_of_range"] == [[str(binding.ERR_INVALID_ARG)]]
    assert got["class_bytes"] == [["0"] + [str(plan.class_bytes(1)[k]) for k in "TEC"]]
    assert got["mem_stats"] == [["0", "0", "0", "0"]]
    assert got["swap_out_unbound"] == [[str(binding.ERR_BAD_STATE)]] and got["swap_in_unbound"] == [[str(binding.ERR_BAD_STATE)]]
    assert got["tensors"] == [[str(len(plan.tensors(1)))]]
    assert got["eq3"] == [["8000000000.0"]]  # 2 * (8e9 / 4 + 4e9 / 2)
    assert got["version"][0][0] == "reshard"


def test_row_pitch_limit():
    """Row pitches are 32-bit in the tile records: 4 GiB and more is refused, just under it is planned
    with 64-bit offsets (the sanitizer build walks every tile of the same case against its buffer)."""
    under = make_spec(family="dense_gqa", L=1, H=8, nq=2, nkv=2, d=8, I=(1 << 29) - 8, V=8, elem_bytes=8)
    plan = Plan(under, make_layout(kind="train", tp=2), make_layout(kind="gen", tp=1))
    down = [d for d in plan.descs() if d["dst_stride"] == ((1 << 29) - 8) * 8]
    assert down and all(d["src_stride"] * 2 == d["dst_stride"] for d in down)
    assert max(t["dst_off"] + (t["rows"] - 1) * t["dst_stride"] for t in plan.tiles()[-64:]) > 1 << 33
    over = dict(under, I=1 << 29)
    with pytest.raises(ReshardError) as e:
        Plan(over, make_layout(kind="train", tp=2), make_layout(kind="gen", tp=1))
    assert e.value.code == binding.ERR_UNSUPPORTED and "4 GiB" in str(e.value)


def test_many_source_buffers_few_of_them_used():
    """The buffer limit counts the buffers a plan touches, not the ranks of the layouts: 512 expert
    ranks on the training side, of which one generation rank of eight reads 64 (plus the dense one)."""
    spec = make_spec(family="moe_gqa", L=2, H=32, nq=4, nkv=4, d=8, V=64, E=512, Ie=8)
    src = make_layout(kind="train", ep=512, expert_layout="grouped")
    dst = make_layout(kind="gen", ep=8, ep_filter=3)
    plan = Plan(spec, src, dst)
    S, D = locate.Layout(spec, src), locate.Layout(spec, dst)
    assert len(plan.buf_bytes(0)) == 513 and sum(plan.buf_used(0)) == 65
    assert plan.buf_used(0) == [i == 0 or 1 + 3 * 64 <= i < 1 + 4 * 64 for i in range(513)]
    rng = np.random.default_rng(5)
    srcb = [rng.integers(0, 256, size=n, dtype=np.uint8) for n in S.buf_bytes]
    for via in ("descs", "tiles"):
        got = [np.full(n, SENT, dtype=np.uint8) for n in D.buf_bytes]
        cnt = [np.zeros(n, dtype=np.int32) for n in D.buf_bytes]
        if via == "descs":
            run_descs(plan.descs(), srcb, got, cnt)
        else:
            run_tiles(plan.tiles(), srcb, got, cnt)
        want = [np.full(n // 2, 0xA5A5, dtype=np.uint16) if D.buffer_used(b) else None for b, n in enumerate(D.buf_bytes)]
        fast.reshard(spec, src, dst, [x.view(np.uint16) for x in srcb], want, threads=2)
        for b, w in enumerate(want):
            if w is None:
                assert not cnt[b].any()
            else:
                assert np.array_equal(got[b].view(np.uint16), w), (via, b)
    # without the filter every one of the 513 source buffers is read: over the limit
    with pytest.raises(ReshardError) as e:
        Plan(spec, src, make_layout(kind="gen", ep=8))
    assert e.value.code == binding.ERR_UNSUPPORTED


def test_plans_can_be_built_from_several_threads_at_once():
    """Plan creation keeps no shared mutable state besides the tuning (read under a lock), and the
    error message is per thread: eight threads build different plans, half of them failing on
    purpose, and each sees its own result and its own message."""
    import threading

    names = sorted(TINY)
    want = {n: Plan(TINY[n]["spec"], TINY[n]["src"], TINY[n]["dst"]).descs() for n in names}
    out = {}

    def work(k):
        res = []
        for rep in range(6):
            n = names[(k + rep) % len(names)]
            if k % 2:
                bad = dict(TINY[n]["src"], tp=7)  # no tiny shape has a head count divisible by 7
                try:
                    Plan(TINY[n]["spec"], bad, TINY[n]["dst"])
                    res.append("no error")
                except ReshardError as e:
                    res.append((e.code, "tp" in str(e)))
            else:
                res.append(Plan(TINY[n]["spec"], TINY[n]["src"], TINY[n]["dst"]).descs() == want[n])
        out[k] = res

    threads = [threading.Thread(target=work, args=(k,)) for k in range(8)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    for k in range(8):
        assert out[k] == ([(binding.ERR_UNSUPPORTED, True)] * 6 if k % 2 else [True] * 6), (k, out[k])


def test_without_a_built_library_the_binding_refuses_to_load(monkeypatch, tmp_path):
    """No fallback of any kind: with the shared library absent every call raises, and nothing
    under oracle/ is touched by the product package."""
    import sys

    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", str(tmp_path / "libreshard.so"))
    with pytest.raises(ImportError, match="not built"):
        binding.version()
    with pytest.raises(ImportError, match="not built"):
        Plan(TINY["tiny_dense"]["spec"], TINY["tiny_dense"]["src"], TINY["tiny_dense"]["dst"])
    pkg = os.path.dirname(os.path.abspath(binding.__file__))
    for name in os.listdir(pkg):
        if name.endswith(".py"):
            text = open(os.path.join(pkg, name)).read()
            assert "oracle" not in text, name + " mentions the oracle"


def test_bench_refuses_more_than_one_gpu():
    """The build is for one GPU: asked for more, the bench says so and exits before touching a device."""
    import sys

    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2", "--steps", "1", "--warmup", "0"],
                         capture_output=True, text=True, timeout=120)
    assert res.returncode != 0
    assert "one GPU" in res.stderr and res.stdout.strip() == ""


def test_rows_more_than_4_gib_apart_stay_separate_descriptors():
    """Two equal single rows of one buffer pair are stacked into one pitched descriptor only when the
    pitch fits the 32 bits a tile record holds; further apart they stay two runs (and the plan is
    accepted instead of refused for its pitch).  Heads of 2 GiB: Q1 sits 6 GiB behind Q0 in the
    fused training tensor."""
    spec = make_spec(family="dense_gqa", L=1, H=65536, nq=2, nkv=2, d=16384, I=8, V=8)
    plan = Plan(spec, make_layout(kind="train"), make_layout(kind="gen"), tuning=dict(tile_bytes=524288))
    descs = plan.descs()
    assert all(d["rows"] == 1 for d in descs)  # nothing was stacked across the 4 GiB limit
    spans = sorted((d["dst_off"], d["dst_off"] + d["row_bytes"]) for d in descs)
    assert all(a[1] <= b[0] for a, b in zip(spans, spans[1:]))  # written once
    assert sum(b - a for a, b in spans) == plan.info()["bytes_moved"] == sum(t["bytes"] for t in plan.tensors(1))
    # the same shape with heads a sixteenth the size stacks the rows as before
    small = make_spec(family="dense_gqa", L=1, H=4096, nq=2, nkv=2, d=16384, I=8, V=8)
    assert any(d["rows"] == 2 for d in Plan(small, make_layout(kind="train"), make_layout(kind="gen")).descs())
