"""Random small workloads through every formulation at once (no GPU).

For each seed: the logical tensors are packed into the source layout with whole-tensor
numpy calls (np_pack), resharded by the definition oracle, by the loop oracle and by an
interpreter of the product's descriptor table, and each result must equal the numpy
construction of the destination layout, pads included.  The cases draw every layout
option the library accepts (KV-head replication, interleaved and uneven pipeline stages,
tied and padded vocabularies, expert tensor parallelism, grouped experts, rank filters,
training-to-training pairs, all element sizes)."""

import numpy as np
import pytest

import np_pack
from oracle import fast, locate
from paper_2507_19017_amd import Plan
from synth_inputs import random_case
from test_oracle import DT, SENT, run_both
from test_plan_host import run_descs, run_tiles

SEEDS = list(range(160))


@pytest.mark.parametrize("seed", SEEDS)
def test_random_case_agrees_across_all_formulations(seed):
    w = random_case(seed)
    spec, eb = w["spec"], w["spec"]["elem_bytes"]
    rng = np.random.default_rng(w["seed"])
    lg = np_pack.make_logical(spec, locate.logical_tensors(spec), rng, DT[eb])
    src = np_pack.pack(spec, w["src"], lg, DT[eb], SENT[eb])
    want = np_pack.pack(spec, w["dst"], lg, DT[eb], SENT[eb])
    d1, d2, cnt, _, nbytes, used = run_both(spec, w["src"], w["dst"], src)
    plan = Plan(spec, w["src"], w["dst"])
    assert plan.buf_bytes(0) == [s.nbytes for s in src] == fast.buffer_sizes(spec, w["src"])
    assert plan.buf_bytes(1) == [x.nbytes for x in want]
    assert plan.buf_used(1) == used
    d3 = [np.full(x.nbytes, SENT[1], dtype=np.uint8) for x in want]
    c3 = [np.zeros(x.nbytes, dtype=np.int32) for x in want]
    run_descs(plan.descs(), [s.view(np.uint8) for s in src], d3, c3)
    total = 0
    for b, u in enumerate(used):
        if not u:
            assert d1[b] is None and not c3[b].any()
            continue
        assert np.array_equal(d1[b], want[b]), f"definition oracle, buffer {b}"
        assert np.array_equal(d2[b], want[b]), f"loop oracle, buffer {b}"
        assert np.array_equal(d3[b].view(DT[eb]), want[b]), f"descriptor table, buffer {b}"
        total += int(cnt[b].sum()) * eb
        assert cnt[b].max(initial=0) <= 1
        assert np.array_equal(c3[b].reshape(-1, eb)[:, 0], cnt[b].astype(np.int32)), "bytes written once, pads never"
    assert nbytes == total == plan.info()["bytes_moved"]


@pytest.mark.parametrize("seed", range(12))
def test_random_midsize_tile_tables(seed):
    """The same generator with widths scaled up, so that tensors span several tiles with ragged
    ends and the transposing descriptors reach the register-path tile shapes: the device tile
    table, interpreted on the host, against the loop oracle."""
    w = random_case(seed, 4)
    spec, eb = w["spec"], w["spec"]["elem_bytes"]
    plan = Plan(spec, w["src"], w["dst"])
    rng = np.random.default_rng(w["seed"])
    src = [rng.integers(0, 256, size=n, dtype=np.uint8) for n in plan.buf_bytes(0)]
    used = plan.buf_used(1)
    got = [np.full(n, SENT[1], dtype=np.uint8) for n in plan.buf_bytes(1)]
    cnt = [np.zeros(n, dtype=np.int32) for n in plan.buf_bytes(1)]
    run_tiles(plan.tiles(), src, got, cnt)
    want = [np.full(n // eb, SENT[eb], dtype=DT[eb]) if u else None for n, u in zip(plan.buf_bytes(1), used)]
    nbytes = fast.reshard(spec, w["src"], w["dst"], [x.view(DT[eb]) for x in src], want, threads=4)
    for b, u in enumerate(used):
        if u:
            assert np.array_equal(got[b].view(DT[eb]), want[b]), f"buffer {b}"
        else:
            assert not cnt[b].any()
    assert sum(int(c.sum()) for c in cnt) == nbytes and max(int(c.max(initial=0)) for c in cnt) <= 1
