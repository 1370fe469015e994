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
from test_plan_host import run_descs

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
