"""The paper's closed forms against the values it prints (tests/golden/paper_values.json)."""

import json
import os

import pytest

from paper_2507_19017_amd import dataflow_model as m

GOLDEN = json.load(open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "paper_values.json")))


def printed_close(got, printed: str):
    """Equal to what the table prints, to one unit of its last printed digit (the table
    truncates some entries and rounds others)."""
    scale = 1000.0 if printed.endswith("K") else 1.0
    digits = printed.rstrip("K")
    unit = scale * (10.0 ** -len(digits.split(".")[1]) if "." in digits else 1.0)
    return abs(got - float(digits) * scale) <= unit


@pytest.mark.parametrize("row", GOLDEN["table1_replay_buffer_volume"]["rows"])
def test_eq2_reproduces_table_1(row):
    G, N, PL, n, SL, M, tcv, t100, t1k = row
    B = GOLDEN["table1_replay_buffer_volume"]["B"]
    v = m.tcv_gb(G, N, B, PL, n, SL, M)
    assert printed_close(v, tcv)
    assert printed_close(m.dispatch_seconds(v, 100), t100)
    assert printed_close(m.dispatch_seconds(v, 1024), t1k)  # the 1 GB/s column


def test_eq1_eq4_reduce_to_each_other():
    args = (256, 8, 4, 2048, 5, 8192, 3)
    # one controller-free warehouse is the centralized buffer of Eq. (2)
    assert m.td_tcv_gb(*args, C=0, S=1) == m.tcv_gb(*args)
    # S warehouses divide the volume; C controllers only add metadata scalars
    assert m.td_tcv_gb(*args, C=0, S=16) == pytest.approx(m.tcv_gb(*args) / 16)
    extra = m.td_tcv_gb(*args, C=10, S=1) - m.tcv_gb(*args)
    assert extra == pytest.approx(256 * 8 * 4 * 8 * 10 * 3 / 1024 ** 3)
    # Eq. (1) is one request: prompt + n response-length items + scalars
    assert m.cv_gb(*args) == 256 * 8 * 4 * (2048 + 5 * 8192 + 3) / 1024 ** 3
    assert m.cv_gb(*args) < m.tcv_gb(*args) < 3 * m.cv_gb(*args) + 1e-3


def test_eq3_matches_the_library():
    from paper_2507_19017_amd import redundant_memory_bytes
    assert m.redundant_memory_gb(4, 3.08, 4, 57.98, 4) == pytest.approx(61.06)
    assert redundant_memory_bytes(4, 3.08e9, 4, 57.98e9, 4) == pytest.approx(61.06e9)
    assert m.redundant_memory_gb(4, 3.08, 4, 57.98, 4) > GOLDEN["redundant_memory_qwen3_moe_30b_lower_bound_gb"]["value"]
