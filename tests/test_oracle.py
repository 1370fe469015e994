"""Pins for the two CPU oracles (no GPU, no product code).

Every check here holds the oracles to something outside themselves: whole-tensor
numpy constructions of both layouts, exact counting of writes, closed-form byte
totals (which for the dense shapes are the public parameter counts of the models
the paper trains), invariants (identity, round trip) and planted mistakes.
"""

import json
import os

import numpy as np
import pytest

import np_pack
from oracle import fast, locate
from synth_inputs import TINY, WORKLOADS, make_layout

DT = {1: np.uint8, 2: np.uint16, 4: np.uint32, 8: np.uint64}
SENT = {1: 0xA5, 2: 0xA5A5, 4: 0xA5A5A5A5, 8: 0xA5A5A5A5A5A5A5A5}


def with_eb(spec, eb):
    s = dict(spec)
    s["elem_bytes"] = eb
    return s


def sentinel_bufs(sizes, used, eb):
    return [np.full(n // eb, SENT[eb], dtype=DT[eb]) if u else None for n, u in zip(sizes, used)]


def tag_logical(spec, dtype=np.uint64):
    """Every logical element carries its own identity: tensor#, row, col."""
    out = {}
    for i, (name, layer, expert, R, C) in enumerate(locate.logical_tensors(spec)):
        r, c = np.divmod(np.arange(R * C, dtype=np.uint64), np.uint64(C))
        out[(name, layer, expert)] = ((np.uint64(i + 1) << np.uint64(40)) | (r << np.uint64(20)) | c).reshape(R, C)
    return out


def run_both(spec, src_lay, dst_lay, src):
    """Run definition and loop oracle from sentinel-filled destinations."""
    eb = spec["elem_bytes"]
    D = locate.Layout(spec, dst_lay)
    used = [D.buffer_used(b) for b in range(D.nbufs)]
    d1 = sentinel_bufs(D.buf_bytes, used, eb)
    cnt = [np.zeros_like(b) if b is not None else None for b in d1]
    read = locate.reshard_definition(spec, src_lay, dst_lay, src, d1, cnt)
    d2 = sentinel_bufs(D.buf_bytes, used, eb)
    nbytes = fast.reshard(spec, src_lay, dst_lay, src, d2, threads=3)
    return d1, d2, cnt, read, nbytes, used


# ---------------------------------------------------------------- tracing ----
@pytest.mark.parametrize("name", sorted(TINY))
def test_tiny_every_element_traced_against_numpy_layouts(name):
    """Tag every element, build the source buffers with numpy library calls,
    reshard with both oracles, and require the result to equal the numpy
    construction of the destination layout, pads included."""
    w = TINY[name]
    spec = with_eb(w["spec"], 8)
    lg = tag_logical(spec)
    src = np_pack.pack(spec, w["src"], lg, np.uint64, SENT[8])
    want = np_pack.pack(spec, w["dst"], lg, np.uint64, SENT[8])
    d1, d2, cnt, read, nbytes, used = run_both(spec, w["src"], w["dst"], src)
    total = 0
    for b, u in enumerate(used):
        if not u:
            assert d1[b] is None
            continue
        assert np.array_equal(d1[b], want[b]), f"definition oracle, buffer {b}"
        assert np.array_equal(d2[b], want[b]), f"loop oracle, buffer {b}"
        # exactly once: tensor elements written once, pad elements never
        is_pad = want[b] == SENT[8]
        assert np.all(cnt[b][~is_pad] == 1) and np.all(cnt[b][is_pad] == 0)
        total += int((~is_pad).sum()) * 8
    assert nbytes == total


@pytest.mark.parametrize("name", sorted(TINY))
@pytest.mark.parametrize("eb", [1, 2, 4])
def test_tiny_random_payload_other_element_sizes(name, eb):
    w = TINY[name]
    spec = with_eb(w["spec"], eb)
    rng = np.random.default_rng(w["seed"] + eb)
    lg = np_pack.make_logical(spec, locate.logical_tensors(spec), rng, DT[eb])
    src = np_pack.pack(spec, w["src"], lg, DT[eb], SENT[eb])
    want = np_pack.pack(spec, w["dst"], lg, DT[eb], SENT[eb])
    d1, d2, _, _, _, used = run_both(spec, w["src"], w["dst"], src)
    for b, u in enumerate(used):
        if u:
            assert np.array_equal(d1[b], want[b])
            assert np.array_equal(d2[b], want[b])


def test_toy_config_against_numpy_layouts():
    """The smallest task workload (toy dense TP2 -> TP1), bf16-sized payload."""
    w = WORKLOADS["C0"]
    spec = w["spec"]
    rng = np.random.default_rng(w["seed"])
    lg = np_pack.make_logical(spec, locate.logical_tensors(spec), rng, np.uint16)
    src = np_pack.pack(spec, w["src"], lg, np.uint16, SENT[2])
    want = np_pack.pack(spec, w["dst"], lg, np.uint16, SENT[2])
    d1, d2, cnt, read, nbytes, _ = run_both(spec, w["src"], w["dst"], src)
    assert np.array_equal(d1[0], want[0]) and np.array_equal(d2[0], want[0])
    assert read == {0, 1}
    assert nbytes == 3951104 == want[0].size * 2  # no pad: every tensor is a multiple of 256 B


# ------------------------------------------------ special cases = library ----
def test_column_parallel_merge_is_concatenate_axis0():
    """gate/up and vocab rows: TP4 -> TP1 must equal np.concatenate(axis=0)."""
    w = TINY["tiny_dense"]
    spec = with_eb(w["spec"], 4)
    src_lay = make_layout(kind="train", tp=4, pp=1)
    dst_lay = make_layout(kind="train", tp=1, pp=1)
    S, D = locate.Layout(spec, src_lay), locate.Layout(spec, dst_lay)
    rng = np.random.default_rng(5)
    src = [rng.integers(0, 2**32, size=n // 4, dtype=np.uint32) for n in S.buf_bytes]
    dst = sentinel_bufs(D.buf_bytes, [True], 4)
    fast.reshard(spec, src_lay, dst_lay, src, dst)
    H, I, V = spec["H"], spec["I"], spec["V"]

    def view(bufs, lay_obj, b, name, layer, rows, cols):
        off = lay_obj.dense_off[0][(name, layer)] // 4
        return bufs[b][off:off + rows * cols].reshape(rows, cols)

    for l in range(spec["L"]):
        shards = [view(src, S, t, "gate_up", l, 2 * I // 4, H) for t in range(4)]
        gate = np.concatenate([s[:I // 4] for s in shards], axis=0)
        up = np.concatenate([s[I // 4:] for s in shards], axis=0)
        got = view(dst, D, 0, "gate_up", l, 2 * I, H)
        assert np.array_equal(got, np.concatenate([gate, up], axis=0))
        # row-parallel merge is concatenate along axis 1
        dn = np.concatenate([view(src, S, t, "down", l, H, I // 4) for t in range(4)], axis=1)
        assert np.array_equal(view(dst, D, 0, "down", l, H, I), dn)
        wo_w = spec["nq"] * spec["d"]
        wo = np.concatenate([view(src, S, t, "wo", l, H, wo_w // 4) for t in range(4)], axis=1)
        assert np.array_equal(view(dst, D, 0, "wo", l, H, wo_w), wo)
    emb = np.concatenate([view(src, S, t, "emb", -1, V // 4, H) for t in range(4)], axis=0)
    assert np.array_equal(view(dst, D, 0, "emb", -1, V, H), emb)


def test_qkv_deinterleave_is_reshape_and_split():
    """TRAIN TP2 -> GEN TP1: the fused [nkv/T, g+2, d, H] blocks split into Q|K|V."""
    w = TINY["tiny_dense"]
    spec = with_eb(w["spec"], 2)
    src_lay = make_layout(kind="train", tp=2, pp=1)
    dst_lay = make_layout(kind="gen", tp=1)
    S, D = locate.Layout(spec, src_lay), locate.Layout(spec, dst_lay)
    rng = np.random.default_rng(6)
    src = [rng.integers(0, 2**16, size=n // 2, dtype=np.uint16) for n in S.buf_bytes]
    dst = sentinel_bufs(D.buf_bytes, [True], 2)
    fast.reshard(spec, src_lay, dst_lay, src, dst)
    H, nq, nkv, d = spec["H"], spec["nq"], spec["nkv"], spec["d"]
    g = nq // nkv
    for l in range(spec["L"]):
        for stored, width in (("qkv_w", H), ("qkv_b", 1)):
            blocks = []
            for t in range(2):
                off = S.dense_off[0][(stored, l)] // 2
                n = (nkv // 2) * (g + 2) * d * width
                blocks.append(src[t][off:off + n].reshape(nkv // 2, g + 2, d, width))
            fused = np.concatenate(blocks, axis=0)  # [nkv, g+2, d, width]
            q = fused[:, :g].reshape(nq * d, width)
            k = fused[:, g].reshape(nkv * d, width)
            v = fused[:, g + 1].reshape(nkv * d, width)
            off = D.dense_off[0][(stored, l)] // 2
            got = dst[0][off:off + (nq + 2 * nkv) * d * width].reshape(-1, width)
            assert np.array_equal(got, np.concatenate([q, k, v], axis=0))


def test_grouped_experts_to_generation_is_transpose():
    """grouped [expert][in][out] -> generation [expert][out][in] is transpose(0, 2, 1)."""
    w = TINY["tiny_moe_grouped"]
    spec = with_eb(w["spec"], 2)
    src_lay = make_layout(kind="train", tp=1, pp=1, ep=2, expert_layout="grouped")
    dst_lay = make_layout(kind="gen", tp=1, ep=2)
    S, D = locate.Layout(spec, src_lay), locate.Layout(spec, dst_lay)
    rng = np.random.default_rng(7)
    src = [rng.integers(0, 2**16, size=n // 2, dtype=np.uint16) for n in S.buf_bytes]
    dst = sentinel_bufs(D.buf_bytes, [True] * D.nbufs, 2)
    fast.reshard(spec, src_lay, dst_lay, src, dst)
    H, Ie, El = spec["H"], spec["Ie"], spec["E"] // 2
    for x in range(2):
        for l in range(spec["L"]):
            o1 = S.expert_off[0][("w1", l, -1)] // 2
            o2 = S.expert_off[0][("w2", l, -1)] // 2
            w1 = src[1 + x][o1:o1 + El * H * 2 * Ie].reshape(El, H, 2 * Ie)
            w2 = src[1 + x][o2:o2 + El * Ie * H].reshape(El, Ie, H)
            p13 = D.expert_off[0][("w13", l, -1)] // 2
            p2 = D.expert_off[0][("w2", l, -1)] // 2
            assert np.array_equal(dst[1 + x][p13:p13 + w1.size].reshape(El, 2 * Ie, H), w1.transpose(0, 2, 1))
            assert np.array_equal(dst[1 + x][p2:p2 + w2.size].reshape(El, H, Ie), w2.transpose(0, 2, 1))


def test_pipeline_merge_same_tp_is_concatenation_of_stage_buffers():
    """TRAIN TP2 PP2 -> TRAIN TP2 PP1: with every tensor a multiple of 256 B the
    destination buffer of rank t is stage-0 buffer then stage-1 buffer."""
    spec = dict(WORKLOADS["C0"]["spec"])
    src_lay = make_layout(kind="train", tp=2, pp=2)
    dst_lay = make_layout(kind="train", tp=2, pp=1)
    S, D = locate.Layout(spec, src_lay), locate.Layout(spec, dst_lay)
    rng = np.random.default_rng(8)
    lg = np_pack.make_logical(spec, locate.logical_tensors(spec), rng, np.uint16)
    src = np_pack.pack(spec, src_lay, lg, np.uint16, SENT[2])  # equal replicas
    dst = sentinel_bufs(D.buf_bytes, [True, True], 2)
    fast.reshard(spec, src_lay, dst_lay, src, dst)
    for t in range(2):
        assert np.array_equal(dst[t], np.concatenate([src[t], src[2 + t]]))


# -------------------------------------------------------------- invariants ----
@pytest.mark.parametrize("name", sorted(TINY) + ["C0"])
def test_identity_when_source_equals_destination(name):
    w = {**TINY, **WORKLOADS}[name]
    spec = with_eb(w["spec"], 2)
    lay = w["src"]
    S = locate.Layout(spec, lay)
    rng = np.random.default_rng(11)
    lg = np_pack.make_logical(spec, locate.logical_tensors(spec), rng, np.uint16)
    src = np_pack.pack(spec, lay, lg, np.uint16, SENT[2])  # equal replicas, sentinel pads
    dst = sentinel_bufs(S.buf_bytes, [True] * S.nbufs, 2)
    fast.reshard(spec, lay, lay, src, dst, threads=2)
    for a, b in zip(src, dst):
        assert np.array_equal(a, b)


@pytest.mark.parametrize("name", sorted(TINY) + ["C0"])
def test_round_trip_train_gen_train(name):
    w = {**TINY, **WORKLOADS}[name]
    spec = with_eb(w["spec"], 2)
    train = w["src"]
    gen = dict(w["dst"], tp_filter=-1, ep_filter=-1)  # a round trip needs every rank
    S, G = locate.Layout(spec, train), locate.Layout(spec, gen)
    rng = np.random.default_rng(12)
    lg = np_pack.make_logical(spec, locate.logical_tensors(spec), rng, np.uint16)
    src = np_pack.pack(spec, train, lg, np.uint16, SENT[2])
    mid = sentinel_bufs(G.buf_bytes, [True] * G.nbufs, 2)
    fast.reshard(spec, train, gen, src, mid, threads=2)
    back = sentinel_bufs(S.buf_bytes, [True] * S.nbufs, 2)
    fast.reshard(spec, gen, train, mid, back, threads=2)
    for a, b in zip(src, back):
        assert np.array_equal(a, b)
    # and through the definition oracle as well
    mid2 = sentinel_bufs(G.buf_bytes, [True] * G.nbufs, 2)
    locate.reshard_definition(spec, train, gen, src, mid2)
    for a, b in zip(mid, mid2):
        assert np.array_equal(a, b)


def test_replicated_tensors_are_read_from_tensor_rank_zero():
    """Make the replicas of the common weights differ: the destination must
    carry rank 0's copy on every rank."""
    w = TINY["tiny_moe"]
    spec = with_eb(w["spec"], 2)
    S, D = locate.Layout(spec, w["src"]), locate.Layout(spec, w["dst"])
    src = [np.full(n // 2, 100 + b, dtype=np.uint16) for b, n in enumerate(S.buf_bytes)]
    for maker in ("definition", "loop"):
        dst = sentinel_bufs(D.buf_bytes, [True] * D.nbufs, 2)
        if maker == "definition":
            locate.reshard_definition(spec, w["src"], w["dst"], src, dst)
        else:
            fast.reshard(spec, w["src"], w["dst"], src, dst)
        for name, layer, j, off, nbytes in D.stored[0]:
            if name in locate.REPLICATED:
                assert np.all(dst[0][off // 2:(off + nbytes) // 2] == 100), name


# ------------------------------------------------------------ closed forms ----
def logical_bytes(spec):
    return sum(R * C for *_, R, C in locate.logical_tensors(spec)) * spec["elem_bytes"]


GOLDEN = json.load(open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "paper_values.json")))


def test_byte_totals_match_public_parameter_counts():
    """bf16 bytes of the Qwen2.5-7B / 32B shapes are twice the models' public
    parameter counts (tests/golden/paper_values.json)."""
    params = GOLDEN["public_parameter_counts"]
    assert logical_bytes(WORKLOADS["C1"]["spec"]) == 2 * params["Qwen2.5-7B"] == 15_231_233_024
    assert logical_bytes(WORKLOADS["C2"]["spec"]) == 2 * params["Qwen2.5-32B"] == 65_527_752_704
    assert logical_bytes(WORKLOADS["C0"]["spec"]) == 3_951_104
    # Qwen3-30B-A3B: its parameters minus the per-layer q/k norm vectors
    # (2 x 128 per layer x 48 layers) that this shape leaves out.
    assert logical_bytes(WORKLOADS["C3"]["spec"]) == 2 * (params["Qwen3-30B-A3B"] - 48 * 256) == 61_064_220_672


def test_redundant_memory_formula_gives_the_papers_order_of_magnitude():
    """Eq. (3): R = GDP * (TW / UTP + EW / GEP).  With the Qwen3-MoE-30B shape split into
    TP weights (everything but the routed experts) and EP weights (the routed experts),
    any setting with GDP == GEP and GDP >= UTP gives more than the paper's 60 GB."""
    spec = WORKLOADS["C3"]["spec"]
    ew = sum(R * C for n, *_, R, C in locate.logical_tensors(spec) if n.startswith("ex_")) * 2 / 1e9
    tw = logical_bytes(spec) / 1e9 - ew
    assert abs(ew - 57.98) < 0.01 and abs(tw - 3.08) < 0.01
    low = GOLDEN["redundant_memory_qwen3_moe_30b_lower_bound_gb"]["value"]
    for utp, gdp in ((1, 1), (2, 2), (2, 4), (4, 4), (4, 8)):
        assert gdp * (tw / utp + ew / gdp) > low


def test_per_device_share_of_the_32b_model_is_about_8_gb():
    """Ablation study, memory profiling of Qwen2.5-32B TP8 -> TP4: about 8 GB is
    released per device, i.e. one TP8 share of the update weights."""
    w = WORKLOADS["C2"]
    S = locate.Layout(w["spec"], w["src"])
    per_tp_rank = [sum(S.buf_bytes[p * 8 + t] for p in range(4)) for t in range(8)]
    printed = GOLDEN["released_gb_per_device_qwen25_32b_tp8_to_tp4"]["value"]
    assert all(round(n / 1e9) == printed for n in per_tp_rank)
    assert all(7.9e9 < n < 8.4e9 for n in per_tp_rank)
    assert abs(sum(per_tp_rank) - 65_527_752_704) < 16e6  # replicated norms + padding only


@pytest.mark.parametrize("name", ["C0", "C1", "C2", "C3", "C3P", "C4"])
def test_destination_bytes_closed_form(name):
    """Destination tensor bytes = logical bytes held by the kept ranks, counting
    replicated (common) weights once per kept tensor rank."""
    w = WORKLOADS[name]
    spec, dl = w["spec"], w["dst"]
    D = locate.Layout(spec, dl)
    eb = spec["elem_bytes"]
    want = 0
    for tname, layer, expert, R, C in locate.logical_tensors(spec):
        n = R * C * eb
        if tname in locate.REPLICATED:
            want += n * (1 if dl["tp_filter"] >= 0 else dl["tp"])
        elif tname.startswith("ex_"):
            x = expert // (spec["E"] // dl["ep"])
            want += n if dl["ep_filter"] in (-1, x) else 0
        else:
            want += n if dl["tp_filter"] < 0 else n // dl["tp"]
    got = sum(nb for b in range(D.nbufs) if D.buffer_used(b) for _, nb in D.owned(b))
    assert got == want
    if name == "C4":
        assert got == 26_276_528_128


def test_buffer_tables_agree_between_oracles():
    for w in list(TINY.values()) + list(WORKLOADS.values()):
        for lay in (w["src"], w["dst"]):
            L = locate.Layout(w["spec"], lay)
            assert fast.buffer_sizes(w["spec"], lay) == L.buf_bytes
            assert fast.buffers_used(w["spec"], lay) == [L.buffer_used(b) for b in range(L.nbufs)]


def test_source_buffers_read_under_a_rank_filter():
    """One rank of EP2 from EP8 sources: only the dense buffers of tensor rank 0
    (common weights) and both ranks (split weights), and 4 of 8 expert buffers."""
    w = TINY["tiny_mla"]
    spec = with_eb(w["spec"], 2)
    S, D = locate.Layout(spec, w["src"]), locate.Layout(spec, w["dst"])
    src = [np.zeros(n // 2, dtype=np.uint16) for n in S.buf_bytes]
    dst = sentinel_bufs(D.buf_bytes, [D.buffer_used(b) for b in range(D.nbufs)], 2)
    read = locate.reshard_definition(spec, w["src"], w["dst"], src, dst)
    assert read == {0, 1, 2 + 4, 2 + 5, 2 + 6, 2 + 7}


# -------------------------------------------------------- planted mistakes ----
@pytest.mark.parametrize("mistake", ["kv_order", "gate_up_order", "row_vs_col", "grouped_not_transposed"])
def test_planted_mistakes_in_the_layout_are_caught(mistake, monkeypatch):
    """Plant a plausible mistake in the definition oracle's layout function and
    check that the numpy-layout pin notices."""
    name = "tiny_moe_grouped" if mistake == "grouped_not_transposed" else "tiny_dense"
    w = TINY[name]
    spec = with_eb(w["spec"], 8)
    lg = tag_logical(spec)
    src = np_pack.pack(spec, w["src"], lg, np.uint64, SENT[8])
    want = np_pack.pack(spec, w["dst"], lg, np.uint64, SENT[8])
    orig = locate.Layout.place

    def bad(self, tname, layer, expert, r, c):
        if mistake == "kv_order" and self.kind == "train" and tname in ("wk", "wv"):
            tname = {"wk": "wv", "wv": "wk"}[tname]
        if mistake == "gate_up_order" and self.kind == "gen" and tname in ("w_gate", "w_up"):
            tname = {"w_gate": "w_up", "w_up": "w_gate"}[tname]
        if mistake == "row_vs_col" and self.kind == "gen" and tname == "w_down":
            # pretend down-projection is split by rows instead of columns
            n = self.spec["H"] // self.T
            I = self.spec["I"]
            r = np.asarray(r); c = np.asarray(c)
            return [(r // n, self.dense_off[0][("down", layer)] + ((r % n) * I + c) * 8)]
        if mistake == "grouped_not_transposed" and self.grouped and tname.startswith("ex_"):
            self = locate.Layout(self.spec, dict(self.lay, expert_layout="per_expert"))
        return orig(self, tname, layer, expert, r, c)

    monkeypatch.setattr(locate.Layout, "place", bad)
    D = locate.Layout(spec, w["dst"])
    used = [D.buffer_used(b) for b in range(D.nbufs)]
    dst = sentinel_bufs(D.buf_bytes, used, 8)
    try:
        locate.reshard_definition(spec, w["src"], w["dst"], src, dst)
    except Exception:
        return  # an out-of-range write is also a detection
    assert any(u and not np.array_equal(dst[b], want[b]) for b, u in enumerate(used))


def test_invalid_shapes_are_rejected():
    spec = dict(WORKLOADS["C0"]["spec"])
    with pytest.raises(ValueError):
        fast.buffer_sizes(spec, make_layout(kind="train", tp=3))
    with pytest.raises(ValueError):
        fast.buffer_sizes(spec, make_layout(kind="gen", tp=1, pp=2))
    # KV heads neither divide nor are divided by the tensor ranks
    odd = dict(spec, nq=12, nkv=4, H=768)
    with pytest.raises(ValueError):
        fast.buffer_sizes(odd, make_layout(kind="train", tp=6))
    with pytest.raises(AssertionError):
        locate.Layout(odd, make_layout(kind="train", tp=6))
    # pipeline shapes
    for bad in (dict(pp=2, vpp=2, first_stage_layers=1, last_stage_layers=1), dict(pp=2, vpp=3),
                dict(pp=2, first_stage_layers=1, last_stage_layers=2), dict(pp=1, first_stage_layers=1, last_stage_layers=1)):
        with pytest.raises(ValueError):
            fast.buffer_sizes(spec, make_layout(kind="train", tp=2, **bad))
        with pytest.raises(AssertionError):
            locate.Layout(spec, make_layout(kind="train", tp=2, **bad))


def test_replicated_kv_heads_and_tied_embedding_are_read_from_their_first_copy():
    """KV heads shared by T/nkv ranks are read from the lowest such rank; a tied embedding
    from the first stage.  Source buffers hold their own index, so the origin shows."""
    w = TINY["tiny_kvrep"]
    spec = with_eb(w["spec"], 2)
    gen1 = make_layout(kind="gen", tp=1)
    S, D = locate.Layout(spec, w["src"]), locate.Layout(spec, gen1)
    src = [np.full(n // 2, 100 + b, dtype=np.uint16) for b, n in enumerate(S.buf_bytes)]
    for maker in ("definition", "loop"):
        dst = sentinel_bufs(D.buf_bytes, [True], 2)
        if maker == "definition":
            locate.reshard_definition(spec, w["src"], gen1, src, dst)
        else:
            fast.reshard(spec, w["src"], gen1, src, dst)
        H, nq, nkv, d = spec["H"], spec["nq"], spec["nkv"], spec["d"]
        for l in range(spec["L"]):
            p = S.layer_stage[l]
            off = D.dense_off[0][("qkv_w", l)] // 2
            blk = dst[0][off:off + (nq + 2 * nkv) * d * H].reshape(-1, H)
            k, v = blk[nq * d:(nq + nkv) * d], blk[(nq + nkv) * d:]
            for head in range(nkv):  # 4 ranks, 2 KV heads: head h is read from rank 2h of its stage
                assert np.all(k[head * d:(head + 1) * d] == 100 + p * 4 + 2 * head)
                assert np.all(v[head * d:(head + 1) * d] == 100 + p * 4 + 2 * head)
        off = D.dense_off[0][("emb", -1)] // 2
        emb = dst[0][off:off + spec["V"] * H].reshape(4, -1)
        assert [int(x[0]) for x in emb] == [100, 101, 102, 103] and all(np.all(x == x[0]) for x in emb)


def test_virtual_pipeline_and_uneven_stage_assignment():
    """Interleaved chunks: with 8 layers, 2 stages, 2 chunks per stage, stage 0 stores layers
    0, 1, 4, 5.  Uneven: 3 + 2 + 2 + 1."""
    a = locate.Layout(TINY["tiny_kvrep"]["spec"], TINY["tiny_kvrep"]["src"])
    assert a.stage_layers == [[0, 1, 4, 5], [2, 3, 6, 7]]
    b = locate.Layout(TINY["tiny_uneven"]["spec"], TINY["tiny_uneven"]["src"])
    assert b.stage_layers == [[0, 1, 2], [3, 4], [5, 6], [7]]
    # storage order inside a stage follows that list
    names = [(n, l) for (n, l, j, off, nb) in a.stored[0] if n == "ln1"]
    assert names == [("ln1", 0), ("ln1", 1), ("ln1", 4), ("ln1", 5)]
