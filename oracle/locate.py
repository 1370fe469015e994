"""Definition oracle for the weight-resharding step (TEST INFRASTRUCTURE ONLY).

This file is a checker.  Nothing in the product path may import it; only the
tests, the smoke check and the benchmark's CPU-baseline leg do.

What it defines.  The resharding flow (Allgather-Swap Technique section, step 2:
every device selects and copies the weight slices it needs for generation)
moves each weight element from its place in the training-side shards to its
place in the generation-side shards, with no arithmetic.  The paper does not
print either layout; the layouts below are the Megatron-style conventions this
repository fixes (column/row tensor-parallel splits, pipeline stages, fused QKV
interleaved per KV-head group, fused gate/up, expert-parallel blocks), and the
weight classes are the paper's T (tensor-parallel), E (expert-parallel) and C
(common, replicated) weights of its redundant-memory example (Problem
Statement, Figure 3 discussion).

The result has a plain definition, written out here literally:

    for every logical weight element e:
        dst[place(DST, e)] = src[place(SRC, e)]

`Layout.place` answers "where does logical element (tensor, layer, expert,
row, col) live", by explicit index arithmetic, for ints or numpy arrays.
Parity status: pinned, by brute-force tracing, per-element write counts,
closed-form byte totals, the per-device bytes the paper's ablation prints and
numpy reshape/concatenate constructions in tests/.  The paper prints no worked
example of the mapping itself, so none of the pins is an element-level value
from the authors; the layout conventions are the public Megatron ones.
"""

from __future__ import annotations

import numpy as np

ALIGN = 256  # every stored tensor starts on a multiple of this many bytes

REPLICATED = ("ln1", "ln2", "final_ln", "router", "q_a", "q_a_ln", "kv_a", "kv_a_ln")


def _align(x: int) -> int:
    return (x + ALIGN - 1) // ALIGN * ALIGN


def check_spec(spec: dict) -> None:
    fam = spec["family"]
    assert fam in ("dense_gqa", "moe_gqa", "moe_mla"), fam
    assert spec["L"] > 0 and spec["H"] > 0 and spec["nq"] > 0
    assert spec["elem_bytes"] in (1, 2, 4, 8)
    if fam != "moe_mla":
        assert spec["nkv"] > 0 and spec["d"] > 0 and spec["nq"] % spec["nkv"] == 0
    else:
        for k in ("q_lora", "kv_lora", "nope", "rope", "v_dim"):
            assert spec[k] > 0, k
    if fam == "dense_gqa":
        assert spec["I"] > 0
    else:
        assert spec["E"] > 0 and spec["Ie"] > 0
    if spec["has_embeddings"]:
        assert spec["V"] > 0


def logical_tensors(spec: dict):
    """Every logical weight tensor once: (name, layer, expert, rows, cols).

    Matrices are row-major [out, in].  Biases are [out, 1]; norm vectors are
    [1, width].  layer / expert are -1 where they do not apply.
    """
    fam = spec["family"]
    H, L = spec["H"], spec["L"]
    out = []
    if spec["has_embeddings"]:
        out.append(("emb", -1, -1, spec["V"], H))
    for l in range(L):
        out.append(("ln1", l, -1, 1, H))
        if fam == "moe_mla":
            nq = spec["nq"]
            out.append(("q_a", l, -1, spec["q_lora"], H))
            out.append(("q_a_ln", l, -1, 1, spec["q_lora"]))
            out.append(("q_b", l, -1, nq * (spec["nope"] + spec["rope"]), spec["q_lora"]))
            out.append(("kv_a", l, -1, spec["kv_lora"] + spec["rope"], H))
            out.append(("kv_a_ln", l, -1, 1, spec["kv_lora"]))
            out.append(("kv_b", l, -1, nq * (spec["nope"] + spec["v_dim"]), spec["kv_lora"]))
            out.append(("wo", l, -1, H, nq * spec["v_dim"]))
        else:
            nq, nkv, d = spec["nq"], spec["nkv"], spec["d"]
            out.append(("wq", l, -1, nq * d, H))
            out.append(("wk", l, -1, nkv * d, H))
            out.append(("wv", l, -1, nkv * d, H))
            if spec["qkv_bias"]:
                out.append(("bq", l, -1, nq * d, 1))
                out.append(("bk", l, -1, nkv * d, 1))
                out.append(("bv", l, -1, nkv * d, 1))
            out.append(("wo", l, -1, H, nq * d))
        out.append(("ln2", l, -1, 1, H))
        if fam == "dense_gqa":
            I = spec["I"]
            out.append(("w_gate", l, -1, I, H))
            out.append(("w_up", l, -1, I, H))
            out.append(("w_down", l, -1, H, I))
        else:
            E, Ie = spec["E"], spec["Ie"]
            out.append(("router", l, -1, E, H))
            if spec["n_shared"]:
                Is = spec["n_shared"] * Ie
                out.append(("sh_gate", l, -1, Is, H))
                out.append(("sh_up", l, -1, Is, H))
                out.append(("sh_down", l, -1, H, Is))
            for e in range(E):
                out.append(("ex_gate", l, e, Ie, H))
                out.append(("ex_up", l, e, Ie, H))
                out.append(("ex_down", l, e, H, Ie))
    if spec["has_embeddings"]:
        out.append(("final_ln", -1, -1, 1, H))
        if not spec.get("tied_embeddings", 0):
            out.append(("lm_head", -1, -1, spec["V"], H))
    return out


class Layout:
    """One side of the resharding: a set of flat buffers and where tensors sit.

    Dense buffers come first, one per (pipeline stage p, tensor rank t), index
    p*T + t; expert buffers follow, one per (p, expert rank x), index
    nd + p*X + x.  A generation layout has a single stage.
    """

    def __init__(self, spec: dict, lay: dict):
        check_spec(spec)
        self.spec, self.lay = spec, lay
        self.kind = lay["kind"]
        assert self.kind in ("train", "gen")
        self.T, self.P, self.X = lay["tp"], lay["pp"], lay["ep"]
        self.grouped = self.kind == "train" and lay["expert_layout"] == "grouped"
        self.moe = spec["family"] != "dense_gqa"
        T, P, X = self.T, self.P, self.X
        assert T >= 1 and P >= 1 and X >= 1
        if self.kind == "gen":
            assert P == 1
        assert spec["nq"] % T == 0
        if spec["family"] != "moe_mla":
            # fewer KV heads than tensor ranks: every KV head is replicated on T/nkv ranks
            assert spec["nkv"] % T == 0 or T % spec["nkv"] == 0
        if spec["family"] == "dense_gqa":
            assert spec["I"] % T == 0
            assert X == 1
        else:
            assert spec["E"] % X == 0
            assert (spec["n_shared"] * spec["Ie"]) % T == 0
        # rows of the embedding / lm_head before the tensor-parallel split: V, or V padded up
        self.Vp = lay.get("vocab_padded", 0) or spec["V"]
        if spec["has_embeddings"]:
            assert self.Vp >= spec["V"] and self.Vp % T == 0
        # expert tensor parallelism: 1 = whole experts, T = every expert split over the tensor
        # ranks like a dense feed-forward (gate/up by rows, down by columns)
        self.Y = lay.get("etp", 1) if self.moe else 1
        assert self.Y in (1, T)
        if self.moe:
            assert spec["Ie"] % self.Y == 0
        self.nd = P * T
        self.ne = P * X * self.Y if self.moe else 0
        self.nbufs = self.nd + self.ne
        self.tied = bool(spec.get("tied_embeddings", 0)) and bool(spec["has_embeddings"])
        self.stage_layers = self._assign_layers()
        self.layer_stage = {l: p for p, ls in enumerate(self.stage_layers) for l in ls}
        self._walk()

    def _assign_layers(self):
        """Layers of every stage, in storage order.

        Even split: contiguous blocks.  Virtual pipeline size v: the layers are cut
        into P*v chunks; chunk c lives on stage c mod P, chunks of a stage stored in
        chunk order.  Uneven split: the first / last stage hold the given numbers of
        layers, the stages between share the rest evenly."""
        L, P = self.spec["L"], self.P
        v = self.lay.get("vpp", 1)
        first, last = self.lay.get("first_stage_layers", 0), self.lay.get("last_stage_layers", 0)
        if first or last:
            assert v == 1 and P >= 2 and first > 0 and last > 0
            mid = L - first - last
            if P == 2:
                assert mid == 0
                counts = [first, last]
            else:
                assert mid > 0 and mid % (P - 2) == 0
                counts = [first] + [mid // (P - 2)] * (P - 2) + [last]
            out, at = [], 0
            for n in counts:
                out.append(list(range(at, at + n)))
                at += n
            return out
        assert v >= 1 and L % (P * v) == 0
        lc = L // (P * v)
        return [[l for k in range(v) for l in range((k * P + p) * lc, (k * P + p + 1) * lc)] for p in range(P)]

    # ---- which buffers a filtered layout really holds -------------------
    def buffer_used(self, b: int) -> bool:
        tf, ef = self.lay["tp_filter"], self.lay["ep_filter"]
        if b < self.nd:
            return tf < 0 or b % self.T == tf
        # expert buffer (stage, expert rank x, expert-tensor rank y): index nd + (p*X + x)*Y + y
        x, y = (b - self.nd) // self.Y % self.X, (b - self.nd) % self.Y
        return (ef < 0 or x == ef) and (self.Y == 1 or tf < 0 or y == tf)

    # ---- in-buffer order and offsets --------------------------------------
    def _dense_sequence(self, p: int):
        """(stored name, layer, element count) in storage order for stage p."""
        s, T = self.spec, self.T
        H, fam = s["H"], s["family"]
        seq = []
        if s["has_embeddings"] and p == 0:
            seq.append(("emb", -1, self.Vp // T * H))
        for l in self.stage_layers[p]:
            seq.append(("ln1", l, H))
            if fam == "moe_mla":
                nql = s["nq"] // T
                seq.append(("q_a", l, s["q_lora"] * H))
                seq.append(("q_a_ln", l, s["q_lora"]))
                seq.append(("q_b", l, nql * (s["nope"] + s["rope"]) * s["q_lora"]))
                seq.append(("kv_a", l, (s["kv_lora"] + s["rope"]) * H))
                seq.append(("kv_a_ln", l, s["kv_lora"]))
                seq.append(("kv_b", l, nql * (s["nope"] + s["v_dim"]) * s["kv_lora"]))
                seq.append(("wo", l, H * nql * s["v_dim"]))
            else:
                rows = (s["nq"] // T + 2 * max(s["nkv"] // T, 1)) * s["d"]
                seq.append(("qkv_w", l, rows * H))
                if s["qkv_bias"]:
                    seq.append(("qkv_b", l, rows))
                seq.append(("wo", l, H * s["nq"] * s["d"] // T))
            seq.append(("ln2", l, H))
            if fam == "dense_gqa":
                seq.append(("gate_up", l, 2 * s["I"] // T * H))
                seq.append(("down", l, H * s["I"] // T))
            else:
                seq.append(("router", l, s["E"] * H))
                if s["n_shared"]:
                    Is = s["n_shared"] * s["Ie"]
                    seq.append(("sh_fc1", l, 2 * Is // T * H))
                    seq.append(("sh_fc2", l, H * Is // T))
        if s["has_embeddings"] and p == self.P - 1:
            seq.append(("final_ln", -1, H))
            if not self.tied:
                seq.append(("lm_head", -1, self.Vp // T * H))
            elif self.P > 1:
                # tied output layer: the last stage keeps its own copy of the embedding shard
                seq.append(("emb_tied", -1, self.Vp // T * H))
        return seq

    def _expert_sequence(self, p: int):
        s = self.spec
        H, Ie, El = s["H"], s["Ie"] // self.Y, s["E"] // self.X  # Ie: width held by one buffer
        seq = []
        for l in self.stage_layers[p]:
            if self.kind == "gen":
                seq.append(("w13", l, -1, El * 2 * Ie * H))
                seq.append(("w2", l, -1, El * H * Ie))
            elif self.grouped:
                seq.append(("w1", l, -1, El * H * 2 * Ie))
                seq.append(("w2", l, -1, El * Ie * H))
            else:
                for j in range(El):
                    seq.append(("fc1", l, j, 2 * Ie * H))
                    seq.append(("fc2", l, j, H * Ie))
        return seq

    def _walk(self):
        eb = self.spec["elem_bytes"]
        self.dense_off = [dict() for _ in range(self.P)]  # per stage: (name, layer) -> bytes
        self.expert_off = [dict() for _ in range(self.P)]  # (name, layer, j) -> bytes
        self.buf_bytes = [0] * self.nbufs
        self.stored = [[] for _ in range(self.nbufs)]  # (name, layer, j, off, nbytes)
        for p in range(self.P):
            off = 0
            for name, l, n in self._dense_sequence(p):
                off = _align(off)
                self.dense_off[p][(name, l)] = off
                for t in range(self.T):
                    self.stored[p * self.T + t].append((name, l, -1, off, n * eb))
                off += n * eb
            for t in range(self.T):
                self.buf_bytes[p * self.T + t] = _align(off)
            if self.moe:
                off = 0
                for name, l, j, n in self._expert_sequence(p):
                    off = _align(off)
                    self.expert_off[p][(name, l, j)] = off
                    for xy in range(self.X * self.Y):
                        self.stored[self.nd + p * self.X * self.Y + xy].append((name, l, j, off, n * eb))
                    off += n * eb
                for xy in range(self.X * self.Y):
                    self.buf_bytes[self.nd + p * self.X * self.Y + xy] = _align(off)

    def owned(self, b: int):
        """(offset, bytes) of the parts of buffer b that hold logical weights: the stored
        tensors minus vocabulary padding rows."""
        s, T = self.spec, self.T
        out = []
        for name, layer, j, off, nbytes in self.stored[b]:
            if name in ("emb", "lm_head", "emb_tied"):
                n, t = self.Vp // T, b % T
                real = max(0, min(n, s["V"] - t * n))
                nbytes = real * s["H"] * s["elem_bytes"]
            if nbytes:
                out.append((off, nbytes))
        return out

    # ---- the layout function -------------------------------------------------
    def place(self, name: str, layer: int, expert: int, r, c):
        """All homes of logical element (r, c) of a tensor: [(buffer, byte offset)].

        One entry for split tensors, several for replicated ones (common weights:
        one per tensor rank, rank 0 first; a KV head shared by T/nkv ranks: the
        lowest rank first; a tied embedding: first stage first).  The first entry
        is the copy a source is read from.  r and c may be ints or equal-shape arrays.
        """
        s, T, X = self.spec, self.T, self.X
        eb, H = s["elem_bytes"], s["H"]
        r = np.asarray(r, dtype=np.int64)
        c = np.asarray(c, dtype=np.int64)
        if name == "emb":
            p = 0
        elif name in ("final_ln", "lm_head"):
            p = self.P - 1
        else:
            p = self.layer_stage[layer]
        dbase = p * T

        def dense(stored, t, elem):
            return (dbase + t, self.dense_off[p][(stored, layer)] + elem * eb)

        if name in REPLICATED:
            cols = {"q_a_ln": s["q_lora"], "kv_a_ln": s["kv_lora"]}.get(name, H)
            return [dense(name, np.zeros_like(r) + t, r * cols + c) for t in range(T)]

        if name in ("emb", "lm_head"):
            n = self.Vp // T  # rows per rank, padding rows included; only rows below V are logical
            homes = [dense(name, r // n, (r % n) * H + c)]
            if name == "emb" and self.tied and self.P > 1:
                last = (self.P - 1) * T
                homes.append((last + r // n, self.dense_off[self.P - 1][("emb_tied", -1)] + ((r % n) * H + c) * eb))
            return homes

        if name in ("wq", "wk", "wv", "bq", "bk", "bv"):
            nq, nkv, d = s["nq"], s["nkv"], s["d"]
            g = nq // nkv
            which = name[1]
            bias = name[0] == "b"
            width = 1 if bias else H
            stored = "qkv_b" if bias else "qkv_w"
            if T > nkv:
                # every rank holds nq/T query heads and one (replicated) KV head, in both
                # layout kinds: [its query rows, the key head, the value head]
                rep, hq = T // nkv, nq // T
                if which == "q":
                    return [dense(stored, r // (hq * d), (r % (hq * d)) * width + c)]
                head, w = r // d, r % d
                row = hq * d + w + (0 if which == "k" else d)
                return [dense(stored, head * rep + i, row * width + c) for i in range(rep)]
            if self.kind == "train":
                # rank t holds nkv/T whole KV groups; inside a group: g query
                # heads, then the key head, then the value head.
                per = nkv // T
                if which == "q":
                    G, w = r // (g * d), r % (g * d)
                    inner = w
                else:
                    G, w = r // d, r % d
                    inner = g * d + w if which == "k" else (g + 1) * d + w
                t, j = G // per, G % per
                row = j * (g + 2) * d + inner
            else:
                # rank t holds its query rows, then its key rows, then its value rows.
                nql, nkl = nq * d // T, nkv * d // T
                if which == "q":
                    t, row = r // nql, r % nql
                elif which == "k":
                    t, row = r // nkl, nql + r % nkl
                else:
                    t, row = r // nkl, nql + nkl + r % nkl
            return [dense(stored, t, row * width + c)]

        if name == "wo":
            wid = s["nq"] * (s["v_dim"] if s["family"] == "moe_mla" else s["d"])
            n = wid // T
            return [dense("wo", c // n, r * n + c % n)]

        if name in ("w_gate", "w_up", "sh_gate", "sh_up"):
            width = s["I"] if name.startswith("w_") else s["n_shared"] * s["Ie"]
            stored = "gate_up" if name.startswith("w_") else "sh_fc1"
            n = width // T
            row = r % n + (n if name.endswith("up") else 0)
            return [dense(stored, r // n, row * H + c)]

        if name in ("w_down", "sh_down"):
            width = s["I"] if name == "w_down" else s["n_shared"] * s["Ie"]
            stored = "down" if name == "w_down" else "sh_fc2"
            n = width // T
            return [dense(stored, c // n, r * n + c % n)]

        if name in ("q_b", "kv_b"):
            per_head = s["nope"] + (s["rope"] if name == "q_b" else s["v_dim"])
            cols = s["q_lora"] if name == "q_b" else s["kv_lora"]
            n = s["nq"] // T * per_head
            return [dense(name, r // n, (r % n) * cols + c)]

        if name in ("ex_gate", "ex_up", "ex_down"):
            Y, El = self.Y, s["E"] // X
            n = s["Ie"] // Y                      # expert width held by one buffer
            x, j = expert // El, expert % El
            if name == "ex_down":                 # [H, Ie]: columns split over the expert-tensor ranks
                y, rl, cl = c // n, r, c % n
            else:                                 # [Ie, H]: rows split
                y, rl, cl = r // n, r % n, c
            buf = self.nd + (p * X + x) * Y + y
            eo = self.expert_off[p]
            up = n if name == "ex_up" else 0
            if self.kind == "gen":
                if name == "ex_down":
                    off = eo[("w2", layer, -1)] + ((j * H + rl) * n + cl) * eb
                else:
                    off = eo[("w13", layer, -1)] + ((j * 2 * n + up + rl) * H + cl) * eb
            elif self.grouped:
                # grouped-matmul orientation: [expert][in][out]
                if name == "ex_down":
                    off = eo[("w2", layer, -1)] + ((j * n + cl) * H + rl) * eb
                else:
                    off = eo[("w1", layer, -1)] + ((j * H + cl) * 2 * n + up + rl) * eb
            else:
                if name == "ex_down":
                    off = eo[("fc2", layer, j)] + (rl * n + cl) * eb
                else:
                    off = eo[("fc1", layer, j)] + ((up + rl) * H + cl) * eb
            return [(buf + np.zeros_like(r), off)]

        raise KeyError(name)


def _np_dtype(eb: int):
    return {1: np.uint8, 2: np.uint16, 4: np.uint32, 8: np.uint64}[eb]


def reshard_definition(spec, src_lay, dst_lay, src_bufs, dst_bufs, counters=None):
    """dst[place(DST, e)] = src[place(SRC, e)] for every logical element e.

    src_bufs / dst_bufs: one numpy array of the element dtype per buffer (an
    unused buffer may be None).  dst arrays are modified in place; bytes no
    tensor owns keep their prior value.  A replicated tensor is read from
    tensor rank 0 of its stage and written to every destination rank.  If
    `counters` (arrays shaped like dst_bufs) is given, each write adds one.
    Returns the set of source buffers that were read.
    """
    S, D = Layout(spec, src_lay), Layout(spec, dst_lay)
    assert src_lay["tp_filter"] < 0 and src_lay["ep_filter"] < 0
    eb = spec["elem_bytes"]
    read = set()
    for name, layer, expert, R, C in logical_tensors(spec):
        r, c = np.divmod(np.arange(R * C, dtype=np.int64), C)
        sb, so = S.place(name, layer, expert, r, c)[0]
        sb = np.broadcast_to(sb, r.shape)
        for db, do in D.place(name, layer, expert, r, c):
            db = np.broadcast_to(db, r.shape)
            for b in np.unique(db):
                if not D.buffer_used(int(b)):
                    continue
                m = db == b
                for a in np.unique(sb[m]):
                    mm = m & (sb == a)
                    read.add(int(a))
                    dst_bufs[b][do[mm] // eb] = src_bufs[a][so[mm] // eb]
                    if counters is not None:
                        np.add.at(counters[b], do[mm] // eb, 1)
    return read


def sample_pairs(spec, src_lay, dst_lay, per_tensor: int, rng: np.random.Generator,
                 max_tensors: int | None = None):
    """Random logical elements and their (src buffer, src byte offset,
    dst buffer, dst byte offset), for spot checks at sizes where tracing every
    element is too slow.  Elements whose destination is filtered out are
    skipped.  Returns four int64 arrays.
    """
    S, D = Layout(spec, src_lay), Layout(spec, dst_lay)
    tensors = logical_tensors(spec)
    if max_tensors is not None and len(tensors) > max_tensors:
        pick = rng.choice(len(tensors), size=max_tensors, replace=False)
        tensors = [tensors[i] for i in sorted(pick)]
    out = [[], [], [], []]
    for name, layer, expert, R, C in tensors:
        n = min(per_tensor, R * C)
        r = rng.integers(0, R, size=n)
        c = rng.integers(0, C, size=n)
        # always include the four corners
        r[:4] = np.array([0, 0, R - 1, R - 1])[:n]
        c[:4] = np.array([0, C - 1, 0, C - 1])[:n]
        sb, so = S.place(name, layer, expert, r, c)[0]
        for db, do in D.place(name, layer, expert, r, c):
            db = np.broadcast_to(db, r.shape)
            used = np.array([D.buffer_used(int(b)) for b in db])
            out[0].append(np.broadcast_to(sb, r.shape)[used])
            out[1].append(np.broadcast_to(so, r.shape)[used])
            out[2].append(db[used])
            out[3].append(np.broadcast_to(do, r.shape)[used])
    return tuple(np.concatenate(x).astype(np.int64) for x in out)
