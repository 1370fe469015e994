"""A third statement of the two layouts, for pinning the oracles: whole-tensor
numpy operations only (reshape, split, concatenate, transpose, stack).

Given every logical tensor as a 2-D array, `pack` builds the flat buffers of a
layout the way a Megatron-style checkpoint writer would: shard each tensor with
library calls, then lay the shards out one after another, each on a 256-byte
boundary.  There is no per-element index arithmetic here, so a mistake in the
oracles' formulas (a wrong sign, stride, head order or rank) shows up as a
mismatch against these constructions.
"""

from __future__ import annotations

import numpy as np


def make_logical(spec, tensors, rng, dtype):
    """Random distinct-ish contents for every logical tensor: dict keyed by
    (name, layer, expert) -> array [rows, cols]."""
    out = {}
    info = np.iinfo(dtype)
    for name, layer, expert, R, C in tensors:
        out[(name, layer, expert)] = rng.integers(0, info.max, size=(R, C), dtype=dtype)
    return out


def _layout_chunks(spec, lay, lg, fill=0):
    """Per buffer, the ordered list of shard arrays (any shape; stored flattened)."""
    fam = spec["family"]
    T, P, X = lay["tp"], lay["pp"], lay["ep"]
    gen = lay["kind"] == "gen"
    grouped = (not gen) and lay["expert_layout"] == "grouped"
    L, H = spec["L"], spec["H"]
    moe = fam != "dense_gqa"
    tied = bool(spec.get("tied_embeddings", 0))
    # layers of each stage in storage order
    vpp = lay.get("vpp", 1)
    first, last = lay.get("first_stage_layers", 0), lay.get("last_stage_layers", 0)
    if first or last:
        mid = (L - first - last) // (P - 2) if P > 2 else 0
        stage_layers = np.split(np.arange(L), np.cumsum([first] + [mid] * (P - 2)))
    else:
        # chunks dealt round-robin: chunk c -> stage c mod P
        chunks = np.arange(L).reshape(vpp, P, L // (P * vpp))
        stage_layers = [chunks[:, p, :].reshape(-1) for p in range(P)]
    nd = P * T
    bufs = [[] for _ in range(nd + (P * X * lay.get("etp", 1) if moe else 0))]
    Vp = lay.get("vocab_padded", 0) or spec["V"]

    def vocab_padded(a):  # padding rows appended before the split; they hold the gap value
        return np.concatenate([a, np.full((Vp - a.shape[0], a.shape[1]), fill, dtype=a.dtype)], axis=0)


    def rows_split(a):  # column-parallel: split the output rows over ranks
        return np.split(a, T, axis=0)

    def cols_split(a):  # row-parallel: split the input columns over ranks
        return np.split(a, T, axis=1)

    for p in range(P):
        dense = [bufs[p * T + t] for t in range(T)]
        if spec["has_embeddings"] and p == 0:
            for t, sh in enumerate(rows_split(vocab_padded(lg[("emb", -1, -1)]))):
                dense[t].append(sh)
        for l in (int(x) for x in stage_layers[p]):
            for t in range(T):
                dense[t].append(lg[("ln1", l, -1)])
            if fam == "moe_mla":
                qb, kvb, wo = (rows_split(lg[("q_b", l, -1)]), rows_split(lg[("kv_b", l, -1)]),
                               cols_split(lg[("wo", l, -1)]))
                for t in range(T):
                    dense[t] += [lg[("q_a", l, -1)], lg[("q_a_ln", l, -1)], qb[t],
                                 lg[("kv_a", l, -1)], lg[("kv_a_ln", l, -1)], kvb[t], wo[t]]
            else:
                nq, nkv, d = spec["nq"], spec["nkv"], spec["d"]
                g = nq // nkv
                names = [("wq", "wk", "wv")] + ([("bq", "bk", "bv")] if spec["qkv_bias"] else [])
                per_rank = [[] for _ in range(T)]
                for qn, kn, vn in names:
                    q, k, v = lg[(qn, l, -1)], lg[(kn, l, -1)], lg[(vn, l, -1)]
                    w = q.shape[1]
                    if T > nkv:
                        # each KV head is repeated for the T/nkv ranks that share it
                        kr = np.repeat(k.reshape(nkv, d, w), T // nkv, axis=0)
                        vr = np.repeat(v.reshape(nkv, d, w), T // nkv, axis=0)
                        for t, a in enumerate(rows_split(q)):
                            per_rank[t].append(np.concatenate([a, kr[t], vr[t]], axis=0))
                    elif gen:
                        # per rank: its query rows, then key rows, then value rows
                        for t, (a, b, c) in enumerate(zip(rows_split(q), rows_split(k), rows_split(v))):
                            per_rank[t].append(np.concatenate([a, b, c], axis=0))
                    else:
                        # per KV group: g query heads, the key head, the value head
                        fused = np.concatenate([q.reshape(nkv, g * d, w), k.reshape(nkv, d, w),
                                                v.reshape(nkv, d, w)], axis=1)
                        for t, sh in enumerate(np.split(fused, T, axis=0)):
                            per_rank[t].append(sh)
                wo = cols_split(lg[("wo", l, -1)])
                for t in range(T):
                    dense[t] += per_rank[t] + [wo[t]]
            for t in range(T):
                dense[t].append(lg[("ln2", l, -1)])
            if fam == "dense_gqa":
                ga, up, dn = (rows_split(lg[("w_gate", l, -1)]), rows_split(lg[("w_up", l, -1)]),
                              cols_split(lg[("w_down", l, -1)]))
                for t in range(T):
                    dense[t] += [np.concatenate([ga[t], up[t]], axis=0), dn[t]]
            else:
                for t in range(T):
                    dense[t].append(lg[("router", l, -1)])
                if spec["n_shared"]:
                    ga, up, dn = (rows_split(lg[("sh_gate", l, -1)]), rows_split(lg[("sh_up", l, -1)]),
                                  cols_split(lg[("sh_down", l, -1)]))
                    for t in range(T):
                        dense[t] += [np.concatenate([ga[t], up[t]], axis=0), dn[t]]
                El = spec["E"] // X
                Y = lay.get("etp", 1)
                for x in range(X):
                  for y in range(Y):
                    eb = bufs[nd + (p * X + x) * Y + y]
                    ex = range(x * El, (x + 1) * El)
                    # expert-tensor rank y: its rows of gate and up, its columns of down
                    fc1 = [np.concatenate([np.split(lg[("ex_gate", l, e)], Y, axis=0)[y],
                                           np.split(lg[("ex_up", l, e)], Y, axis=0)[y]], axis=0) for e in ex]
                    fc2 = [np.split(lg[("ex_down", l, e)], Y, axis=1)[y] for e in ex]
                    if gen:
                        eb += [np.stack(fc1), np.stack(fc2)]
                    elif grouped:
                        eb += [np.stack(fc1).transpose(0, 2, 1), np.stack(fc2).transpose(0, 2, 1)]
                    else:
                        for a, b in zip(fc1, fc2):
                            eb += [a, b]
        if spec["has_embeddings"] and p == P - 1:
            if not tied:
                tail = rows_split(vocab_padded(lg[("lm_head", -1, -1)]))
            elif P > 1:
                tail = rows_split(vocab_padded(lg[("emb", -1, -1)]))  # the last stage's own copy of the tied embedding
            else:
                tail = [None] * T
            for t in range(T):
                dense[t].append(lg[("final_ln", -1, -1)])
                if tail[t] is not None:
                    dense[t].append(tail[t])
    return bufs


def pack(spec, lay, lg, dtype, fill):
    """Flat buffers (1-D arrays of `dtype`) of a layout; gaps hold `fill`."""
    eb = np.dtype(dtype).itemsize
    out = []
    for chunks in _layout_chunks(spec, lay, lg, fill):
        parts, off = [], 0
        for a in chunks:
            pad = (-off) % 256
            assert pad % eb == 0
            if pad:
                parts.append(np.full(pad // eb, fill, dtype=dtype))
            flat = np.ascontiguousarray(a).reshape(-1)
            parts.append(flat)
            off += pad + flat.size * eb
        pad = (-off) % 256
        if pad:
            parts.append(np.full(pad // eb, fill, dtype=dtype))
        out.append(np.concatenate(parts) if parts else np.zeros(0, dtype=dtype))
    return out
