"""Seeded synthetic workloads: model shapes, layout degrees and raw buffer fills.

This module is shared by the tests, the benchmark and the smoke check.  It holds
no layout arithmetic at all: a workload is a set of plain integers (the shape of
a model and the parallel degrees of its training and generation layouts), and a
fill writes pseudo-random 16-bit words into a flat buffer by (buffer index,
offset) only.  Both the CPU oracle and the HIP library translate the plain
dictionaries below into their own structures.

The shapes stand in for the checkpoints the paper trains (Qwen2.5-7B/32B,
Qwen3-MoE-30B, DeepSeek-R1-671B; Evaluation section): a byte-moving path depends
on shapes and degrees only, never on weight values.
"""

from __future__ import annotations

import torch

# Keys of a model shape.  `family`: "dense_gqa", "moe_gqa" or "moe_mla".
_SPEC_DEFAULTS = dict(
    family="dense_gqa", L=1, H=0, nq=0, nkv=0, d=0, I=0, V=0, qkv_bias=0,
    has_embeddings=1, E=0, Ie=0, n_shared=0, q_lora=0, kv_lora=0, nope=0,
    rope=0, v_dim=0, elem_bytes=2, tied_embeddings=0,
)
# Keys of a layout.  `kind`: "train" or "gen"; `expert_layout`: "per_expert" or
# "grouped"; the two filters select one rank of the layout (-1 = every rank).
# `vpp`: virtual pipeline size (interleaved layer chunks); `first_stage_layers` /
# `last_stage_layers`: uneven pipeline split (0 = even); `vocab_padded`: rows the
# embedding / lm_head are padded to before the tensor-parallel split (0 = V); `etp`:
# expert tensor parallelism, 1 (whole experts) or tp (every expert split like a dense FFN).
_LAYOUT_DEFAULTS = dict(kind="train", tp=1, pp=1, ep=1,
                        expert_layout="per_expert", tp_filter=-1, ep_filter=-1,
                        vpp=1, first_stage_layers=0, last_stage_layers=0, vocab_padded=0, etp=1)


def make_spec(**kw) -> dict:
    s = dict(_SPEC_DEFAULTS)
    s.update(kw)
    return s


def make_layout(**kw) -> dict:
    l = dict(_LAYOUT_DEFAULTS)
    l.update(kw)
    return l


def _wl(name, spec, src, dst, seed, note):
    return dict(name=name, spec=spec, src=src, dst=dst, seed=seed, note=note)


WORKLOADS = {
    # Toy dense decoder, training TP2 -> generation TP1.
    "C0": _wl(
        "C0",
        make_spec(family="dense_gqa", L=2, H=256, nq=4, nkv=2, d=64, I=688, V=1024),
        make_layout(kind="train", tp=2, pp=1),
        make_layout(kind="gen", tp=1),
        1000, "toy dense, TP2 -> TP1"),
    # Qwen2.5-7B-shaped dense decoder, training TP4 PP2 -> generation TP2.
    "C1": _wl(
        "C1",
        make_spec(family="dense_gqa", L=28, H=3584, nq=28, nkv=4, d=128, I=18944,
                  V=152064, qkv_bias=1),
        make_layout(kind="train", tp=4, pp=2),
        make_layout(kind="gen", tp=2),
        1001, "Qwen2.5-7B-shaped, TP4 PP2 -> TP2"),
    # Not a task config: an 8B-class GQA shape (32 query / 8 KV heads) under a wide training
    # layout, TP16 (every KV head shared by two ranks), PP2 with 2 interleaved chunks per
    # stage -> generation TP4.  It exercises the layout options beyond the task's at full size.
    "C1R": _wl(
        "C1R",
        make_spec(family="dense_gqa", L=32, H=4096, nq=32, nkv=8, d=128, I=14336,
                  V=128256),
        make_layout(kind="train", tp=16, pp=2, vpp=2),
        make_layout(kind="gen", tp=4),
        1005, "8B-class GQA shape, TP16 (KV heads replicated) PP2 VPP2 -> TP4"),
    # Qwen2.5-32B-shaped dense decoder, training TP8 PP4 -> generation TP4.
    "C2": _wl(
        "C2",
        make_spec(family="dense_gqa", L=64, H=5120, nq=40, nkv=8, d=128, I=27648,
                  V=152064, qkv_bias=1),
        make_layout(kind="train", tp=8, pp=4),
        make_layout(kind="gen", tp=4),
        1002, "Qwen2.5-32B-shaped, TP8 PP4 -> TP4"),
    # Qwen3-30B-A3B-shaped MoE, training EP8 TP1 PP2 -> generation EP4 TP2.
    # Source experts in the grouped-matmul orientation (transposing repack).
    "C3": _wl(
        "C3",
        make_spec(family="moe_gqa", L=48, H=2048, nq=32, nkv=4, d=128, V=151936,
                  E=128, Ie=768),
        make_layout(kind="train", tp=1, pp=2, ep=8, expert_layout="grouped"),
        make_layout(kind="gen", tp=2, ep=4),
        1003, "Qwen3-30B-A3B-shaped, EP8 TP1 PP2 (grouped experts) -> EP4 TP2"),
    # The same model with per-expert [out][in] source experts (pure regrouping).
    "C3P": _wl(
        "C3P",
        make_spec(family="moe_gqa", L=48, H=2048, nq=32, nkv=4, d=128, V=151936,
                  E=128, Ie=768),
        make_layout(kind="train", tp=1, pp=2, ep=8, expert_layout="per_expert"),
        make_layout(kind="gen", tp=2, ep=4),
        1003, "Qwen3-30B-A3B-shaped, EP8 TP1 PP2 (per-expert) -> EP4 TP2"),
    # Not a task config: the same model with every expert also split over the tensor ranks
    # (expert tensor parallelism) on both sides, grouped source experts: TP2 ETP2 EP4 PP2 ->
    # TP4 ETP4 EP2.  Half- and quarter-width transposes at full size.
    "C3E": _wl(
        "C3E",
        make_spec(family="moe_gqa", L=48, H=2048, nq=32, nkv=4, d=128, V=151936,
                  E=128, Ie=768),
        make_layout(kind="train", tp=2, pp=2, ep=4, etp=2, expert_layout="grouped"),
        make_layout(kind="gen", tp=4, ep=2, etp=4),
        1006, "Qwen3-30B-A3B-shaped, TP2 ETP2 EP4 PP2 (grouped experts) -> TP4 ETP4 EP2"),
    # DeepSeek-671B-shaped share: 8 MoE layers, EP64 -> rank 0 of EP8.
    "C4": _wl(
        "C4",
        make_spec(family="moe_mla", L=8, H=7168, nq=128, V=0, has_embeddings=0,
                  E=256, Ie=2048, n_shared=1, q_lora=1536, kv_lora=512, nope=128,
                  rope=64, v_dim=128),
        make_layout(kind="train", tp=1, pp=1, ep=64),
        make_layout(kind="gen", tp=1, ep=8, ep_filter=0),
        1004, "DeepSeek-671B-shaped share, EP64 -> one rank of EP8"),
}

# Small shapes for exhaustive checks (every element traced).
TINY = {
    # Dense GQA with bias, several KV groups per rank on both sides.
    "tiny_dense": _wl(
        "tiny_dense",
        make_spec(family="dense_gqa", L=4, H=48, nq=8, nkv=4, d=8, I=40, V=64,
                  qkv_bias=1),
        make_layout(kind="train", tp=4, pp=2),
        make_layout(kind="gen", tp=2),
        2000, "tiny dense TP4 PP2 -> TP2"),
    # The degrees of the paper's redundant-memory example (TP2 EP2 -> TP1 EP4).
    "tiny_moe": _wl(
        "tiny_moe",
        make_spec(family="moe_gqa", L=2, H=32, nq=4, nkv=2, d=8, V=48, E=8, Ie=24,
                  n_shared=1),
        make_layout(kind="train", tp=2, pp=1, ep=2),
        make_layout(kind="gen", tp=1, ep=4),
        2001, "tiny MoE TP2 EP2 -> TP1 EP4"),
    "tiny_moe_grouped": _wl(
        "tiny_moe_grouped",
        make_spec(family="moe_gqa", L=2, H=32, nq=4, nkv=2, d=8, V=48, E=8, Ie=24,
                  n_shared=1),
        make_layout(kind="train", tp=2, pp=2, ep=2, expert_layout="grouped"),
        make_layout(kind="gen", tp=1, ep=4),
        2002, "tiny MoE, grouped experts, TP2 PP2 EP2 -> TP1 EP4"),
    # Grouped experts large enough for full register-transposed tiles plus ragged edges.
    "mid_moe_grouped": _wl(
        "mid_moe_grouped",
        make_spec(family="moe_gqa", L=1, H=320, nq=4, nkv=2, d=16, V=64, E=4, Ie=200),
        make_layout(kind="train", tp=1, pp=1, ep=2, expert_layout="grouped"),
        make_layout(kind="gen", tp=2, ep=1),
        2004, "mid-size MoE, grouped experts (transposing), EP2 -> TP2 EP1"),
    # The same with matrices that hold several of the largest transposing tiles (512 long) and
    # ragged strips of every kind; all rows are multiples of 16 bytes at every element size.
    "big_moe_grouped": _wl(
        "big_moe_grouped",
        make_spec(family="moe_gqa", L=1, H=1232, nq=4, nkv=2, d=16, V=64, E=2, Ie=464),
        make_layout(kind="train", tp=1, pp=1, ep=2, expert_layout="grouped"),
        make_layout(kind="gen", tp=1, ep=1),
        2010, "grouped experts (transposing) with 1232 x 464 and 464 x 1232 matrices, EP2 -> EP1"),
    # KV-head replication: 2 KV heads on 4 tensor ranks (training) and 8 (the way back is
    # exercised by the round-trip tests), interleaved pipeline chunks, tied embeddings.
    "tiny_kvrep": _wl(
        "tiny_kvrep",
        make_spec(family="dense_gqa", L=8, H=48, nq=8, nkv=2, d=8, I=40, V=64,
                  qkv_bias=1, tied_embeddings=1),
        make_layout(kind="train", tp=4, pp=2, vpp=2),
        make_layout(kind="gen", tp=8),
        2005, "tiny dense, KV replication TP4 PP2 VPP2 -> TP8, tied embeddings"),
    # Uneven pipeline stages (3 + 2 + 2 + 1 layers) and a destination with fewer ranks than KV heads.
    "tiny_uneven": _wl(
        "tiny_uneven",
        make_spec(family="dense_gqa", L=8, H=32, nq=8, nkv=2, d=8, I=24, V=48),
        make_layout(kind="train", tp=4, pp=4, first_stage_layers=3, last_stage_layers=1),
        make_layout(kind="gen", tp=2),
        2006, "tiny dense, uneven PP4 (3,2,2,1), TP4 (KV replicated) -> TP2"),
    # Vocabulary padded differently on the two sides: 50 real rows, padded to 64 for TP4
    # (the last rank holds 2 real rows and 14 padding rows) and to 54 for TP2.
    "tiny_vocabpad": _wl(
        "tiny_vocabpad",
        make_spec(family="dense_gqa", L=2, H=24, nq=4, nkv=4, d=8, I=24, V=50),
        make_layout(kind="train", tp=4, pp=2, vocab_padded=64),
        make_layout(kind="gen", tp=2, vocab_padded=54),
        2007, "tiny dense, vocabulary 50 padded to 64 (TP4 PP2) -> padded to 54 (TP2)"),
    # Experts split over the tensor ranks as well (expert tensor parallelism) on both sides,
    # grouped orientation on the training side.
    "tiny_etp": _wl(
        "tiny_etp",
        make_spec(family="moe_gqa", L=2, H=32, nq=4, nkv=4, d=8, V=48, E=4, Ie=24, n_shared=1),
        make_layout(kind="train", tp=4, pp=1, ep=2, etp=4, expert_layout="grouped"),
        make_layout(kind="gen", tp=2, ep=1, etp=2),
        2008, "tiny MoE, expert tensor parallelism TP4 EP2 ETP4 (grouped) -> TP2 EP1 ETP2"),
    "tiny_mla": _wl(
        "tiny_mla",
        make_spec(family="moe_mla", L=2, H=40, nq=4, V=0, has_embeddings=0, E=8,
                  Ie=16, n_shared=1, q_lora=24, kv_lora=16, nope=8, rope=8,
                  v_dim=8),
        make_layout(kind="train", tp=2, pp=1, ep=8),
        make_layout(kind="gen", tp=1, ep=2, ep_filter=1),
        2003, "tiny MLA MoE TP2 EP8 -> TP1, rank 1 of EP2"),
}

# Mid-size dense shapes whose row-parallel weights (attention output, feed-forward down projection)
# have shard rows of at least 1 KiB (64 and 88 vectors of 16 bytes at 2-byte elements): the row
# lengths from which the library may cut a side-by-side merge as one contiguous stream.
_MID_SPEC = make_spec(family="dense_gqa", L=1, H=256, nq=8, nkv=4, d=256, I=2816, V=256)
MID = {
    "mid_merge2": _wl("mid_merge2", _MID_SPEC, make_layout(kind="train", tp=4), make_layout(kind="gen", tp=2),
                      2020, "mid-size dense, TP4 -> TP2: two shards side by side per destination row"),
    "mid_merge4": _wl("mid_merge4", _MID_SPEC, make_layout(kind="train", tp=4, pp=1), make_layout(kind="gen", tp=1),
                      2021, "mid-size dense, TP4 -> TP1: four shards side by side"),
    "mid_merge8": _wl("mid_merge8", dict(_MID_SPEC, elem_bytes=4), make_layout(kind="train", tp=8), make_layout(kind="gen", tp=1),
                      2022, "mid-size dense, 4-byte elements, TP8 -> TP1: eight shards side by side"),
    "mid_split": _wl("mid_split", _MID_SPEC, make_layout(kind="train", tp=1), make_layout(kind="gen", tp=2),
                     2023, "mid-size dense, TP1 -> TP2: destination rows packed out of wider source rows"),
}


def random_case(seed: int, scale: int = 1) -> dict:
    """A small random workload that the shape rules allow (divisibility only: no layout
    arithmetic): family, sizes, both layouts and every layout option drawn from `seed`.
    `scale` multiplies the widths (hidden size, head size, feed-forward widths, vocabulary):
    1 gives kilobyte tensors, 8 to 16 tensors of many tiles with ragged ends."""
    import math
    import random

    r = random.Random(seed * 1000 + scale)
    family = r.choice(["dense_gqa", "dense_gqa", "moe_gqa", "moe_gqa", "moe_mla"])
    moe = family != "dense_gqa"
    dst_train = r.random() < 0.2
    tp_s, tp_d = r.choice([1, 2, 4]), r.choice([1, 2, 4, 8])
    m = math.lcm(tp_s, tp_d)
    nkv = r.choice([1, 2, 4, 8])
    # heads: nq a multiple of both degrees and of nkv
    g = m // math.gcd(m, nkv) * r.choice([1, 2])
    nq = nkv * g if family != "moe_mla" else m * r.choice([1, 2])
    pp_s = r.choice([1, 1, 2, 4])
    pp_d = r.choice([1, 2]) if dst_train else 1
    src = dict(kind="train", tp=tp_s, pp=pp_s)
    dst = dict(kind="train" if dst_train else "gen", tp=tp_d, pp=pp_d)
    L = pp_s * pp_d * r.choice([1, 2])
    if pp_s >= 2 and r.random() < 0.3:  # uneven stages
        first, last = r.choice([1, 2, 3]), r.choice([1, 2])
        mid = (pp_s - 2) * r.choice([1, 2])
        L = (first + mid + last) * (2 if pp_d == 2 and (first + mid + last) % 2 else 1)
        if L != first + mid + last:  # keep the sum exact: fold the doubling into the stage sizes
            first, mid, last = 2 * first, 2 * mid, 2 * last
        src.update(first_stage_layers=first, last_stage_layers=last)
    elif r.random() < 0.4:
        src["vpp"] = 2
        L *= 2
    spec = dict(family=family, L=L, H=8 * r.choice([2, 3, 5, 8]) * scale, nq=nq, elem_bytes=r.choice([1, 2, 2, 4, 8]))
    if family != "moe_mla":
        spec.update(nkv=nkv, d=r.choice([4, 8, 16]) * min(scale, 8), qkv_bias=r.choice([0, 1]))
    else:
        spec.update(q_lora=r.choice([8, 24]) * scale, kv_lora=r.choice([8, 16]) * scale, nope=r.choice([4, 8]) * min(scale, 8),
                    rope=r.choice([4, 8]) * min(scale, 8), v_dim=r.choice([4, 8]) * min(scale, 8))
    if family == "dense_gqa":
        spec["I"] = m * r.choice([3, 5, 8]) * scale
    else:
        E = r.choice([2, 4, 8])
        spec.update(E=E, Ie=m * r.choice([1, 3, 4]) * scale, n_shared=r.choice([0, 1, 2]))
        src["ep"] = r.choice([x for x in (1, 2, 4, 8) if E % x == 0])
        dst["ep"] = r.choice([x for x in (1, 2, 4, 8) if E % x == 0])
        src["expert_layout"] = r.choice(["per_expert", "grouped"])
        if dst_train:
            dst["expert_layout"] = r.choice(["per_expert", "grouped"])
        if r.random() < 0.3:
            src["etp"] = tp_s
        if r.random() < 0.3:
            dst["etp"] = tp_d
    if r.random() < 0.8:
        V = r.choice([40, 50, 64, 96]) * scale + (r.choice([0, 1, 7]) if scale > 1 else 0)
        spec.update(V=V, has_embeddings=1, tied_embeddings=r.choice([0, 0, 1]))
        for lay in (src, dst):
            pad = -V % lay["tp"]
            if pad or r.random() < 0.3:
                lay["vocab_padded"] = V + pad + lay["tp"] * r.choice([0, 1, 3])
    else:
        spec.update(V=0, has_embeddings=0)
    if r.random() < 0.25 and tp_d > 1:
        dst["tp_filter"] = r.randrange(tp_d)
    if r.random() < 0.25 and dst.get("ep", 1) > 1:
        dst["ep_filter"] = r.randrange(dst["ep"])
    return _wl("random_%d_x%d" % (seed, scale), make_spec(**spec), make_layout(**src), make_layout(**dst), 3000 + seed + 7919 * (scale - 1),
               "random small workload")


def fill_buffer(nbytes: int, seed: int, device="cpu", mode: str = "normal") -> torch.Tensor:
    """A flat int16 tensor of nbytes/2 words filled from `seed`.

    mode "normal": bf16 words drawn from N(0, 0.02) (round-to-nearest-even by
    torch's cast); mode "raw16": uniformly random 16-bit patterns, which include
    NaN payloads, negative zero and subnormals.
    """
    assert nbytes % 2 == 0
    n = nbytes // 2
    dev = torch.device(device)
    g = torch.Generator(device=dev)
    g.manual_seed(int(seed))
    if mode == "normal":
        t = torch.empty(n, dtype=torch.bfloat16, device=dev)
        step = 1 << 28  # bounded temporaries for multi-GB buffers
        for s in range(0, n, step):
            t[s:s + step].normal_(0.0, 0.02, generator=g)
        return t.view(torch.int16)
    if mode == "raw16":
        t = torch.empty(n, dtype=torch.int16, device=dev)
        step = 1 << 28
        for s in range(0, n, step):
            t[s:s + step].random_(-32768, 32768, generator=g)
        return t
    raise ValueError(mode)


def fill_buffers(sizes, seed: int, device="cpu", mode: str = "normal"):
    """One filled buffer per entry of `sizes` (bytes); buffer i uses seed+i."""
    return [fill_buffer(int(n), seed * 1000 + i, device, mode) for i, n in enumerate(sizes)]


BF16_ONE = 0x3F80  # the 16-bit word of bf16 1.0, written over norm vectors
