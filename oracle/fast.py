"""ctypes front end of the loop oracle (reshard_oracle.c).  TEST INFRASTRUCTURE ONLY.

Builds the C file with gcc on first use (or through `build()`), converts the
plain workload dictionaries into the oracle's own structs and runs the
resharding on host memory.  Nothing here touches the GPU or the product
library.
"""

from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "reshard_oracle.c")
_LIB = os.path.join(_HERE, "libreshard_oracle.so")

_FAMILY = {"dense_gqa": 0, "moe_gqa": 1, "moe_mla": 2}
_KIND = {"train": 0, "gen": 1}
_EXPERT = {"per_expert": 0, "grouped": 1}


class OrcSpec(C.Structure):
    _fields_ = [(k, C.c_int) for k in (
        "family", "L", "H", "nq", "nkv", "d", "I", "V", "qkv_bias", "has_embeddings",
        "E", "Ie", "n_shared", "q_lora", "kv_lora", "nope", "rope", "v_dim", "elem_bytes",
        "tied_embeddings")]


class OrcLayout(C.Structure):
    _fields_ = [(k, C.c_int) for k in (
        "kind", "tp", "pp", "ep", "expert_layout", "tp_filter", "ep_filter", "vpp",
        "first_stage_layers", "last_stage_layers", "vocab_padded", "etp")]


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        l = C.CDLL(build())
        l.orc_num_bufs.argtypes = [C.POINTER(OrcSpec), C.POINTER(OrcLayout)]
        l.orc_buf_bytes.argtypes = [C.POINTER(OrcSpec), C.POINTER(OrcLayout), C.c_int]
        l.orc_buf_bytes.restype = C.c_int64
        l.orc_buf_used.argtypes = [C.POINTER(OrcSpec), C.POINTER(OrcLayout), C.c_int]
        l.orc_reshard.argtypes = [C.POINTER(OrcSpec), C.POINTER(OrcLayout), C.POINTER(OrcLayout),
                                  C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.c_int,
                                  C.POINTER(C.c_int64)]
        l.orc_max_threads.restype = C.c_int
        _lib = l
    return _lib


def c_spec(spec: dict) -> OrcSpec:
    s = OrcSpec()
    for k, _ in OrcSpec._fields_:
        setattr(s, k, _FAMILY[spec[k]] if k == "family" else int(spec.get(k, 0)))
    return s


def c_layout(lay: dict) -> OrcLayout:
    l = OrcLayout()
    l.kind = _KIND[lay["kind"]]
    l.tp, l.pp, l.ep = lay["tp"], lay["pp"], lay["ep"]
    l.expert_layout = _EXPERT[lay["expert_layout"]]
    l.tp_filter, l.ep_filter = lay["tp_filter"], lay["ep_filter"]
    l.vpp = lay.get("vpp", 1)
    l.first_stage_layers = lay.get("first_stage_layers", 0)
    l.last_stage_layers = lay.get("last_stage_layers", 0)
    l.vocab_padded = lay.get("vocab_padded", 0)
    l.etp = lay.get("etp", 1)
    return l


def buffer_sizes(spec: dict, lay: dict):
    s, l = c_spec(spec), c_layout(lay)
    n = lib().orc_num_bufs(s, l)
    if n < 0:
        raise ValueError("invalid spec/layout")
    return [int(lib().orc_buf_bytes(s, l, i)) for i in range(n)]


def buffers_used(spec: dict, lay: dict):
    s, l = c_spec(spec), c_layout(lay)
    n = lib().orc_num_bufs(s, l)
    if n < 0:
        raise ValueError("invalid spec/layout")
    return [bool(lib().orc_buf_used(s, l, i)) for i in range(n)]


def max_threads() -> int:
    return int(lib().orc_max_threads())


def reshard(spec: dict, src_lay: dict, dst_lay: dict, src_bufs, dst_bufs, threads: int = 1) -> int:
    """Fill dst_bufs (numpy arrays, modified in place; None for unused) from src_bufs.

    Returns the number of destination bytes written.
    """
    s, sl, dl = c_spec(spec), c_layout(src_lay), c_layout(dst_lay)

    def ptrs(bufs, writable):
        arr = (C.c_void_p * len(bufs))()
        for i, b in enumerate(bufs):
            if b is None:
                arr[i] = None
            else:
                assert isinstance(b, np.ndarray) and b.flags["C_CONTIGUOUS"]
                if writable:
                    assert b.flags["WRITEABLE"]
                arr[i] = b.ctypes.data
        return arr

    total = C.c_int64(0)
    rc = lib().orc_reshard(s, sl, dl, ptrs(src_bufs, False), ptrs(dst_bufs, True), int(threads),
                           C.byref(total))
    if rc != 0:
        raise ValueError("invalid spec/layout pair")
    return int(total.value)
