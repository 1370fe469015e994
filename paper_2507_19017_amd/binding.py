"""ctypes binding of the C ABI in include/reshard.h.

Argument marshalling only: every step of the path (plan building, repack
kernels, swap copies, ledger) runs inside libreshard.so.  There is no fallback:
if the library is missing, importing a symbol from it raises.
"""

from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libreshard.so")

FAMILY = {"dense_gqa": 0, "moe_gqa": 1, "moe_mla": 2}
KIND = {"train": 0, "gen": 1}
EXPERT_LAYOUT = {"per_expert": 0, "grouped": 1}
STATE = {0: "unbound", 1: "resident", 2: "swapping_out", 3: "on_host", 4: "released", 5: "swapping_in", 6: "mixed"}

OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_OOM, ERR_HOST_OOM, ERR_BAD_STATE, ERR_HIP = 0, -1, -2, -3, -4, -5, -6
_ERR_NAMES = {-1: "INVALID_ARG", -2: "UNSUPPORTED", -3: "OOM", -4: "HOST_OOM", -5: "BAD_STATE", -6: "HIP"}


class ModelSpec(C.Structure):
    _fields_ = [("struct_size", C.c_uint32)] + [(k, C.c_int32) for k in (
        "family", "L", "H", "nq", "nkv", "d", "I", "V", "qkv_bias", "has_embeddings", "E", "Ie",
        "n_shared", "q_lora", "kv_lora", "nope", "rope", "v_dim", "elem_bytes", "tied_embeddings")]


class Layout(C.Structure):
    _fields_ = [("struct_size", C.c_uint32)] + [(k, C.c_int32) for k in (
        "kind", "tp", "pp", "ep", "expert_layout", "tp_rank_filter", "ep_rank_filter", "vpp",
        "first_stage_layers", "last_stage_layers", "vocab_padded", "etp")]


class TensorInfo(C.Structure):
    _fields_ = [("name", C.c_char * 24), ("layer", C.c_int32), ("expert", C.c_int32),
                ("buffer", C.c_int32), ("replicated", C.c_int32), ("offset", C.c_int64),
                ("bytes", C.c_int64), ("weight_class", C.c_int32), ("reserved_", C.c_int32)]


class Desc(C.Structure):
    _fields_ = [("src_buf", C.c_int32), ("dst_buf", C.c_int32), ("kind", C.c_int32),
                ("elem_bytes", C.c_int32), ("src_off", C.c_int64), ("dst_off", C.c_int64),
                ("rows", C.c_int64), ("row_bytes", C.c_int64), ("src_stride", C.c_int64),
                ("dst_stride", C.c_int64)]


class TileView(C.Structure):
    _fields_ = [("src_buf", C.c_int32), ("dst_buf", C.c_int32), ("kind", C.c_int32), ("tile_class", C.c_int32),
                ("src_off", C.c_int64), ("dst_off", C.c_int64), ("rows", C.c_int64), ("row_units", C.c_int64),
                ("src_stride", C.c_int64), ("dst_stride", C.c_int64), ("vec_bytes", C.c_int32),
                ("order", C.c_int32), ("sources", C.c_int64), ("phase", C.c_int64)]


class PlanInfo(C.Structure):
    _fields_ = [("num_src_bufs", C.c_int32), ("num_dst_bufs", C.c_int32), ("num_descs", C.c_int64),
                ("num_tiles", C.c_int64), ("num_transpose_tiles", C.c_int64),
                ("bytes_moved", C.c_int64), ("table_bytes", C.c_int64)]


class MemStats(C.Structure):
    _fields_ = [("src_live", C.c_int64), ("dst_live", C.c_int64), ("host_pinned", C.c_int64),
                ("peak_device", C.c_int64), ("released", C.c_int64), ("state", C.c_int32)]


class Tuning(C.Structure):
    _fields_ = [(k, C.c_int32) for k in ("tile_bytes", "block_threads", "blocks_per_cu", "unroll", "flags", "transpose_rows", "transpose_cols",
                                          "tail_pool_percent", "tail_chunk_tiles", "table_copies")]


class ReshardError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__("RESHARD_ERR_%s (%d): %s" % (_ERR_NAMES.get(code, "?"), code, msg))
        self.code = code


_lib = None


def lib():
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError("libreshard.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
        l = C.CDLL(_LIB_PATH)
        P = C.c_void_p
        sig = {
            "reshard_last_error": (C.c_char_p, []),
            "reshard_version": (C.c_char_p, []),
            "reshard_set_tuning": (C.c_int, [C.POINTER(Tuning)]),
            "reshard_get_tuning": (C.c_int, [C.POINTER(Tuning)]),
            "reshard_plan_create": (C.c_int, [C.POINTER(ModelSpec), C.POINTER(Layout), C.POINTER(Layout), C.POINTER(P)]),
            "reshard_plan_create_tuned": (C.c_int, [C.POINTER(ModelSpec), C.POINTER(Layout), C.POINTER(Layout), C.POINTER(Tuning), C.POINTER(P)]),
            "reshard_plan_set_tuning": (C.c_int, [P, C.POINTER(Tuning)]),
            "reshard_plan_get_tuning": (C.c_int, [P, C.POINTER(Tuning)]),
            "reshard_plan_destroy": (C.c_int, [P]),
            "reshard_plan_num_bufs": (C.c_int, [P, C.c_int]),
            "reshard_plan_buf_bytes": (C.c_int64, [P, C.c_int, C.c_int]),
            "reshard_plan_buf_used": (C.c_int, [P, C.c_int, C.c_int]),
            "reshard_plan_num_tensors": (C.c_int64, [P, C.c_int]),
            "reshard_plan_tensor": (C.c_int, [P, C.c_int, C.c_int64, C.POINTER(TensorInfo)]),
            "reshard_plan_get_info": (C.c_int, [P, C.POINTER(PlanInfo)]),
            "reshard_plan_class_bytes": (C.c_int, [P, C.c_int, C.POINTER(C.c_int64)]),
            "reshard_redundant_memory_bytes": (C.c_double, [C.c_int, C.c_double, C.c_int, C.c_double, C.c_int]),
            "reshard_plan_desc": (C.c_int, [P, C.c_int64, C.POINTER(Desc)]),
            "reshard_plan_tile": (C.c_int, [P, C.c_int64, C.POINTER(TileView)]),
            "reshard_plan_prepare": (C.c_int, [P]),
            "reshard_execute": (C.c_int, [P, C.POINTER(P), C.POINTER(P), P]),
            "reshard_execute_noalloc": (C.c_int, [P, C.POINTER(P), C.POINTER(P), P]),
            "reshard_execute_source": (C.c_int, [P, C.c_int, P, C.POINTER(P), P]),
            "reshard_swap_out_source": (C.c_int, [P, C.c_int, P]),
            "reshard_mark_src_buffer_released": (C.c_int, [P, C.c_int]),
            "reshard_src_buffer_state": (C.c_int, [P, C.c_int]),
            "reshard_bind_src": (C.c_int, [P, C.POINTER(P)]),
            "reshard_swap_out": (C.c_int, [P, P]),
            "reshard_swap_in": (C.c_int, [P, P]),
            "reshard_swap_wait": (C.c_int, [P]),
            "reshard_swap_wait_buffer": (C.c_int, [P, C.c_int, P, C.c_int]),
            "reshard_mark_src_released": (C.c_int, [P]),
            "reshard_mark_dst_released": (C.c_int, [P]),
            "reshard_swap_in_source": (C.c_int, [P, C.c_int, C.c_void_p, C.c_void_p]),
            "reshard_reserve_host": (C.c_int, [P]),
            "reshard_release_host": (C.c_int, [P]),
            "reshard_host_copy": (P, [P, C.c_int]),
            "reshard_set_host_limit": (None, [C.c_int64]),
            "reshard_mem_stats": (C.c_int, [P, C.POINTER(MemStats)]),
            "reshard_copy_baseline": (C.c_int, [P, P, C.c_int64, P]),
            "reshard_read_baseline": (C.c_int, [P, C.c_int64, P]),
            "reshard_write_baseline": (C.c_int, [P, C.c_int64, P]),
        }
        for name, (res, args) in sig.items():
            fn = getattr(l, name)
            fn.restype, fn.argtypes = res, args
        _lib = l
    return _lib


EXPORTS = (
    "reshard_last_error", "reshard_version", "reshard_set_tuning", "reshard_get_tuning",
    "reshard_plan_create", "reshard_plan_create_tuned", "reshard_plan_set_tuning", "reshard_plan_get_tuning", "reshard_plan_destroy", "reshard_plan_num_bufs", "reshard_plan_buf_bytes",
    "reshard_plan_buf_used", "reshard_plan_num_tensors", "reshard_plan_tensor", "reshard_plan_get_info",
    "reshard_plan_class_bytes", "reshard_redundant_memory_bytes",
    "reshard_plan_desc", "reshard_plan_tile", "reshard_plan_prepare", "reshard_execute", "reshard_execute_noalloc", "reshard_execute_source",
    "reshard_swap_out_source", "reshard_mark_src_buffer_released", "reshard_src_buffer_state", "reshard_bind_src", "reshard_swap_out", "reshard_swap_in",
    "reshard_swap_wait", "reshard_swap_wait_buffer", "reshard_mark_src_released", "reshard_mark_dst_released", "reshard_swap_in_source", "reshard_reserve_host", "reshard_release_host",
    "reshard_host_copy", "reshard_set_host_limit", "reshard_mem_stats", "reshard_copy_baseline",
    "reshard_read_baseline", "reshard_write_baseline",
)


def last_error() -> str:
    return lib().reshard_last_error().decode()


def _check(rc: int) -> int:
    if rc < 0:
        raise ReshardError(rc, last_error())
    return rc


def version() -> str:
    return lib().reshard_version().decode()


def set_tuning(**kw) -> None:
    """tile_bytes, block_threads, blocks_per_cu, unroll, flags, transpose_rows, transpose_cols; no argument = defaults."""
    if not kw:
        _check(lib().reshard_set_tuning(None))
        return
    t = Tuning(**{k: int(v) for k, v in kw.items()})
    _check(lib().reshard_set_tuning(C.byref(t)))


def get_tuning() -> dict:
    t = Tuning()
    _check(lib().reshard_get_tuning(C.byref(t)))
    return {k: getattr(t, k) for k, _ in Tuning._fields_}


def set_host_limit(limit: int) -> None:
    lib().reshard_set_host_limit(int(limit))


def read_baseline(src_ptr: int, nbytes: int, stream: int = 0) -> None:
    _check(lib().reshard_read_baseline(C.c_void_p(src_ptr), int(nbytes), C.c_void_p(stream)))


def write_baseline(dst_ptr: int, nbytes: int, stream: int = 0) -> None:
    _check(lib().reshard_write_baseline(C.c_void_p(dst_ptr), int(nbytes), C.c_void_p(stream)))


def copy_baseline(dst_ptr: int, src_ptr: int, nbytes: int, stream: int = 0) -> None:
    _check(lib().reshard_copy_baseline(C.c_void_p(dst_ptr), C.c_void_p(src_ptr), int(nbytes), C.c_void_p(stream)))


def redundant_memory_bytes(gen_dp: int, tp_weight_bytes: float, update_tp: int, ep_weight_bytes: float, gen_ep: int) -> float:
    return lib().reshard_redundant_memory_bytes(gen_dp, tp_weight_bytes, update_tp, ep_weight_bytes, gen_ep)


def make_spec(spec: dict) -> ModelSpec:
    s = ModelSpec()
    s.struct_size = C.sizeof(ModelSpec)
    for k, _ in ModelSpec._fields_[1:]:
        setattr(s, k, FAMILY[spec[k]] if k == "family" else int(spec.get(k, 0)))
    return s


def make_layout(lay: dict) -> Layout:
    l = Layout()
    l.struct_size = C.sizeof(Layout)
    l.kind = KIND[lay["kind"]]
    l.tp, l.pp, l.ep = int(lay["tp"]), int(lay["pp"]), int(lay["ep"])
    l.expert_layout = EXPERT_LAYOUT[lay["expert_layout"]]
    l.tp_rank_filter, l.ep_rank_filter = int(lay["tp_filter"]), int(lay["ep_filter"])
    l.vpp = int(lay.get("vpp", 1))
    l.first_stage_layers = int(lay.get("first_stage_layers", 0))
    l.last_stage_layers = int(lay.get("last_stage_layers", 0))
    l.vocab_padded = int(lay.get("vocab_padded", 0))
    l.etp = int(lay.get("etp", 1))
    return l


def _ptr_array(ptrs):
    arr = (C.c_void_p * max(1, len(ptrs)))()
    for i, p in enumerate(ptrs):
        arr[i] = None if not p else int(p)
    return arr


class Plan:
    """Thin owner of a reshard_plan*; methods mirror the C entry points one to one."""

    def __init__(self, spec: dict, src: dict, dst: dict, tuning: dict | None = None):
        """tuning: fields of reshard_tuning for this plan alone (None: the process-wide default)."""
        self._h = C.c_void_p()
        s, a, b = make_spec(spec), make_layout(src), make_layout(dst)
        if tuning is None:
            _check(lib().reshard_plan_create(C.byref(s), C.byref(a), C.byref(b), C.byref(self._h)))
        else:
            t = Tuning(**{k: int(v) for k, v in tuning.items()})
            _check(lib().reshard_plan_create_tuned(C.byref(s), C.byref(a), C.byref(b), C.byref(t), C.byref(self._h)))

    def set_tuning(self, **kw) -> None:
        """Launch shape of this plan's later executes (block_threads, blocks_per_cu, unroll, flags)."""
        t = Tuning(**{k: int(v) for k, v in kw.items()})
        _check(lib().reshard_plan_set_tuning(self._h, C.byref(t)))

    def get_tuning(self) -> dict:
        t = Tuning()
        _check(lib().reshard_plan_get_tuning(self._h, C.byref(t)))
        return {k: getattr(t, k) for k, _ in Tuning._fields_}

    def destroy(self) -> None:
        if self._h:
            lib().reshard_plan_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    # ---- queries ---------------------------------------------------------
    def num_bufs(self, side: int) -> int:
        return _check(lib().reshard_plan_num_bufs(self._h, side))

    def buf_bytes(self, side: int):
        return [_check(lib().reshard_plan_buf_bytes(self._h, side, i)) for i in range(self.num_bufs(side))]

    def buf_used(self, side: int):
        return [bool(_check(lib().reshard_plan_buf_used(self._h, side, i))) for i in range(self.num_bufs(side))]

    def tensors(self, side: int):
        n = _check(lib().reshard_plan_num_tensors(self._h, side))
        out, ti = [], TensorInfo()
        for i in range(n):
            _check(lib().reshard_plan_tensor(self._h, side, i, C.byref(ti)))
            out.append(dict(name=ti.name.decode(), layer=ti.layer, expert=ti.expert, buffer=ti.buffer,
                            replicated=bool(ti.replicated), offset=ti.offset, bytes=ti.bytes,
                            weight_class="TEC"[ti.weight_class]))
        return out

    def class_bytes(self, side: int) -> dict:
        out = (C.c_int64 * 3)()
        _check(lib().reshard_plan_class_bytes(self._h, side, out))
        return {"T": out[0], "E": out[1], "C": out[2]}

    def info(self) -> dict:
        pi = PlanInfo()
        _check(lib().reshard_plan_get_info(self._h, C.byref(pi)))
        return {k: getattr(pi, k) for k, _ in PlanInfo._fields_}

    def descs(self):
        n = self.info()["num_descs"]
        out, d = [], Desc()
        for i in range(n):
            _check(lib().reshard_plan_desc(self._h, i, C.byref(d)))
            out.append({k: getattr(d, k) for k, _ in Desc._fields_})
        return out

    def tiles(self):
        n = self.info()["num_tiles"]
        out, t = [], TileView()
        for i in range(n):
            _check(lib().reshard_plan_tile(self._h, i, C.byref(t)))
            out.append({k: getattr(t, k) for k, _ in TileView._fields_ if k != "reserved_"})
        return out

    # ---- the hot path ----------------------------------------------------
    def prepare(self) -> None:
        _check(lib().reshard_plan_prepare(self._h))

    def execute(self, src_ptrs, dst_ptrs, stream: int = 0) -> None:
        _check(lib().reshard_execute(self._h, _ptr_array(src_ptrs), _ptr_array(dst_ptrs), C.c_void_p(stream)))

    def execute_noalloc(self, src_ptrs, dst_ptrs, stream: int = 0) -> None:
        _check(lib().reshard_execute_noalloc(self._h, _ptr_array(src_ptrs), _ptr_array(dst_ptrs), C.c_void_p(stream)))

    def execute_source(self, src_index: int, src_ptr: int, dst_ptrs, stream: int = 0) -> None:
        _check(lib().reshard_execute_source(self._h, src_index, C.c_void_p(src_ptr), _ptr_array(dst_ptrs), C.c_void_p(stream)))

    def swap_out_source(self, src_index: int, stream: int = 0) -> None:
        _check(lib().reshard_swap_out_source(self._h, src_index, C.c_void_p(stream)))

    def mark_src_buffer_released(self, src_index: int) -> None:
        _check(lib().reshard_mark_src_buffer_released(self._h, src_index))

    def src_buffer_state(self, src_index: int) -> str:
        return STATE[_check(lib().reshard_src_buffer_state(self._h, src_index))]

    def bind_src(self, src_ptrs) -> None:
        _check(lib().reshard_bind_src(self._h, _ptr_array(src_ptrs)))

    def swap_out(self, stream: int = 0) -> None:
        _check(lib().reshard_swap_out(self._h, C.c_void_p(stream)))

    def swap_in(self, stream: int = 0) -> None:
        _check(lib().reshard_swap_in(self._h, C.c_void_p(stream)))

    def swap_wait(self) -> None:
        _check(lib().reshard_swap_wait(self._h))

    def swap_wait_buffer(self, index: int, stream: int = 0, host_wait: bool = True) -> None:
        _check(lib().reshard_swap_wait_buffer(self._h, index, C.c_void_p(stream), 1 if host_wait else 0))

    def mark_src_released(self) -> None:
        _check(lib().reshard_mark_src_released(self._h))

    def mark_dst_released(self) -> None:
        _check(lib().reshard_mark_dst_released(self._h))

    def swap_in_source(self, src_index: int, src_ptr: int = 0, stream: int = 0) -> None:
        _check(lib().reshard_swap_in_source(self._h, src_index, C.c_void_p(src_ptr or None), C.c_void_p(stream)))

    def reserve_host(self) -> None:
        _check(lib().reshard_reserve_host(self._h))

    def release_host(self) -> None:
        _check(lib().reshard_release_host(self._h))

    def host_copy(self, index: int) -> int:
        return lib().reshard_host_copy(self._h, index) or 0

    def mem_stats(self) -> dict:
        ms = MemStats()
        _check(lib().reshard_mem_stats(self._h, C.byref(ms)))
        d = {k: getattr(ms, k) for k, _ in MemStats._fields_}
        d["state"] = STATE[d["state"]]
        return d
