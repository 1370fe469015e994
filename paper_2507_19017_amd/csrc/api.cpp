// C ABI of the resharding library: plan lifetime, queries, execute, the swap
// path (steps 3 and 3b of the allgather-swap technique: device-to-host after the
// repack, host-to-device before the next update) and the byte ledger.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cstring>
#include <new>
#include <string>

#include "internal.h"

namespace reshard {
const char *last_error_cstr();
int ensure_device_table(reshard_plan *plan);
int ensure_by_source_table(reshard_plan *plan);
int launch_repack(reshard_plan *plan, hipStream_t stream);
int launch_repack_static(reshard_plan *plan, hipStream_t stream);
int launch_source(reshard_plan *plan, int src_index, hipStream_t stream);
}  // namespace reshard

using namespace reshard;

namespace {

std::atomic<int64_t> g_host_limit{-1};
std::atomic<uint64_t> g_plan_serial{0};

int hip_fail(hipError_t e, const char *what) {
    return fail(RESHARD_ERR_HIP, std::string(what) + ": " + hipGetErrorString(e));
}

const Side *side_of(const reshard_plan *plan, int side) {
    if (!plan || (side != 0 && side != 1)) return nullptr;
    return side == 0 ? &plan->src : &plan->dst;
}

int64_t used_bytes(const Side &s) {
    int64_t n = 0;
    for (size_t i = 0; i < s.buf_bytes.size(); ++i)
        if (s.used[i]) n += s.buf_bytes[i];
    return n;
}

// Checks one pointer set against a side: non-NULL and 256-byte aligned where used.
int check_ptrs(const Side &s, const void *const *ptrs, const char *what) {
    if (!ptrs) return fail(RESHARD_ERR_INVALID_ARG, std::string(what) + " is NULL");
    for (size_t i = 0; i < s.buf_bytes.size(); ++i) {
        if (!s.used[i]) continue;
        if (!ptrs[i]) return fail(RESHARD_ERR_INVALID_ARG, std::string(what) + "[" + std::to_string(i) + "] is NULL but the buffer is used");
        if (reinterpret_cast<uintptr_t>(ptrs[i]) % 256)
            return fail(RESHARD_ERR_INVALID_ARG, std::string(what) + "[" + std::to_string(i) + "] is not 256-byte aligned");
    }
    return RESHARD_OK;
}

// ---- per-buffer residency ------------------------------------------------------------
// Every used source buffer carries its own RESHARD_SRC_* state; the plan-level state is the
// common state of the used buffers, or RESHARD_SRC_MIXED while they differ (streaming).

bool is_live(int st) {
    return st == RESHARD_SRC_RESIDENT || st == RESHARD_SRC_SWAPPING_OUT || st == RESHARD_SRC_ON_HOST ||
           st == RESHARD_SRC_SWAPPING_IN;
}

// Recomputes the plan-level state and the ledger's source figures from the buffer states.
void recompute(reshard_plan *p) {
    int common = -1;
    bool mixed = false;
    int64_t live = 0, released = 0;
    for (size_t i = 0; i < p->buf_state.size(); ++i) {
        if (!p->src.used[i]) continue;
        const int st = p->buf_state[i];
        if (common < 0) common = st;
        else if (common != st) mixed = true;
        // a buffer on the host whose device pointer was dropped is not live
        if (is_live(st) && p->src_ptrs[i]) live += p->src.buf_bytes[i];
        if (st == RESHARD_SRC_RELEASED) released += p->src.buf_bytes[i];
    }
    p->state = common < 0 ? RESHARD_SRC_UNBOUND : mixed ? RESHARD_SRC_MIXED : common;
    bool any_out = false;
    for (size_t i = 0; i < p->buf_state.size(); ++i) any_out = any_out || (p->src.used[i] && p->buf_state[i] == RESHARD_SRC_SWAPPING_OUT);
    if (!any_out) p->exec_during_swap = false;
    p->src_live = live;
    p->released = released;
    p->touch_peak();
}

void set_all(reshard_plan *p, int st) {
    for (size_t i = 0; i < p->buf_state.size(); ++i)
        if (p->src.used[i]) p->buf_state[i] = st;
    recompute(p);
}

int ensure_swap_objects(reshard_plan *p) {
    if (!p->side_stream) {
        hipStream_t s;
        if (hipError_t e = hipStreamCreateWithFlags(&s, hipStreamNonBlocking)) return hip_fail(e, "hipStreamCreate");
        p->side_stream = s;
    }
    for (void **slot : {&p->ev_ready, &p->ev_exec}) {
        if (*slot) continue;
        hipEvent_t ev;
        if (hipError_t e = hipEventCreateWithFlags(&ev, hipEventDisableTiming)) return hip_fail(e, "hipEventCreate");
        *slot = ev;
    }
    if (p->ev_buf.empty()) p->ev_buf.assign(p->src.buf_bytes.size(), nullptr);
    for (size_t i = 0; i < p->ev_buf.size(); ++i) {
        if (!p->src.used[i] || p->ev_buf[i]) continue;
        hipEvent_t ev;
        if (hipError_t e = hipEventCreateWithFlags(&ev, hipEventDisableTiming)) return hip_fail(e, "hipEventCreate");
        p->ev_buf[i] = ev;
    }
    return RESHARD_OK;
}

void free_host_copies(reshard_plan *p) {
    for (void *&h : p->host_copy) {
        if (h) (void)hipHostFree(h);
        h = nullptr;
    }
    p->host_pinned = 0;
}

// All-or-nothing allocation of the pinned copies of the buffers selected by `only` (-1 = all used).
int ensure_host_copies(reshard_plan *p, int only = -1) {
    const Side &s = p->src;
    auto wanted = [&](size_t i) { return s.used[i] && !p->host_copy[i] && (only < 0 || size_t(only) == i); };
    int64_t need = 0;
    for (size_t i = 0; i < s.buf_bytes.size(); ++i)
        if (wanted(i)) need += s.buf_bytes[i];
    if (need == 0) return RESHARD_OK;
    const int64_t limit = g_host_limit.load();
    if (limit >= 0 && p->host_pinned + need > limit)
        return fail(RESHARD_ERR_HOST_OOM, "pinned host allocation refused by the configured limit");
    std::vector<size_t> fresh;
    for (size_t i = 0; i < s.buf_bytes.size(); ++i) {
        if (!wanted(i)) continue;
        void *h = nullptr;
        if (hipError_t e = hipHostMalloc(&h, size_t(s.buf_bytes[i]), hipHostMallocDefault)) {
            (void)hipGetLastError();
            for (size_t j : fresh) {
                (void)hipHostFree(p->host_copy[j]);
                p->host_copy[j] = nullptr;
                p->host_pinned -= s.buf_bytes[j];
            }
            return fail(RESHARD_ERR_HOST_OOM, std::string("hipHostMalloc: ") + hipGetErrorString(e));
        }
        p->host_copy[i] = h;
        p->host_pinned += s.buf_bytes[i];
        fresh.push_back(i);
    }
    return RESHARD_OK;
}

// Completes the copy of one buffer on the host side (blocks until its event has fired).
int finish_buffer(reshard_plan *p, size_t i) {
    const int st = p->buf_state[i];
    if (st != RESHARD_SRC_SWAPPING_OUT && st != RESHARD_SRC_SWAPPING_IN) return RESHARD_OK;
    if (hipError_t e = hipEventSynchronize(static_cast<hipEvent_t>(p->ev_buf[i]))) return hip_fail(e, "hipEventSynchronize");
    // ON_HOST tells the caller the device copy may go: a repack launched while the copies were in
    // flight reads the same buffers on the caller's stream and must have finished as well
    if (st == RESHARD_SRC_SWAPPING_OUT && p->exec_during_swap)
        if (hipError_t e = hipEventSynchronize(static_cast<hipEvent_t>(p->ev_exec))) return hip_fail(e, "hipEventSynchronize");
    p->buf_state[i] = st == RESHARD_SRC_SWAPPING_OUT ? RESHARD_SRC_ON_HOST : RESHARD_SRC_RESIDENT;
    return RESHARD_OK;
}

int finish_swap(reshard_plan *p) {
    for (size_t i = 0; i < p->buf_state.size(); ++i)
        if (p->src.used[i])
            if (int rc = finish_buffer(p, i)) return rc;
    recompute(p);
    return RESHARD_OK;
}

bool overlaps(const void *a, int64_t an, const void *b, int64_t bn) {
    const uintptr_t a0 = reinterpret_cast<uintptr_t>(a), a1 = a0 + uintptr_t(an);
    const uintptr_t b0 = reinterpret_cast<uintptr_t>(b), b1 = b0 + uintptr_t(bn);
    return a0 < b1 && b0 < a1;
}

// One device-to-host or host-to-device copy of buffer i on the side stream, followed by its event.
int queue_copy(reshard_plan *p, size_t i, bool to_host) {
    hipStream_t side = static_cast<hipStream_t>(p->side_stream);
    const size_t n = size_t(p->src.buf_bytes[i]);
    hipError_t e = to_host ? hipMemcpyAsync(p->host_copy[i], p->src_ptrs[i], n, hipMemcpyDeviceToHost, side)
                           : hipMemcpyAsync(const_cast<void *>(p->src_ptrs[i]), p->host_copy[i], n, hipMemcpyHostToDevice, side);
    if (e) return hip_fail(e, to_host ? "hipMemcpyAsync device-to-host" : "hipMemcpyAsync host-to-device");
    if (hipError_t e2 = hipEventRecord(static_cast<hipEvent_t>(p->ev_buf[i]), side)) return hip_fail(e2, "hipEventRecord");
    p->swapped_once = true;
    return RESHARD_OK;
}

// Makes the side stream wait for everything queued on `stream` so far.
int order_after(reshard_plan *p, void *stream) {
    hipEvent_t ready = static_cast<hipEvent_t>(p->ev_ready);
    if (hipError_t e = hipEventRecord(ready, static_cast<hipStream_t>(stream))) return hip_fail(e, "hipEventRecord");
    if (hipError_t e = hipStreamWaitEvent(static_cast<hipStream_t>(p->side_stream), ready, 0)) return hip_fail(e, "hipStreamWaitEvent");
    return RESHARD_OK;
}

}  // namespace

extern "C" const char *reshard_last_error(void) { return last_error_cstr(); }

extern "C" const char *reshard_version(void) { return "reshard 0.1 gfx950"; }

extern "C" void reshard_set_host_limit(int64_t limit) { g_host_limit.store(limit); }

namespace {
int create_plan(const reshard_model_spec *spec, const reshard_layout *src, const reshard_layout *dst,
                const Tuning &tuning, reshard_plan **out) {
    if (spec->struct_size != sizeof(reshard_model_spec) || src->struct_size != sizeof(reshard_layout) ||
        dst->struct_size != sizeof(reshard_layout))
        return fail(RESHARD_ERR_INVALID_ARG, "struct_size does not match this library's headers");
    reshard_plan *p = nullptr;
    try {
        p = new reshard_plan();
        p->serial = ++g_plan_serial;
        p->spec = *spec;
        if (int rc = build_side(*spec, *src, true, p->src)) { delete p; return rc; }
        if (int rc = build_side(*spec, *dst, false, p->dst)) { delete p; return rc; }
        const int ns = int(p->src.buf_bytes.size()), nd = int(p->dst.buf_bytes.size());
        if (int rc = compile_descriptors(*spec, p->src, p->dst, p->descs)) { delete p; return rc; }
        p->tuning = tuning;
        p->fast_rows = tuning.transpose_rows;
        p->fast_cols = tuning.transpose_cols;
        if (!transpose_shape_ok(spec->elem_bytes, p->fast_rows, p->fast_cols))
            transpose_default_shape(spec->elem_bytes, p->fast_rows, p->fast_cols);
        if (int rc = cut_tiles(p->descs, ns, tuning, p->fast_rows, p->fast_cols, p->classes)) {
            delete p;
            return rc;
        }
        // the kernels get the pointers of the used buffers only: renumber the tiles' buffer indices
        p->src_slot.assign(ns, -1);
        p->dst_slot.assign(nd, -1);
        for (int i = 0; i < ns; ++i)
            if (p->src.used[i]) {
                p->src_slot[i] = int(p->slot_buf.size());
                p->slot_buf.push_back(i);
            }
        p->num_src_slots = int(p->slot_buf.size());
        for (int j = 0; j < nd; ++j)
            if (p->dst.used[j]) {
                p->dst_slot[j] = int(p->slot_buf.size());
                p->slot_buf.push_back(j);
            }
        if (p->slot_buf.size() > size_t(RESHARD_MAX_BUFFERS)) {
            delete p;
            return fail(RESHARD_ERR_UNSUPPORTED, "used source plus destination buffers exceed RESHARD_MAX_BUFFERS");
        }
        for (TileClass &c : p->classes)
            for (Tile &t : c.tiles) {
                t.src_buf = uint16_t(p->src_slot[t.src_buf]);
                t.dst_buf = uint16_t(p->dst_slot[t.dst_buf - ns]);
            }
        p->info.num_tiles = p->info.num_transpose_tiles = 0;
        for (const TileClass &c : p->classes) {
            if (c.tiles.size() > 0x7FFFFFF0ull) {
                delete p;
                return fail(RESHARD_ERR_UNSUPPORTED, "too many tiles");
            }
            p->info.num_tiles += int64_t(c.tiles.size());
            if (c.kind != 0) p->info.num_transpose_tiles += int64_t(c.tiles.size());
        }
        p->info.num_src_bufs = ns;
        p->info.num_dst_bufs = nd;
        p->info.num_descs = int64_t(p->descs.size());
        int64_t moved = 0;
        for (const reshard_desc &d : p->descs) moved += d.rows * d.row_bytes;
        p->info.bytes_moved = moved;
        p->info.table_bytes = p->info.num_tiles * int64_t(sizeof(Tile));
        p->src_ptrs.assign(ns, nullptr);
        p->dst_ptrs.assign(nd, nullptr);
        p->host_copy.assign(ns, nullptr);
        p->buf_state.assign(ns, RESHARD_SRC_UNBOUND);
    } catch (const std::bad_alloc &) {
        delete p;
        return fail(RESHARD_ERR_OOM, "out of host memory while building the plan");
    }
    *out = p;
    return RESHARD_OK;
}
}  // namespace

extern "C" int reshard_plan_create(const reshard_model_spec *spec, const reshard_layout *src,
                                   const reshard_layout *dst, reshard_plan **out) {
    return reshard_plan_create_tuned(spec, src, dst, nullptr, out);
}

extern "C" int reshard_plan_create_tuned(const reshard_model_spec *spec, const reshard_layout *src,
                                         const reshard_layout *dst, const reshard_tuning *tuning, reshard_plan **out) {
    if (!spec || !src || !dst || !out) return fail(RESHARD_ERR_INVALID_ARG, "NULL argument");
    *out = nullptr;
    Tuning tn = current_tuning();
    if (tuning)
        if (int rc = tuning_from_abi(tuning, tn)) return rc;
    return create_plan(spec, src, dst, tn, out);
}

extern "C" int reshard_set_tuning(const reshard_tuning *t) {
    Tuning n;
    if (int rc = tuning_from_abi(t, n)) return rc;
    set_default_tuning(n);
    return RESHARD_OK;
}

extern "C" int reshard_get_tuning(reshard_tuning *out) {
    if (!out) return fail(RESHARD_ERR_INVALID_ARG, "out is NULL");
    tuning_to_abi(current_tuning(), out);
    return RESHARD_OK;
}

extern "C" int reshard_plan_set_tuning(reshard_plan *p, const reshard_tuning *t) {
    if (!p) return fail(RESHARD_ERR_INVALID_ARG, "plan is NULL");
    Tuning n;
    if (int rc = tuning_from_abi(t, n)) return rc;
    // the tiles are cut: what shaped them stays (a zero field means "as the plan has it" here)
    if ((t && t->tile_bytes && t->tile_bytes != p->tuning.tile_bytes) ||
        (t && t->transpose_rows && t->transpose_rows != p->tuning.transpose_rows) ||
        (t && t->transpose_cols && t->transpose_cols != p->tuning.transpose_cols))
        return fail(RESHARD_ERR_INVALID_ARG, "tile_bytes and the transposing tile shape are fixed when the plan is created");
    n.tile_bytes = p->tuning.tile_bytes;
    n.transpose_rows = p->tuning.transpose_rows;
    n.transpose_cols = p->tuning.transpose_cols;
    if (p->d_tiles || !(t && t->table_copies)) n.table_copies = p->tuning.table_copies;  // fixed once the table is on the device
    p->tuning = n;
    return RESHARD_OK;
}

extern "C" int reshard_plan_get_tuning(const reshard_plan *p, reshard_tuning *out) {
    if (!p || !out) return fail(RESHARD_ERR_INVALID_ARG, "NULL argument");
    tuning_to_abi(p->tuning, out);
    return RESHARD_OK;
}

extern "C" int reshard_plan_destroy(reshard_plan *p) {
    if (!p) return RESHARD_OK;
    for (size_t i = 0; i < p->buf_state.size(); ++i)  // copies still in flight use the host blocks
        if (p->src.used[i] && (p->buf_state[i] == RESHARD_SRC_SWAPPING_OUT || p->buf_state[i] == RESHARD_SRC_SWAPPING_IN))
            (void)hipEventSynchronize(static_cast<hipEvent_t>(p->ev_buf[i]));
    free_host_copies(p);
    if (p->side_stream) (void)hipStreamDestroy(static_cast<hipStream_t>(p->side_stream));
    if (p->ev_ready) (void)hipEventDestroy(static_cast<hipEvent_t>(p->ev_ready));
    if (p->ev_exec) (void)hipEventDestroy(static_cast<hipEvent_t>(p->ev_exec));
    for (void *ev : p->ev_buf)
        if (ev) (void)hipEventDestroy(static_cast<hipEvent_t>(ev));
    if (p->d_tiles) (void)hipFree(p->d_tiles);
    if (p->d_by_src) (void)hipFree(p->d_by_src);
    delete p;
    return RESHARD_OK;
}

extern "C" int reshard_plan_num_bufs(const reshard_plan *plan, int side) {
    const Side *s = side_of(plan, side);
    if (!s) return fail(RESHARD_ERR_INVALID_ARG, "bad plan or side");
    return int(s->buf_bytes.size());
}

extern "C" int64_t reshard_plan_buf_bytes(const reshard_plan *plan, int side, int index) {
    const Side *s = side_of(plan, side);
    if (!s || index < 0 || index >= int(s->buf_bytes.size())) return fail(RESHARD_ERR_INVALID_ARG, "bad plan, side or index");
    return s->buf_bytes[index];
}

extern "C" int reshard_plan_buf_used(const reshard_plan *plan, int side, int index) {
    const Side *s = side_of(plan, side);
    if (!s || index < 0 || index >= int(s->buf_bytes.size())) return fail(RESHARD_ERR_INVALID_ARG, "bad plan, side or index");
    return s->used[index];
}

extern "C" int64_t reshard_plan_num_tensors(const reshard_plan *plan, int side) {
    const Side *s = side_of(plan, side);
    if (!s) return fail(RESHARD_ERR_INVALID_ARG, "bad plan or side");
    return int64_t(s->tensors.size());
}

extern "C" int reshard_plan_tensor(const reshard_plan *plan, int side, int64_t index, reshard_tensor_info *out) {
    const Side *s = side_of(plan, side);
    if (!s || !out || index < 0 || index >= int64_t(s->tensors.size())) return fail(RESHARD_ERR_INVALID_ARG, "bad plan, side, index or out");
    *out = s->tensors[size_t(index)];
    return RESHARD_OK;
}

extern "C" int reshard_plan_class_bytes(const reshard_plan *plan, int side, int64_t out[3]) {
    const Side *s = side_of(plan, side);
    if (!s || !out) return fail(RESHARD_ERR_INVALID_ARG, "bad plan, side or out");
    out[0] = out[1] = out[2] = 0;
    for (const reshard_tensor_info &t : s->tensors) out[t.weight_class] += t.bytes;
    return RESHARD_OK;
}

extern "C" double reshard_redundant_memory_bytes(int gen_dp, double tp_weight_bytes, int update_tp,
                                                 double ep_weight_bytes, int gen_ep) {
    if (gen_dp <= 0 || update_tp <= 0 || gen_ep <= 0) return -1.0;
    return gen_dp * (tp_weight_bytes / update_tp + ep_weight_bytes / gen_ep);
}

extern "C" int reshard_plan_get_info(const reshard_plan *plan, reshard_plan_info *out) {
    if (!plan || !out) return fail(RESHARD_ERR_INVALID_ARG, "NULL argument");
    *out = plan->info;
    return RESHARD_OK;
}

extern "C" int reshard_plan_desc(const reshard_plan *plan, int64_t index, reshard_desc *out) {
    if (!plan || !out || index < 0 || index >= int64_t(plan->descs.size())) return fail(RESHARD_ERR_INVALID_ARG, "bad plan, index or out");
    *out = plan->descs[size_t(index)];
    return RESHARD_OK;
}

extern "C" int reshard_plan_tile(const reshard_plan *plan, int64_t index, reshard_tile *out) {
    if (!plan || !out || index < 0 || index >= plan->info.num_tiles) return fail(RESHARD_ERR_INVALID_ARG, "bad plan, index or out");
    size_t cls = 0, at = size_t(index);
    while (at >= plan->classes[cls].tiles.size()) at -= plan->classes[cls++].tiles.size();
    const TileClass &c = plan->classes[cls];
    const Tile &t = c.tiles[at];
    out->src_buf = plan->slot_buf[t.src_buf];
    out->dst_buf = plan->slot_buf[t.dst_buf];
    out->kind = t.kind;
    // 0 copy; 1 register transpose of the preferred shape; 2 register transpose of another shape; 3 generic
    out->tile_class = c.kind == 0 ? 0 : c.kind == 2 ? 3 : cls == 1 ? 1 : 2;
    out->src_off = int64_t(t.src_off);
    out->dst_off = int64_t(t.dst_off);
    out->rows = t.rows;
    out->row_units = t.row_units;
    out->src_stride = t.src_stride;
    out->dst_stride = t.dst_stride;
    out->vec_bytes = 1 << t.vec_log2;
    out->order = 0;
    out->sources = 1;
    out->phase = 0;
    if (c.kind == 0) {
        // row blocks that have a gathered form go out in the XCD-contiguous order only, that form in the woven order only
        if (at >= size_t(c.num_blocks - c.num_regathered) && at < size_t(c.num_blocks)) out->order = 1;
        if (t.kind == 2) {
            const uint32_t c0 = t.src_stride & 0xFFFFu, j0 = (t.src_stride >> 16) & 0xFFu, lk = t.src_stride >> 24;
            out->order = 2;
            out->sources = int64_t(1) << lk;
            out->phase = int64_t(j0) * t.row_units + c0;
            out->src_stride = int64_t(t.dst_stride) * 16;
            out->dst_stride = 0;
        }
    }
    return RESHARD_OK;
}

extern "C" int reshard_plan_prepare(reshard_plan *p) {
    if (!p) return fail(RESHARD_ERR_INVALID_ARG, "plan is NULL");
    return ensure_device_table(p);
}

extern "C" int reshard_bind_src(reshard_plan *p, const void *const *src_ptrs) {
    if (!p) return fail(RESHARD_ERR_INVALID_ARG, "plan is NULL");
    if (p->state != RESHARD_SRC_UNBOUND && p->state != RESHARD_SRC_RESIDENT && p->state != RESHARD_SRC_ON_HOST &&
        p->state != RESHARD_SRC_RELEASED)
        return fail(RESHARD_ERR_BAD_STATE, "swap copies are in flight, or the buffers are in different states");
    if (int rc = check_ptrs(p->src, src_ptrs, "src_ptrs")) return rc;
    for (size_t i = 0; i < p->src_ptrs.size(); ++i) p->src_ptrs[i] = p->src.used[i] ? src_ptrs[i] : nullptr;
    set_all(p, p->state == RESHARD_SRC_UNBOUND ? RESHARD_SRC_RESIDENT
             : p->state == RESHARD_SRC_RELEASED ? RESHARD_SRC_ON_HOST : p->state);
    return RESHARD_OK;
}

namespace {
// reshard_execute and reshard_execute_noalloc: the same checks, binding and ledger; they differ in
// where the kernels read the tile table from (plan-owned device memory / the static device array).
int execute_common(reshard_plan *p, const void *const *src_ptrs, void *const *dst_ptrs, void *stream, bool static_table) {
    if (!p) return fail(RESHARD_ERR_INVALID_ARG, "plan is NULL");
    if (static_table && p->info.table_bytes > int64_t(RESHARD_STATIC_TABLE_BYTES))
        return fail(RESHARD_ERR_UNSUPPORTED, "the plan's tile table (" + std::to_string(p->info.table_bytes) +
                    " bytes) does not fit the static device array of " + std::to_string(RESHARD_STATIC_TABLE_BYTES) +
                    " bytes: create the plan with a larger tile_bytes, or use reshard_execute");
    // while a swap-out is in flight the sources are still valid in HBM and only read
    const bool swapping_out = p->state == RESHARD_SRC_SWAPPING_OUT;
    if (p->state != RESHARD_SRC_UNBOUND && p->state != RESHARD_SRC_RESIDENT && !swapping_out)
        return fail(RESHARD_ERR_BAD_STATE, "the source weights are not (all) resident on the device");
    if (int rc = check_ptrs(p->src, src_ptrs, "src_ptrs")) return rc;
    if (swapping_out)
        for (size_t i = 0; i < p->src_ptrs.size(); ++i)
            if (p->src.used[i] && src_ptrs[i] != p->src_ptrs[i])
                return fail(RESHARD_ERR_BAD_STATE, "a swap-out of other source pointers is in flight");
    if (int rc = check_ptrs(p->dst, reinterpret_cast<const void *const *>(dst_ptrs), "dst_ptrs")) return rc;
    for (size_t i = 0; i < p->src.buf_bytes.size(); ++i) {
        if (!p->src.used[i]) continue;
        for (size_t j = 0; j < p->dst.buf_bytes.size(); ++j)
            if (p->dst.used[j] && overlaps(src_ptrs[i], p->src.buf_bytes[i], dst_ptrs[j], p->dst.buf_bytes[j]))
                return fail(RESHARD_ERR_INVALID_ARG, "a source and a destination buffer overlap");
    }
    if (swapping_out) {
        // the event recorded below is waited for on the host later, which a captured record cannot serve
        hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
        if (hipError_t e = hipStreamIsCapturing(static_cast<hipStream_t>(stream), &cap)) return hip_fail(e, "hipStreamIsCapturing");
        if (cap != hipStreamCaptureStatusNone)
            return fail(RESHARD_ERR_BAD_STATE, "an execute cannot be captured into a graph while a swap-out is in flight");
    }
    if (!static_table)
        if (int rc = ensure_device_table(p)) return rc;
    for (size_t i = 0; i < p->src_ptrs.size(); ++i) p->src_ptrs[i] = p->src.used[i] ? src_ptrs[i] : nullptr;
    for (size_t j = 0; j < p->dst_ptrs.size(); ++j) p->dst_ptrs[j] = p->dst.used[j] ? dst_ptrs[j] : nullptr;
    if (int rc = static_table ? launch_repack_static(p, static_cast<hipStream_t>(stream))
                              : launch_repack(p, static_cast<hipStream_t>(stream)))
        return rc;
    if (swapping_out) {
        // reshard_swap_wait must not report the sources free to go before this repack has read them
        p->exec_during_swap = true;
        if (hipError_t e = hipEventRecord(static_cast<hipEvent_t>(p->ev_exec), static_cast<hipStream_t>(stream)))
            return hip_fail(e, "hipEventRecord");
    }
    p->dst_bound = true;
    p->dst_live = used_bytes(p->dst);
    if (swapping_out) recompute(p);
    else set_all(p, RESHARD_SRC_RESIDENT);
    return RESHARD_OK;
}
}  // namespace

extern "C" int reshard_execute(reshard_plan *p, const void *const *src_ptrs, void *const *dst_ptrs, void *stream) {
    return execute_common(p, src_ptrs, dst_ptrs, stream, false);
}

extern "C" int reshard_execute_noalloc(reshard_plan *p, const void *const *src_ptrs, void *const *dst_ptrs, void *stream) {
    return execute_common(p, src_ptrs, dst_ptrs, stream, true);
}

extern "C" int reshard_execute_source(reshard_plan *p, int src_index, const void *src_ptr, void *const *dst_ptrs,
                                      void *stream) {
    if (!p) return fail(RESHARD_ERR_INVALID_ARG, "plan is NULL");
    if (src_index < 0 || src_index >= int(p->src.buf_bytes.size()) || !p->src.used[size_t(src_index)])
        return fail(RESHARD_ERR_INVALID_ARG, "src_index does not name a used source buffer");
    const size_t i = size_t(src_index);
    if (p->buf_state[i] != RESHARD_SRC_UNBOUND && p->buf_state[i] != RESHARD_SRC_RESIDENT)
        return fail(RESHARD_ERR_BAD_STATE, "this source buffer is not resident on the device");
    if (!src_ptr || reinterpret_cast<uintptr_t>(src_ptr) % 256)
        return fail(RESHARD_ERR_INVALID_ARG, "src_ptr is NULL or not 256-byte aligned");
    if (int rc = check_ptrs(p->dst, reinterpret_cast<const void *const *>(dst_ptrs), "dst_ptrs")) return rc;
    for (size_t j = 0; j < p->dst.buf_bytes.size(); ++j)
        if (p->dst.used[j] && overlaps(src_ptr, p->src.buf_bytes[i], dst_ptrs[j], p->dst.buf_bytes[j]))
            return fail(RESHARD_ERR_INVALID_ARG, "the source buffer overlaps a destination buffer");
    if (int rc = ensure_by_source_table(p)) return rc;
    p->src_ptrs[i] = src_ptr;
    for (size_t j = 0; j < p->dst_ptrs.size(); ++j) p->dst_ptrs[j] = p->dst.used[j] ? dst_ptrs[j] : nullptr;
    if (int rc = launch_source(p, src_index, static_cast<hipStream_t>(stream))) return rc;
    p->dst_bound = true;
    p->dst_live = used_bytes(p->dst);
    p->buf_state[i] = RESHARD_SRC_RESIDENT;
    recompute(p);
    return RESHARD_OK;
}

extern "C" int reshard_swap_out(reshard_plan *p, void *stream) {
    if (!p) return fail(RESHARD_ERR_INVALID_ARG, "plan is NULL");
    if (p->state != RESHARD_SRC_RESIDENT) return fail(RESHARD_ERR_BAD_STATE, "swap_out needs bound, resident source buffers");
    if (int rc = ensure_host_copies(p)) return rc;
    if (int rc = ensure_swap_objects(p)) return rc;
    if (int rc = order_after(p, stream)) return rc;
    // states change buffer by buffer, so that after a failure half way the copies already
    // queued are still waited for (the plan is then MIXED; reshard_swap_wait settles it)
    for (size_t i = 0; i < p->src_ptrs.size(); ++i) {
        if (!p->src.used[i]) continue;
        if (int rc = queue_copy(p, i, true)) { recompute(p); return rc; }
        p->buf_state[i] = RESHARD_SRC_SWAPPING_OUT;
    }
    recompute(p);
    return RESHARD_OK;
}

extern "C" int reshard_swap_out_source(reshard_plan *p, int src_index, void *stream) {
    if (!p) return fail(RESHARD_ERR_INVALID_ARG, "plan is NULL");
    if (src_index < 0 || src_index >= int(p->src.buf_bytes.size()) || !p->src.used[size_t(src_index)])
        return fail(RESHARD_ERR_INVALID_ARG, "src_index does not name a used source buffer");
    const size_t i = size_t(src_index);
    if (p->buf_state[i] != RESHARD_SRC_RESIDENT) return fail(RESHARD_ERR_BAD_STATE, "this source buffer is not bound and resident");
    if (int rc = ensure_host_copies(p, src_index)) return rc;
    if (int rc = ensure_swap_objects(p)) return rc;
    if (int rc = order_after(p, stream)) return rc;
    if (int rc = queue_copy(p, i, true)) return rc;
    p->buf_state[i] = RESHARD_SRC_SWAPPING_OUT;
    recompute(p);
    return RESHARD_OK;
}

extern "C" int reshard_swap_in(reshard_plan *p, void *stream) {
    if (!p) return fail(RESHARD_ERR_INVALID_ARG, "plan is NULL");
    if (p->state == RESHARD_SRC_RELEASED) return fail(RESHARD_ERR_BAD_STATE, "the device copy was released: bind new source pointers first");
    if (p->state != RESHARD_SRC_ON_HOST) return fail(RESHARD_ERR_BAD_STATE, "swap_in needs a completed swap_out of every buffer");
    if (int rc = ensure_swap_objects(p)) return rc;
    // work already queued on `stream` may still use the memory being overwritten
    if (int rc = order_after(p, stream)) return rc;
    size_t last = 0;
    for (size_t i = 0; i < p->src_ptrs.size(); ++i) {
        if (!p->src.used[i]) continue;
        if (int rc = queue_copy(p, i, false)) { recompute(p); return rc; }
        p->buf_state[i] = RESHARD_SRC_SWAPPING_IN;
        last = i;
    }
    recompute(p);
    // the copies run in buffer order, so the last buffer's event marks the end of all of them
    if (hipError_t e = hipStreamWaitEvent(static_cast<hipStream_t>(stream), static_cast<hipEvent_t>(p->ev_buf[last]), 0))
        return hip_fail(e, "hipStreamWaitEvent");
    return RESHARD_OK;
}

extern "C" int reshard_swap_in_source(reshard_plan *p, int src_index, void *src_ptr, void *stream) {
    if (!p) return fail(RESHARD_ERR_INVALID_ARG, "plan is NULL");
    if (src_index < 0 || src_index >= int(p->src.buf_bytes.size()) || !p->src.used[size_t(src_index)])
        return fail(RESHARD_ERR_INVALID_ARG, "src_index does not name a used source buffer");
    const size_t i = size_t(src_index);
    const int st = p->buf_state[i];
    if (st != RESHARD_SRC_ON_HOST && st != RESHARD_SRC_RELEASED)
        return fail(RESHARD_ERR_BAD_STATE, "this source buffer has no completed swap-out to bring back");
    if (reinterpret_cast<uintptr_t>(src_ptr) % 256) return fail(RESHARD_ERR_INVALID_ARG, "src_ptr is not 256-byte aligned");
    if (!src_ptr && !p->src_ptrs[i])
        return fail(RESHARD_ERR_BAD_STATE, "the device copy was released: give the buffer's new device pointer");
    if (int rc = ensure_swap_objects(p)) return rc;
    if (int rc = order_after(p, stream)) return rc;
    if (src_ptr) p->src_ptrs[i] = src_ptr;
    p->buf_state[i] = RESHARD_SRC_ON_HOST;
    if (int rc = queue_copy(p, i, false)) { recompute(p); return rc; }
    p->buf_state[i] = RESHARD_SRC_SWAPPING_IN;
    recompute(p);
    if (hipError_t e = hipStreamWaitEvent(static_cast<hipStream_t>(stream), static_cast<hipEvent_t>(p->ev_buf[i]), 0))
        return hip_fail(e, "hipStreamWaitEvent");
    return RESHARD_OK;
}

extern "C" int reshard_swap_wait_buffer(reshard_plan *p, int index, void *stream, int host_wait) {
    if (!p) return fail(RESHARD_ERR_INVALID_ARG, "plan is NULL");
    if (index < 0 || index >= int(p->src.buf_bytes.size()) || !p->src.used[size_t(index)])
        return fail(RESHARD_ERR_INVALID_ARG, "index does not name a used source buffer");
    if (!p->swapped_once || p->ev_buf.empty() || !p->ev_buf[size_t(index)])
        return fail(RESHARD_ERR_BAD_STATE, "no swap has been started on this plan");
    if (host_wait) {
        // also completes this buffer's state change (SWAPPING_OUT -> ON_HOST, SWAPPING_IN -> RESIDENT)
        const int st = p->buf_state[size_t(index)];
        if (st == RESHARD_SRC_SWAPPING_OUT || st == RESHARD_SRC_SWAPPING_IN) {
            if (int rc = finish_buffer(p, size_t(index))) return rc;
            recompute(p);
        } else if (hipError_t e = hipEventSynchronize(static_cast<hipEvent_t>(p->ev_buf[size_t(index)]))) {
            return hip_fail(e, "hipEventSynchronize");
        }
    } else if (hipError_t e = hipStreamWaitEvent(static_cast<hipStream_t>(stream), static_cast<hipEvent_t>(p->ev_buf[size_t(index)]), 0)) {
        return hip_fail(e, "hipStreamWaitEvent");
    }
    return RESHARD_OK;
}

extern "C" int reshard_swap_wait(reshard_plan *p) {
    if (!p) return fail(RESHARD_ERR_INVALID_ARG, "plan is NULL");
    return finish_swap(p);
}

extern "C" int reshard_mark_src_released(reshard_plan *p) {
    if (!p) return fail(RESHARD_ERR_INVALID_ARG, "plan is NULL");
    if (p->state != RESHARD_SRC_ON_HOST) return fail(RESHARD_ERR_BAD_STATE, "sources can be released only after a completed swap_out");
    std::fill(p->src_ptrs.begin(), p->src_ptrs.end(), nullptr);
    set_all(p, RESHARD_SRC_RELEASED);
    return RESHARD_OK;
}

extern "C" int reshard_mark_src_buffer_released(reshard_plan *p, int src_index) {
    if (!p) return fail(RESHARD_ERR_INVALID_ARG, "plan is NULL");
    if (src_index < 0 || src_index >= int(p->src.buf_bytes.size()) || !p->src.used[size_t(src_index)])
        return fail(RESHARD_ERR_INVALID_ARG, "src_index does not name a used source buffer");
    if (p->buf_state[size_t(src_index)] != RESHARD_SRC_ON_HOST)
        return fail(RESHARD_ERR_BAD_STATE, "a source buffer can be released only after its swap-out has completed");
    p->src_ptrs[size_t(src_index)] = nullptr;
    p->buf_state[size_t(src_index)] = RESHARD_SRC_RELEASED;
    recompute(p);
    return RESHARD_OK;
}

extern "C" int reshard_mark_dst_released(reshard_plan *p) {
    if (!p) return fail(RESHARD_ERR_INVALID_ARG, "plan is NULL");
    p->dst_live = 0;
    p->dst_bound = false;
    std::fill(p->dst_ptrs.begin(), p->dst_ptrs.end(), nullptr);
    return RESHARD_OK;
}

extern "C" int reshard_reserve_host(reshard_plan *p) {
    if (!p) return fail(RESHARD_ERR_INVALID_ARG, "plan is NULL");
    return ensure_host_copies(p);
}

extern "C" int reshard_release_host(reshard_plan *p) {
    if (!p) return fail(RESHARD_ERR_INVALID_ARG, "plan is NULL");
    if (p->state != RESHARD_SRC_UNBOUND && p->state != RESHARD_SRC_RESIDENT)
        return fail(RESHARD_ERR_BAD_STATE, "the host copy is the only copy, or a swap is in flight");
    free_host_copies(p);
    return RESHARD_OK;
}

extern "C" const void *reshard_host_copy(const reshard_plan *p, int index) {
    if (!p || index < 0 || index >= int(p->host_copy.size())) return nullptr;
    return p->host_copy[size_t(index)];
}

extern "C" int reshard_src_buffer_state(const reshard_plan *p, int src_index) {
    if (!p || src_index < 0 || src_index >= int(p->buf_state.size())) return fail(RESHARD_ERR_INVALID_ARG, "bad plan or index");
    return p->buf_state[size_t(src_index)];
}

extern "C" int reshard_mem_stats(const reshard_plan *p, reshard_mem_stats_t *out) {
    if (!p || !out) return fail(RESHARD_ERR_INVALID_ARG, "NULL argument");
    out->src_live = p->src_live;
    out->dst_live = p->dst_live;
    out->host_pinned = p->host_pinned;
    out->peak_device = p->peak_device;
    out->released = p->released;
    out->state = p->state;
    return RESHARD_OK;
}
