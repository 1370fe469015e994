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
int launch_repack(reshard_plan *plan, hipStream_t stream);
}  // namespace reshard

using namespace reshard;

namespace {

std::atomic<int64_t> g_host_limit{-1};

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

int ensure_swap_objects(reshard_plan *p) {
    if (!p->side_stream) {
        hipStream_t s;
        if (hipError_t e = hipStreamCreateWithFlags(&s, hipStreamNonBlocking)) return hip_fail(e, "hipStreamCreate");
        p->side_stream = s;
    }
    if (!p->ev_ready) {
        hipEvent_t ev;
        if (hipError_t e = hipEventCreateWithFlags(&ev, hipEventDisableTiming)) return hip_fail(e, "hipEventCreate");
        p->ev_ready = ev;
    }
    if (!p->ev_done) {
        hipEvent_t ev;
        if (hipError_t e = hipEventCreateWithFlags(&ev, hipEventDisableTiming)) return hip_fail(e, "hipEventCreate");
        p->ev_done = ev;
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

// All-or-nothing allocation of the pinned copies.
int ensure_host_copies(reshard_plan *p) {
    const Side &s = p->src;
    int64_t need = 0;
    for (size_t i = 0; i < s.buf_bytes.size(); ++i)
        if (s.used[i] && !p->host_copy[i]) need += s.buf_bytes[i];
    if (need == 0) return RESHARD_OK;
    const int64_t limit = g_host_limit.load();
    if (limit >= 0 && p->host_pinned + need > limit)
        return fail(RESHARD_ERR_HOST_OOM, "pinned host allocation refused by the configured limit");
    std::vector<size_t> fresh;
    for (size_t i = 0; i < s.buf_bytes.size(); ++i) {
        if (!s.used[i] || p->host_copy[i]) continue;
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

int finish_swap(reshard_plan *p) {
    if (p->state != RESHARD_SRC_SWAPPING_OUT && p->state != RESHARD_SRC_SWAPPING_IN) return RESHARD_OK;
    if (hipError_t e = hipEventSynchronize(static_cast<hipEvent_t>(p->ev_done))) return hip_fail(e, "hipEventSynchronize");
    p->state = p->state == RESHARD_SRC_SWAPPING_OUT ? RESHARD_SRC_ON_HOST : RESHARD_SRC_RESIDENT;
    return RESHARD_OK;
}

}  // namespace

extern "C" const char *reshard_last_error(void) { return last_error_cstr(); }

extern "C" const char *reshard_version(void) { return "reshard 0.1 gfx950"; }

extern "C" void reshard_set_host_limit(int64_t limit) { g_host_limit.store(limit); }

extern "C" int reshard_plan_create(const reshard_model_spec *spec, const reshard_layout *src,
                                   const reshard_layout *dst, reshard_plan **out) {
    if (!spec || !src || !dst || !out) return fail(RESHARD_ERR_INVALID_ARG, "NULL argument");
    *out = nullptr;
    if (spec->struct_size != sizeof(reshard_model_spec) || src->struct_size != sizeof(reshard_layout) ||
        dst->struct_size != sizeof(reshard_layout))
        return fail(RESHARD_ERR_INVALID_ARG, "struct_size does not match this library's headers");
    reshard_plan *p = nullptr;
    try {
        p = new reshard_plan();
        p->spec = *spec;
        if (int rc = build_side(*spec, *src, true, p->src)) { delete p; return rc; }
        if (int rc = build_side(*spec, *dst, false, p->dst)) { delete p; return rc; }
        const int ns = int(p->src.buf_bytes.size()), nd = int(p->dst.buf_bytes.size());
        if (ns + nd > RESHARD_MAX_BUFFERS) {
            delete p;
            return fail(RESHARD_ERR_UNSUPPORTED, "source plus destination buffers exceed RESHARD_MAX_BUFFERS");
        }
        if (int rc = compile_descriptors(*spec, p->src, p->dst, p->descs)) { delete p; return rc; }
        const Tuning tuning = current_tuning();
        p->fast_rows = tuning.transpose_rows;
        p->fast_cols = tuning.transpose_cols;
        if (int rc = cut_tiles(p->descs, ns, tuning, p->copy_tiles, p->fast_transpose_tiles, p->edge_transpose_tiles,
                               p->transpose_tiles)) {
            delete p;
            return rc;
        }
        if (p->copy_tiles.size() > 0x7FFFFFF0ull || p->transpose_tiles.size() > 0x7FFFFFF0ull ||
            p->fast_transpose_tiles.size() > 0x7FFFFFF0ull || p->edge_transpose_tiles.size() > 0x7FFFFFF0ull) {
            delete p;
            return fail(RESHARD_ERR_UNSUPPORTED, "too many tiles");
        }
        p->info.num_src_bufs = ns;
        p->info.num_dst_bufs = nd;
        p->info.num_descs = int64_t(p->descs.size());
        p->info.num_transpose_tiles = int64_t(p->transpose_tiles.size() + p->fast_transpose_tiles.size() +
                                              p->edge_transpose_tiles.size());
        p->info.num_tiles = int64_t(p->copy_tiles.size()) + p->info.num_transpose_tiles;
        int64_t moved = 0;
        for (const reshard_desc &d : p->descs) moved += d.rows * d.row_bytes;
        p->info.bytes_moved = moved;
        p->info.table_bytes = p->info.num_tiles * int64_t(sizeof(Tile));
        p->src_ptrs.assign(ns, nullptr);
        p->dst_ptrs.assign(nd, nullptr);
        p->host_copy.assign(ns, nullptr);
    } catch (const std::bad_alloc &) {
        delete p;
        return fail(RESHARD_ERR_OOM, "out of host memory while building the plan");
    }
    *out = p;
    return RESHARD_OK;
}

extern "C" int reshard_plan_destroy(reshard_plan *p) {
    if (!p) return RESHARD_OK;
    if (p->state == RESHARD_SRC_SWAPPING_OUT || p->state == RESHARD_SRC_SWAPPING_IN)
        (void)hipEventSynchronize(static_cast<hipEvent_t>(p->ev_done));
    free_host_copies(p);
    if (p->side_stream) (void)hipStreamDestroy(static_cast<hipStream_t>(p->side_stream));
    if (p->ev_ready) (void)hipEventDestroy(static_cast<hipEvent_t>(p->ev_ready));
    if (p->ev_done) (void)hipEventDestroy(static_cast<hipEvent_t>(p->ev_done));
    for (void *ev : p->ev_buf)
        if (ev) (void)hipEventDestroy(static_cast<hipEvent_t>(ev));
    if (p->d_tiles) (void)hipFree(p->d_tiles);
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
    const std::vector<Tile> *lists[4] = {&plan->copy_tiles, &plan->fast_transpose_tiles, &plan->edge_transpose_tiles,
                                         &plan->transpose_tiles};
    int cls = 0;
    size_t at = size_t(index);
    while (at >= lists[cls]->size()) at -= lists[cls++]->size();
    const Tile &t = (*lists[cls])[at];
    out->src_buf = t.src_buf;
    out->dst_buf = int32_t(t.dst_buf) - plan->info.num_src_bufs;
    out->kind = t.kind;
    out->tile_class = cls;
    out->src_off = int64_t(t.src_off);
    out->dst_off = int64_t(t.dst_off);
    out->rows = t.rows;
    out->row_units = t.row_units;
    out->src_stride = t.src_stride;
    out->dst_stride = t.dst_stride;
    out->vec_bytes = 1 << t.vec_log2;
    out->reserved_ = 0;
    return RESHARD_OK;
}

extern "C" int reshard_plan_prepare(reshard_plan *p) {
    if (!p) return fail(RESHARD_ERR_INVALID_ARG, "plan is NULL");
    return ensure_device_table(p);
}

extern "C" int reshard_bind_src(reshard_plan *p, const void *const *src_ptrs) {
    if (!p) return fail(RESHARD_ERR_INVALID_ARG, "plan is NULL");
    if (p->state == RESHARD_SRC_SWAPPING_OUT || p->state == RESHARD_SRC_SWAPPING_IN)
        return fail(RESHARD_ERR_BAD_STATE, "swap copies are in flight; call reshard_swap_wait first");
    if (int rc = check_ptrs(p->src, src_ptrs, "src_ptrs")) return rc;
    for (size_t i = 0; i < p->src_ptrs.size(); ++i) p->src_ptrs[i] = p->src.used[i] ? src_ptrs[i] : nullptr;
    p->src_live = used_bytes(p->src);
    if (p->state == RESHARD_SRC_UNBOUND) p->state = RESHARD_SRC_RESIDENT;
    if (p->state == RESHARD_SRC_RELEASED) p->state = RESHARD_SRC_ON_HOST;
    p->touch_peak();
    return RESHARD_OK;
}

extern "C" int reshard_execute(reshard_plan *p, const void *const *src_ptrs, void *const *dst_ptrs, void *stream) {
    if (!p) return fail(RESHARD_ERR_INVALID_ARG, "plan is NULL");
    // while a swap-out is in flight the sources are still valid in HBM and only read
    const bool swapping_out = p->state == RESHARD_SRC_SWAPPING_OUT;
    if (p->state != RESHARD_SRC_UNBOUND && p->state != RESHARD_SRC_RESIDENT && !swapping_out)
        return fail(RESHARD_ERR_BAD_STATE, "the source weights are not resident on the device");
    if (int rc = check_ptrs(p->src, src_ptrs, "src_ptrs")) return rc;
    if (swapping_out)
        for (size_t i = 0; i < p->src_ptrs.size(); ++i)
            if (p->src.used[i] && src_ptrs[i] != p->src_ptrs[i])
                return fail(RESHARD_ERR_BAD_STATE, "a swap-out of other source pointers is in flight");
    if (int rc = check_ptrs(p->dst, reinterpret_cast<const void *const *>(dst_ptrs), "dst_ptrs")) return rc;
    // the two sets must not overlap
    for (size_t i = 0; i < p->src.buf_bytes.size(); ++i) {
        if (!p->src.used[i]) continue;
        const uintptr_t a0 = reinterpret_cast<uintptr_t>(src_ptrs[i]), a1 = a0 + uintptr_t(p->src.buf_bytes[i]);
        for (size_t j = 0; j < p->dst.buf_bytes.size(); ++j) {
            if (!p->dst.used[j]) continue;
            const uintptr_t b0 = reinterpret_cast<uintptr_t>(dst_ptrs[j]), b1 = b0 + uintptr_t(p->dst.buf_bytes[j]);
            if (a0 < b1 && b0 < a1) return fail(RESHARD_ERR_INVALID_ARG, "a source and a destination buffer overlap");
        }
    }
    if (int rc = ensure_device_table(p)) return rc;
    {
        int dev = -1;
        if (hipError_t e = hipGetDevice(&dev)) return hip_fail(e, "hipGetDevice");
        if (dev != p->device) return fail(RESHARD_ERR_INVALID_ARG, "the plan's tile table lives on another device than the current one");
    }
    for (size_t i = 0; i < p->src_ptrs.size(); ++i) p->src_ptrs[i] = p->src.used[i] ? src_ptrs[i] : nullptr;
    for (size_t j = 0; j < p->dst_ptrs.size(); ++j) p->dst_ptrs[j] = p->dst.used[j] ? dst_ptrs[j] : nullptr;
    if (int rc = launch_repack(p, static_cast<hipStream_t>(stream))) return rc;
    if (!swapping_out) p->state = RESHARD_SRC_RESIDENT;
    p->dst_bound = true;
    p->src_live = used_bytes(p->src);
    p->dst_live = used_bytes(p->dst);
    p->touch_peak();
    return RESHARD_OK;
}

extern "C" int reshard_swap_out(reshard_plan *p, void *stream) {
    if (!p) return fail(RESHARD_ERR_INVALID_ARG, "plan is NULL");
    if (p->state != RESHARD_SRC_RESIDENT) return fail(RESHARD_ERR_BAD_STATE, "swap_out needs bound, resident source buffers");
    if (int rc = ensure_host_copies(p)) return rc;
    if (int rc = ensure_swap_objects(p)) return rc;
    hipStream_t side = static_cast<hipStream_t>(p->side_stream);
    hipEvent_t ready = static_cast<hipEvent_t>(p->ev_ready), done = static_cast<hipEvent_t>(p->ev_done);
    if (hipError_t e = hipEventRecord(ready, static_cast<hipStream_t>(stream))) return hip_fail(e, "hipEventRecord");
    if (hipError_t e = hipStreamWaitEvent(side, ready, 0)) return hip_fail(e, "hipStreamWaitEvent");
    for (size_t i = 0; i < p->src_ptrs.size(); ++i) {
        if (!p->src.used[i]) continue;
        if (hipError_t e = hipMemcpyAsync(p->host_copy[i], p->src_ptrs[i], size_t(p->src.buf_bytes[i]), hipMemcpyDeviceToHost, side))
            return hip_fail(e, "hipMemcpyAsync device-to-host");
        if (hipError_t e = hipEventRecord(static_cast<hipEvent_t>(p->ev_buf[i]), side)) return hip_fail(e, "hipEventRecord");
    }
    p->swapped_once = true;
    if (hipError_t e = hipEventRecord(done, side)) return hip_fail(e, "hipEventRecord");
    p->state = RESHARD_SRC_SWAPPING_OUT;
    return RESHARD_OK;
}

extern "C" int reshard_swap_in(reshard_plan *p, void *stream) {
    if (!p) return fail(RESHARD_ERR_INVALID_ARG, "plan is NULL");
    if (p->state == RESHARD_SRC_RELEASED) return fail(RESHARD_ERR_BAD_STATE, "the device copy was released: bind new source pointers first");
    if (p->state != RESHARD_SRC_ON_HOST) return fail(RESHARD_ERR_BAD_STATE, "swap_in needs a completed swap_out");
    if (int rc = ensure_swap_objects(p)) return rc;
    hipStream_t side = static_cast<hipStream_t>(p->side_stream);
    hipEvent_t ready = static_cast<hipEvent_t>(p->ev_ready), done = static_cast<hipEvent_t>(p->ev_done);
    // work already queued on `stream` may still use the memory being overwritten
    if (hipError_t e = hipEventRecord(ready, static_cast<hipStream_t>(stream))) return hip_fail(e, "hipEventRecord");
    if (hipError_t e = hipStreamWaitEvent(side, ready, 0)) return hip_fail(e, "hipStreamWaitEvent");
    for (size_t i = 0; i < p->src_ptrs.size(); ++i) {
        if (!p->src.used[i]) continue;
        if (hipError_t e = hipMemcpyAsync(const_cast<void *>(p->src_ptrs[i]), p->host_copy[i], size_t(p->src.buf_bytes[i]), hipMemcpyHostToDevice, side))
            return hip_fail(e, "hipMemcpyAsync host-to-device");
        if (hipError_t e = hipEventRecord(static_cast<hipEvent_t>(p->ev_buf[i]), side)) return hip_fail(e, "hipEventRecord");
    }
    if (hipError_t e = hipEventRecord(done, side)) return hip_fail(e, "hipEventRecord");
    if (hipError_t e = hipStreamWaitEvent(static_cast<hipStream_t>(stream), done, 0)) return hip_fail(e, "hipStreamWaitEvent");
    p->state = RESHARD_SRC_SWAPPING_IN;
    return RESHARD_OK;
}

extern "C" int reshard_swap_wait_buffer(reshard_plan *p, int index, void *stream, int host_wait) {
    if (!p) return fail(RESHARD_ERR_INVALID_ARG, "plan is NULL");
    if (index < 0 || index >= int(p->src.buf_bytes.size()) || !p->src.used[size_t(index)])
        return fail(RESHARD_ERR_INVALID_ARG, "index does not name a used source buffer");
    if (!p->swapped_once || p->ev_buf.empty() || !p->ev_buf[size_t(index)])
        return fail(RESHARD_ERR_BAD_STATE, "no swap has been started on this plan");
    hipEvent_t ev = static_cast<hipEvent_t>(p->ev_buf[size_t(index)]);
    if (host_wait) {
        if (hipError_t e = hipEventSynchronize(ev)) return hip_fail(e, "hipEventSynchronize");
    } else if (hipError_t e = hipStreamWaitEvent(static_cast<hipStream_t>(stream), ev, 0)) {
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
    p->released = p->src_live;
    p->src_live = 0;
    std::fill(p->src_ptrs.begin(), p->src_ptrs.end(), nullptr);
    p->state = RESHARD_SRC_RELEASED;
    return RESHARD_OK;
}

extern "C" int reshard_mark_dst_released(reshard_plan *p) {
    if (!p) return fail(RESHARD_ERR_INVALID_ARG, "plan is NULL");
    p->dst_live = 0;
    p->dst_bound = false;
    std::fill(p->dst_ptrs.begin(), p->dst_ptrs.end(), nullptr);
    return RESHARD_OK;
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
