// Host-only driver for the C ABI (api.cpp + plan.cpp) built against tests/fake_hip under
// AddressSanitizer and UndefinedBehaviorSanitizer by tests/test_plan_sanitizers.py.  The two
// launch functions of the HIP file are replaced here by an interpreter of the tile table on host
// memory, so whole flows (execute, swap-out, release, re-bind, swap-in, streaming per buffer,
// error paths, destroy with copies pending) run through the real state machine and ledger, and
// the sanitizers see every allocation, copy and free the library makes.  Test infrastructure.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "internal.h"

long fake_hip_host_limit = -1, fake_hip_host_bytes = 0, fake_hip_copies = 0;

namespace reshard {
static void run_tile(const reshard_plan *p, const Tile &t) {
    const char *s = static_cast<const char *>(p->src_ptrs[size_t(p->slot_buf[t.src_buf])]) + t.src_off;
    char *d = static_cast<char *>(p->dst_ptrs[size_t(p->slot_buf[t.dst_buf])]) + t.dst_off;
    const size_t v = size_t(1) << t.vec_log2;
    if (t.kind == 2) {  // gathered: consecutive units of the destination, from 2^lk sources in turn
        const uint32_t c0 = t.src_stride & 0xFFFFu, j0 = (t.src_stride >> 16) & 0xFFu, lk = t.src_stride >> 24;
        for (uint32_t u = 0; u < t.rows; ++u) {
            const uint64_t w = uint64_t(j0) * t.row_units + c0 + u, seg = w / t.row_units, c = w % t.row_units;
            const char *sj = static_cast<const char *>(p->src_ptrs[size_t(p->slot_buf[t.src_buf + (seg & ((1u << lk) - 1))])]) + t.src_off;
            std::memcpy(d + size_t(u) * 16, sj + (seg >> lk) * t.dst_stride * 16 + c * 16, 16);
        }
        return;
    }
    for (uint32_t i = 0; i < t.rows; ++i)
        for (uint32_t k = 0; k < t.row_units; ++k)
            if (t.kind == 0) std::memcpy(d + size_t(i) * t.dst_stride + k * v, s + size_t(i) * t.src_stride + k * v, v);
            else std::memcpy(d + size_t(k) * t.dst_stride + i * v, s + size_t(i) * t.src_stride + k * v, v);
}
int ensure_device_table(reshard_plan *p) {
    if (!p->d_tiles) p->d_tiles = std::malloc(16);  // something for destroy to free
    return RESHARD_OK;
}
int ensure_by_source_table(reshard_plan *p) {
    if (!p->d_by_src) p->d_by_src = std::malloc(16);
    return RESHARD_OK;
}
int launch_repack(reshard_plan *p, hipStream_t) {
    const bool woven = (p->tuning.flags & 96) == 96 && p->tuning.block_threads == 1024 && p->tuning.blocks_per_cu == 0;
    for (const TileClass &c : p->classes)
        for (size_t i = 0; i < c.tiles.size(); ++i) {
            // the copy class holds some bytes twice: as row blocks and as gathered tiles
            if (c.kind == 0 && woven && i >= c.num_blocks - c.num_regathered && i < c.num_blocks) continue;
            if (c.kind == 0 && !woven && i >= size_t(c.num_blocks) + c.num_runs) continue;
            run_tile(p, c.tiles[i]);
        }
    return RESHARD_OK;
}
int launch_repack_static(reshard_plan *p, hipStream_t s) { return launch_repack(p, s); }
int launch_source(reshard_plan *p, int src_index, hipStream_t) {
    for (const TileClass &c : p->classes)
        for (const Tile &t : c.tiles)
            if (t.kind != 2 && p->slot_buf[t.src_buf] == src_index && t.src_buf < p->num_src_slots) run_tile(p, t);
    return RESHARD_OK;
}
}  // namespace reshard

#define REQUIRE(cond) do { if (!(cond)) { std::printf("line %d: %s is false (last error: %s)\n", __LINE__, #cond, reshard_last_error()); return 1; } } while (0)

static reshard_model_spec moe_spec(int eb) {
    reshard_model_spec s{};
    s.struct_size = sizeof s;
    s.family = RESHARD_MOE_GQA; s.L = 2; s.H = 64; s.nq = 4; s.nkv = 2; s.d = 16; s.V = 96; s.has_embeddings = 1;
    s.E = 4; s.Ie = 40; s.n_shared = 1; s.elem_bytes = eb; s.qkv_bias = 1;
    return s;
}
static reshard_layout lay(int kind, int tp, int pp, int ep, int grouped) {
    reshard_layout l{};
    l.struct_size = sizeof l;
    l.kind = kind; l.tp = tp; l.pp = pp; l.ep = ep; l.expert_layout = grouped; l.tp_rank_filter = l.ep_rank_filter = -1;
    return l;
}
struct Buffers {
    std::vector<void *> p;
    std::vector<int64_t> n;
    ~Buffers() { for (void *q : p) std::free(q); }
    void make(const reshard_plan *plan, int side, int fill) {
        const int nb = reshard_plan_num_bufs(plan, side);
        for (int i = 0; i < nb; ++i) {
            const int64_t bytes = reshard_plan_buf_bytes(plan, side, i);
            void *q = nullptr;
            if (reshard_plan_buf_used(plan, side, i)) {
                q = std::aligned_alloc(256, size_t(bytes));
                unsigned char *c = static_cast<unsigned char *>(q);
                for (int64_t k = 0; k < bytes; ++k) c[k] = fill < 0 ? (unsigned char)((k * 131 + i * 17) >> 2) : (unsigned char)fill;
            }
            p.push_back(q);
            n.push_back(bytes);
        }
    }
    bool same(const Buffers &o) const {
        for (size_t i = 0; i < p.size(); ++i)
            if (p[i] && std::memcmp(p[i], o.p[i], size_t(n[i]))) return false;
        return true;
    }
};

static int flows(int eb) {
    const reshard_model_spec spec = moe_spec(eb);
    const reshard_layout src = lay(RESHARD_TRAIN, 2, 2, 2, 1), dst = lay(RESHARD_GEN, 1, 1, 4, 0);
    reshard_plan *plan = nullptr, *stream_plan = nullptr;
    REQUIRE(reshard_plan_create(&spec, &src, &dst, &plan) == RESHARD_OK);
    REQUIRE(reshard_plan_create(&spec, &src, &dst, &stream_plan) == RESHARD_OK);
    const int ns = reshard_plan_num_bufs(plan, 0);
    Buffers S, D, D2, keep;
    S.make(plan, 0, -1);
    keep.make(plan, 0, -1);
    D.make(plan, 1, 0xA5);
    D2.make(plan, 1, 0xA5);
    reshard_mem_stats_t st;
    int64_t sbytes = 0, dbytes = 0;
    for (int i = 0; i < ns; ++i) sbytes += reshard_plan_buf_used(plan, 0, i) ? S.n[size_t(i)] : 0;
    for (size_t j = 0; j < D.n.size(); ++j) dbytes += D.n[j];

    // errors before anything is bound
    REQUIRE(reshard_swap_out(plan, nullptr) == RESHARD_ERR_BAD_STATE);
    REQUIRE(reshard_swap_in(plan, nullptr) == RESHARD_ERR_BAD_STATE);
    REQUIRE(reshard_mark_src_released(plan) == RESHARD_ERR_BAD_STATE);
    REQUIRE(reshard_swap_wait_buffer(plan, 0, nullptr, 1) == RESHARD_ERR_BAD_STATE);
    REQUIRE(reshard_execute(plan, nullptr, D.p.data(), nullptr) == RESHARD_ERR_INVALID_ARG);
    {
        std::vector<const void *> bad(S.p.begin(), S.p.end());
        bad[0] = static_cast<const char *>(bad[0]) + 8;  // misaligned
        REQUIRE(reshard_execute(plan, bad.data(), D.p.data(), nullptr) == RESHARD_ERR_INVALID_ARG);
        bad[0] = D.p[0];                                  // a source that is also a destination
        REQUIRE(reshard_execute(plan, bad.data(), D.p.data(), nullptr) == RESHARD_ERR_INVALID_ARG);
    }

    // one-shot flow
    std::vector<const void *> sp(S.p.begin(), S.p.end());
    REQUIRE(reshard_execute(plan, sp.data(), D.p.data(), nullptr) == RESHARD_OK);
    REQUIRE(reshard_mem_stats(plan, &st) == RESHARD_OK && st.src_live == sbytes && st.dst_live == dbytes && st.state == RESHARD_SRC_RESIDENT);
    fake_hip_host_limit = 1000;  // pinned memory refused: nothing changes, nothing leaks
    REQUIRE(reshard_swap_out(plan, nullptr) == RESHARD_ERR_HOST_OOM);
    REQUIRE(reshard_reserve_host(plan) == RESHARD_ERR_HOST_OOM && fake_hip_host_bytes == 0);
    fake_hip_host_limit = sbytes - 1;  // refused half way: the blocks already taken go back
    REQUIRE(reshard_swap_out(plan, nullptr) == RESHARD_ERR_HOST_OOM && fake_hip_host_bytes == 0);
    fake_hip_host_limit = -1;
    REQUIRE(reshard_swap_out(plan, nullptr) == RESHARD_OK && fake_hip_host_bytes == sbytes);
    REQUIRE(reshard_execute_noalloc(plan, sp.data(), D2.p.data(), nullptr) == RESHARD_OK);  // allowed while swapping out
    REQUIRE(D.same(D2));
    REQUIRE(reshard_mark_src_released(plan) == RESHARD_ERR_BAD_STATE);  // copies not waited for
    REQUIRE(reshard_swap_wait(plan) == RESHARD_OK);
    REQUIRE(reshard_swap_out(plan, nullptr) == RESHARD_ERR_BAD_STATE);
    REQUIRE(reshard_release_host(plan) == RESHARD_ERR_BAD_STATE);      // the only copy
    REQUIRE(reshard_mark_src_released(plan) == RESHARD_OK);
    REQUIRE(reshard_mem_stats(plan, &st) == RESHARD_OK && st.src_live == 0 && st.released == sbytes && st.peak_device == sbytes + dbytes);
    REQUIRE(reshard_swap_in(plan, nullptr) == RESHARD_ERR_BAD_STATE);  // no device home
    REQUIRE(reshard_execute(plan, sp.data(), D2.p.data(), nullptr) == RESHARD_ERR_BAD_STATE);
    for (size_t i = 0; i < S.p.size(); ++i)
        if (S.p[i]) std::memset(S.p[i], 0, size_t(S.n[i]));            // "freed and allocated again"
    REQUIRE(reshard_bind_src(plan, sp.data()) == RESHARD_OK);
    REQUIRE(reshard_swap_in(plan, nullptr) == RESHARD_OK);
    REQUIRE(reshard_bind_src(plan, sp.data()) == RESHARD_ERR_BAD_STATE);  // copies in flight
    REQUIRE(reshard_swap_wait_buffer(plan, 0, nullptr, 1) == RESHARD_OK);
    REQUIRE(reshard_swap_wait(plan) == RESHARD_OK);
    REQUIRE(S.same(keep));
    REQUIRE(reshard_mem_stats(plan, &st) == RESHARD_OK && st.state == RESHARD_SRC_RESIDENT && st.src_live == sbytes);

    // streaming flow on the second plan, buffers in reverse order, then back one buffer at a time
    Buffers D3;
    D3.make(stream_plan, 1, 0xA5);
    for (int i = ns - 1; i >= 0; --i) {
        if (!reshard_plan_buf_used(stream_plan, 0, i)) continue;
        REQUIRE(reshard_execute_source(stream_plan, i, S.p[size_t(i)], D3.p.data(), nullptr) == RESHARD_OK);
        REQUIRE(reshard_swap_out_source(stream_plan, i, nullptr) == RESHARD_OK);
        REQUIRE(reshard_execute_source(stream_plan, i, S.p[size_t(i)], D3.p.data(), nullptr) == RESHARD_ERR_BAD_STATE);
        REQUIRE(reshard_mark_src_buffer_released(stream_plan, i) == RESHARD_ERR_BAD_STATE);
        REQUIRE(reshard_swap_wait_buffer(stream_plan, i, nullptr, 1) == RESHARD_OK);
        REQUIRE(reshard_mark_src_buffer_released(stream_plan, i) == RESHARD_OK);
        REQUIRE(reshard_mem_stats(stream_plan, &st) == RESHARD_OK && st.src_live == 0);
    }
    REQUIRE(D3.same(D));
    REQUIRE(reshard_mem_stats(stream_plan, &st) == RESHARD_OK && st.state == RESHARD_SRC_RELEASED && st.released == sbytes);
    int64_t largest = 0;
    for (int i = 0; i < ns; ++i) largest = std::max<int64_t>(largest, reshard_plan_buf_used(stream_plan, 0, i) ? S.n[size_t(i)] : 0);
    REQUIRE(st.peak_device == dbytes + largest);
    Buffers back;
    back.make(stream_plan, 0, 0);
    for (int i = 0; i < ns; ++i) {
        if (!reshard_plan_buf_used(stream_plan, 0, i)) continue;
        REQUIRE(reshard_swap_in_source(stream_plan, i, nullptr, nullptr) == RESHARD_ERR_BAD_STATE);  // released: needs a home
        REQUIRE(reshard_swap_in_source(stream_plan, i, back.p[size_t(i)], nullptr) == RESHARD_OK);
        REQUIRE(reshard_src_buffer_state(stream_plan, i) == RESHARD_SRC_SWAPPING_IN);
    }
    REQUIRE(reshard_swap_wait(stream_plan) == RESHARD_OK);
    REQUIRE(back.same(keep));
    REQUIRE(reshard_mem_stats(stream_plan, &st) == RESHARD_OK && st.state == RESHARD_SRC_RESIDENT);

    // destroy with a swap-out pending and pinned memory held: everything must be given back
    REQUIRE(reshard_swap_out(stream_plan, nullptr) == RESHARD_OK);
    REQUIRE(reshard_plan_destroy(stream_plan) == RESHARD_OK);
    REQUIRE(reshard_release_host(plan) == RESHARD_OK);
    REQUIRE(reshard_plan_destroy(plan) == RESHARD_OK);
    REQUIRE(fake_hip_host_bytes == 0);
    return 0;
}

// Random sequences of calls against a model of the residency rules written from reshard.h: every
// return code, every buffer state and the ledger must match the model after every call.
static int random_calls(unsigned seed, int steps) {
    const reshard_model_spec spec = moe_spec(2);
    const reshard_layout src = lay(RESHARD_TRAIN, 2, 1, 2, 0), dst = lay(RESHARD_GEN, 1, 1, 1, 0);
    reshard_plan *plan = nullptr;
    REQUIRE(reshard_plan_create(&spec, &src, &dst, &plan) == RESHARD_OK);
    const int ns = reshard_plan_num_bufs(plan, 0);
    Buffers A, B, D;  // two device homes per source buffer, one destination set
    A.make(plan, 0, -1);
    B.make(plan, 0, 0);
    D.make(plan, 1, 0xA5);
    enum { UNB = RESHARD_SRC_UNBOUND, RES = RESHARD_SRC_RESIDENT, OUT = RESHARD_SRC_SWAPPING_OUT, HOST = RESHARD_SRC_ON_HOST,
           REL = RESHARD_SRC_RELEASED, IN = RESHARD_SRC_SWAPPING_IN, MIX = RESHARD_SRC_MIXED };
    std::vector<int> st(size_t(ns), UNB);
    std::vector<const void *> ptr(size_t(ns), nullptr);
    bool swapped_once = false;
    unsigned r = seed * 2654435761u + 12345u;
    auto rnd = [&](unsigned n) { r = r * 1664525u + 1013904223u; return (r >> 8) % n; };
    auto plan_state = [&] {
        int c = st[0];
        for (int s_ : st) if (s_ != c) return int(MIX);
        return c;
    };
    auto all = [&](int from, int to) { for (int &s_ : st) if (s_ == from) s_ = to; };
    for (int step = 0; step < steps; ++step) {
        const int op = int(rnd(13)), i = int(rnd(unsigned(ns)));
        const Buffers &home = rnd(2) ? A : B;
        std::vector<const void *> sp(home.p.begin(), home.p.end());
        const int ps = plan_state();
        int want = RESHARD_OK, got = RESHARD_OK;
        switch (op) {
            case 0: {  // execute
                bool same = true;
                for (int k = 0; k < ns; ++k) same = same && ptr[size_t(k)] == sp[size_t(k)];
                if (!(ps == UNB || ps == RES || (ps == OUT && same))) want = RESHARD_ERR_BAD_STATE;
                got = reshard_execute(plan, sp.data(), D.p.data(), nullptr);
                if (want == RESHARD_OK) {
                    ptr = sp;
                    if (ps != OUT) all(ps, RES);
                }
                break;
            }
            case 1:  // execute_source
                if (st[size_t(i)] != UNB && st[size_t(i)] != RES) want = RESHARD_ERR_BAD_STATE;
                got = reshard_execute_source(plan, i, sp[size_t(i)], D.p.data(), nullptr);
                if (want == RESHARD_OK) { ptr[size_t(i)] = sp[size_t(i)]; st[size_t(i)] = RES; }
                break;
            case 2:
                if (ps != RES) want = RESHARD_ERR_BAD_STATE;
                got = reshard_swap_out(plan, nullptr);
                if (want == RESHARD_OK) { all(RES, OUT); swapped_once = true; }
                break;
            case 3:
                if (st[size_t(i)] != RES) want = RESHARD_ERR_BAD_STATE;
                got = reshard_swap_out_source(plan, i, nullptr);
                if (want == RESHARD_OK) { st[size_t(i)] = OUT; swapped_once = true; }
                break;
            case 4:
                got = reshard_swap_wait(plan);
                all(OUT, HOST);
                all(IN, RES);
                break;
            case 5:
                if (!swapped_once) want = RESHARD_ERR_BAD_STATE;
                got = reshard_swap_wait_buffer(plan, i, nullptr, 1);
                if (want == RESHARD_OK) st[size_t(i)] = st[size_t(i)] == OUT ? int(HOST) : st[size_t(i)] == IN ? int(RES) : st[size_t(i)];
                break;
            case 6:
                if (ps != HOST) want = RESHARD_ERR_BAD_STATE;
                got = reshard_mark_src_released(plan);
                if (want == RESHARD_OK) { all(HOST, REL); std::fill(ptr.begin(), ptr.end(), nullptr); }
                break;
            case 7:
                if (st[size_t(i)] != HOST) want = RESHARD_ERR_BAD_STATE;
                got = reshard_mark_src_buffer_released(plan, i);
                if (want == RESHARD_OK) { st[size_t(i)] = REL; ptr[size_t(i)] = nullptr; }
                break;
            case 8:
                if (!(ps == UNB || ps == RES || ps == HOST || ps == REL)) want = RESHARD_ERR_BAD_STATE;
                got = reshard_bind_src(plan, sp.data());
                if (want == RESHARD_OK) { ptr = sp; all(UNB, RES); all(REL, HOST); }
                break;
            case 9:
                if (ps != HOST) want = RESHARD_ERR_BAD_STATE;
                got = reshard_swap_in(plan, nullptr);
                if (want == RESHARD_OK) { all(HOST, IN); swapped_once = true; }
                break;
            case 10: {
                const bool give = rnd(2) != 0;
                void *to = give ? const_cast<void *>(sp[size_t(i)]) : nullptr;
                if ((st[size_t(i)] != HOST && st[size_t(i)] != REL) || (!give && !ptr[size_t(i)])) want = RESHARD_ERR_BAD_STATE;
                got = reshard_swap_in_source(plan, i, to, nullptr);
                if (want == RESHARD_OK) { if (give) ptr[size_t(i)] = to; st[size_t(i)] = IN; swapped_once = true; }
                break;
            }
            case 11:
                if (ps != UNB && ps != RES) want = RESHARD_ERR_BAD_STATE;
                got = reshard_release_host(plan);
                break;
            default:
                got = reshard_reserve_host(plan);
                break;
        }
        if (got != want) { std::printf("seed %u step %d op %d buffer %d: returned %d, model says %d (%s)\n", seed, step, op, i, got, want, reshard_last_error()); return 1; }
        reshard_mem_stats_t ms;
        REQUIRE(reshard_mem_stats(plan, &ms) == RESHARD_OK);
        int64_t live = 0, released = 0;
        for (int k = 0; k < ns; ++k) {
            if (reshard_src_buffer_state(plan, k) != st[size_t(k)]) { std::printf("seed %u step %d op %d: buffer %d is %d, model says %d\n", seed, step, op, k, reshard_src_buffer_state(plan, k), st[size_t(k)]); return 1; }
            const bool is_live = st[size_t(k)] == RES || st[size_t(k)] == OUT || st[size_t(k)] == HOST || st[size_t(k)] == IN;
            if (is_live && ptr[size_t(k)]) live += A.n[size_t(k)];
            if (st[size_t(k)] == REL) released += A.n[size_t(k)];
        }
        if (ms.state != plan_state() || ms.src_live != live || ms.released != released) {
            std::printf("seed %u step %d op %d: ledger state %d live %lld released %lld, model %d %lld %lld\n", seed, step, op, ms.state,
                        (long long)ms.src_live, (long long)ms.released, plan_state(), (long long)live, (long long)released);
            return 1;
        }
    }
    REQUIRE(reshard_plan_destroy(plan) == RESHARD_OK);
    REQUIRE(fake_hip_host_bytes == 0);
    return 0;
}

int main() {
    int bad = 0;
    for (int eb : {1, 2, 4, 8}) bad += flows(eb);
    for (unsigned seed = 1; seed <= 40 && !bad; ++seed) bad += random_calls(seed, 400);
    // NULL plans and bad indices on every entry point that takes them
    bad += reshard_plan_destroy(nullptr) != RESHARD_OK;
    bad += reshard_execute(nullptr, nullptr, nullptr, nullptr) != RESHARD_ERR_INVALID_ARG;
    bad += reshard_swap_out(nullptr, nullptr) != RESHARD_ERR_INVALID_ARG;
    bad += reshard_mem_stats(nullptr, nullptr) != RESHARD_ERR_INVALID_ARG;
    bad += reshard_host_copy(nullptr, 0) != nullptr;
    std::printf(bad ? "FAILED %d\n" : "ok\n", bad);
    return bad ? 1 : 0;
}
