// Host-only driver: the REAL kernels of repack.hip, compiled for the host against
// tests/host_simt (one host thread per lane, real barriers) and run under AddressSanitizer, on
// small workloads that reach every kernel, tile class, element size and launch shape.  Each
// result is compared with an interpretation of the plan's descriptor table.  Built and run by
// tests/test_plan_sanitizers.py; test infrastructure only.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <memory>
#include <vector>

#include "internal.h"

long fake_hip_host_limit = -1, fake_hip_host_bytes = 0, fake_hip_copies = 0;
thread_local uint3_ threadIdx;
uint3_ blockIdx, blockDim, gridDim;
namespace host_simt {
long launches = 0, blocks_run = 0;
Pool &pool(uint32_t lanes) {
    static std::map<uint32_t, std::unique_ptr<Pool>> pools;  // one pool per workgroup size in use
    std::unique_ptr<Pool> &p = pools[lanes];
    if (!p) p.reset(new Pool(lanes));
    return *p;
}
pthread_barrier_t *current_sync = nullptr;
}  // namespace host_simt

#define REQUIRE(cond) do { if (!(cond)) { std::printf("line %d: %s is false (last error: %s)\n", __LINE__, #cond, reshard_last_error()); return 1; } } while (0)

static reshard_layout lay(int kind, int tp, int pp, int ep, int grouped, int etp = 1) {
    reshard_layout l{};
    l.struct_size = sizeof l;
    l.kind = kind; l.tp = tp; l.pp = pp; l.ep = ep; l.expert_layout = grouped; l.tp_rank_filter = l.ep_rank_filter = -1; l.etp = etp;
    return l;
}

static int run(const reshard_model_spec &spec, const reshard_layout &src, const reshard_layout &dst, const reshard_tuning *tn,
               bool by_source) {
    reshard_plan *plan = nullptr;
    REQUIRE(reshard_plan_create_tuned(&spec, &src, &dst, tn, &plan) == RESHARD_OK);
    const int ns = reshard_plan_num_bufs(plan, 0), nd = reshard_plan_num_bufs(plan, 1);
    std::vector<void *> S(size_t(ns), nullptr), D(size_t(nd), nullptr), W(size_t(nd), nullptr);
    for (int i = 0; i < ns; ++i) {
        if (!reshard_plan_buf_used(plan, 0, i)) continue;
        const size_t n = size_t(reshard_plan_buf_bytes(plan, 0, i));
        S[size_t(i)] = std::aligned_alloc(256, n);  // exact extent: one byte too far is reported
        unsigned char *c = static_cast<unsigned char *>(S[size_t(i)]);
        for (size_t k = 0; k < n; ++k) c[k] = (unsigned char)((k * 2654435761u + unsigned(i) * 97u) >> 11);
    }
    for (int j = 0; j < nd; ++j) {
        if (!reshard_plan_buf_used(plan, 1, j)) continue;
        const size_t n = size_t(reshard_plan_buf_bytes(plan, 1, j));
        D[size_t(j)] = std::aligned_alloc(256, n);
        W[size_t(j)] = std::aligned_alloc(256, n);
        std::memset(D[size_t(j)], 0xA5, n);
        std::memset(W[size_t(j)], 0xA5, n);
    }
    // what the descriptor table says, byte by byte
    reshard_plan_info info;
    REQUIRE(reshard_plan_get_info(plan, &info) == RESHARD_OK);
    for (int64_t q = 0; q < info.num_descs; ++q) {
        reshard_desc d;
        REQUIRE(reshard_plan_desc(plan, q, &d) == RESHARD_OK);
        const char *s = static_cast<const char *>(S[size_t(d.src_buf)]) + d.src_off;
        char *w = static_cast<char *>(W[size_t(d.dst_buf)]) + d.dst_off;
        if (d.kind == 0) {
            for (int64_t i = 0; i < d.rows; ++i) std::memcpy(w + i * d.dst_stride, s + i * d.src_stride, size_t(d.row_bytes));
        } else {
            const int64_t cols = d.row_bytes / d.elem_bytes;
            for (int64_t i = 0; i < d.rows; ++i)
                for (int64_t k = 0; k < cols; ++k)
                    std::memcpy(w + k * d.dst_stride + i * d.elem_bytes, s + i * d.src_stride + k * d.elem_bytes, size_t(d.elem_bytes));
        }
    }
    // A plan that keeps several copies of its tile table reads another one at every execute: run it through all
    // of them and once round, every execute from sentinel-filled destinations and checked like the first.
    const int executes = (tn && tn->table_copies > 1 && !by_source) ? tn->table_copies + 1 : 1;
    int bad = 0;
    for (int rep = 0; rep < executes && !bad; ++rep) {
        for (int j = 0; j < nd; ++j)
            if (D[size_t(j)]) std::memset(D[size_t(j)], 0xA5, size_t(reshard_plan_buf_bytes(plan, 1, j)));
        if (by_source) {
            for (int i = 0; i < ns; ++i)
                if (S[size_t(i)]) REQUIRE(reshard_execute_source(plan, i, S[size_t(i)], D.data(), nullptr) == RESHARD_OK);
        } else {
            // alternately through the plan's own table and through the static array (which the
            // previous case's table still fills: a new table must replace it)
            static int flip = 0;
            std::vector<const void *> sp(S.begin(), S.end());
            REQUIRE(((executes == 1 && (flip++ & 1)) ? reshard_execute_noalloc : reshard_execute)(plan, sp.data(), D.data(), nullptr) == RESHARD_OK);
        }
        for (int j = 0; j < nd; ++j)
            if (D[size_t(j)] && std::memcmp(D[size_t(j)], W[size_t(j)], size_t(reshard_plan_buf_bytes(plan, 1, j)))) {
                std::printf("destination buffer %d differs from the descriptor table's result (execute %d)\n", j, rep);
                bad = 1;
            }
    }
    REQUIRE(reshard_plan_destroy(plan) == RESHARD_OK);
    for (void *p : S) std::free(p);
    for (void *p : D) std::free(p);
    for (void *p : W) std::free(p);
    return bad;
}

// Cases from a file, one per line, in the format of tests/plan_sanitize.cpp (the leading
// "expect" field is ignored: every case in the file is a valid one).
static int run_file(const char *path, const reshard_tuning *tn) {
    std::FILE *f = std::fopen(path, "r");
    if (!f) { std::printf("cannot open %s\n", path); return 1; }
    int bad = 0, n = 0, v[45];
    for (;;) {
        int got = 0;
        while (got < 45 && std::fscanf(f, "%d", &v[got]) == 1) ++got;
        if (got < 45) break;
        reshard_model_spec s{};
        s.struct_size = sizeof s;
        int32_t *sp = &s.family;
        for (int k = 0; k < 20; ++k) sp[k] = v[1 + k];
        reshard_layout l[2]{};
        for (int side = 0; side < 2; ++side) {
            l[side].struct_size = sizeof(reshard_layout);
            int32_t *lp = &l[side].kind;
            for (int k = 0; k < 12; ++k) lp[k] = v[21 + 12 * side + k];
        }
        bad += run(s, l[0], l[1], tn, n % 3 == 2);
        ++n;
    }
    std::fclose(f);
    std::printf("%d cases from file\n", n);
    return bad;
}
static_assert(sizeof(reshard_model_spec) == 21 * 4 && sizeof(reshard_layout) == 13 * 4, "field counts used by run_file");

int main(int argc, char **argv) {
    int bad = 0;
    if (argc > 1) {
        reshard_tuning tiny{};
        tiny.tile_bytes = 4096; tiny.block_threads = 128; tiny.unroll = 1;
        // 128-lane workgroups are cheap to emulate; "default" as a second argument runs the default launch shape
        // (1024 lanes, woven order) instead
        bad = run_file(argv[1], argc > 2 && !std::strcmp(argv[2], "default") ? nullptr : &tiny);
        std::printf(bad ? "FAILED %d\n" : "ok\n", bad);
        return bad ? 1 : 0;
    }
    // dense: fused QKV, gate/up, row-parallel merges, bias vectors, two pipeline stages
    reshard_model_spec dense{};
    dense.struct_size = sizeof dense;
    dense.family = RESHARD_DENSE_GQA; dense.L = 2; dense.H = 64; dense.nq = 4; dense.nkv = 2; dense.d = 16; dense.I = 88; dense.V = 96;
    dense.has_embeddings = 1; dense.qkv_bias = 1;
    // grouped experts whose matrices hold whole register-path tiles, smaller shapes on the strips and a ragged rest
    reshard_model_spec moe{};
    moe.struct_size = sizeof moe;
    moe.family = RESHARD_MOE_GQA; moe.L = 1; moe.H = 336; moe.nq = 4; moe.nkv = 2; moe.d = 16; moe.V = 32; moe.has_embeddings = 1;
    moe.E = 2; moe.Ie = 208; moe.n_shared = 0;
    reshard_tuning small{}, odd{}, persistent{}, plain_order{}, wide192{}, pooled{}, woven{}, woven_small{};
    small.table_copies = 3;  // three copies of the tile table, read in turn
    woven.flags = 127;                                  // the XCDs share every group of 8 tiles
    woven_small.flags = 100; woven_small.tile_bytes = 4096;  // plain accesses with the barrier, tiles of 256 units
    pooled.tile_bytes = 4096; pooled.flags = 31; pooled.tail_pool_percent = 30; pooled.tail_chunk_tiles = 1;  // 1024-lane workgroups, a shared tail
    wide192.transpose_rows = 192; wide192.transpose_cols = 192;
    small.tile_bytes = 4096; small.block_threads = 64; small.unroll = 1; small.transpose_rows = 64; small.transpose_cols = 64;
    odd.tile_bytes = 8192; odd.block_threads = 256; odd.unroll = 2; odd.flags = 11; odd.transpose_rows = 128; odd.transpose_cols = 64;
    persistent.blocks_per_cu = 2; persistent.block_threads = 128; persistent.tile_bytes = 4096;
    plain_order.flags = 7; plain_order.tile_bytes = 16384; plain_order.unroll = 8;
    for (int eb : {2, 1, 4, 8}) {
        dense.elem_bytes = moe.elem_bytes = eb;
        // every launch shape at 2 bytes; the default and the smallest shapes at the other sizes
        std::vector<const reshard_tuning *> tunings{nullptr, &small, &woven, &woven_small};
        if (eb == 2) tunings.insert(tunings.end(), {&odd, &persistent, &plain_order, &wide192, &pooled});
        for (const reshard_tuning *tn : tunings) {
            bad += run(dense, lay(RESHARD_TRAIN, 2, 2, 1, 0), lay(RESHARD_GEN, 1, 1, 1, 0), tn, false);
            bad += run(moe, lay(RESHARD_TRAIN, 1, 1, 2, 1), lay(RESHARD_GEN, 2, 1, 1, 0), tn, false);   // transposing
            bad += run(moe, lay(RESHARD_GEN, 2, 1, 1, 0), lay(RESHARD_TRAIN, 1, 1, 2, 1), tn, tn == nullptr);  // and back
            if (bad) break;
        }
        if (bad) break;
        std::printf("element size %d done: %ld launches, %ld workgroups so far\n", eb, host_simt::launches, host_simt::blocks_run);
        std::fflush(stdout);
    }
    if (!bad) {
        // a table long enough for the copy kernel's shared tail pool: a zeroing launch and the pooled launch
        reshard_model_spec wide = dense;
        wide.elem_bytes = 2; wide.H = 256; wide.d = 64; wide.I = 688; wide.V = 1024;
        const long before = host_simt::launches;
        for (int twice = 0; twice < 2; ++twice)  // once through the plan's own table (pooled), once through the static array (not)
            bad += run(wide, lay(RESHARD_TRAIN, 2, 1, 1, 0), lay(RESHARD_GEN, 1, 1, 1, 0), &pooled, false);
        if (host_simt::launches - before != 3) { std::printf("the tail pool was not used (%ld launches)\n", host_simt::launches - before); bad += 1; }
    }
    if (!bad) {
        // shards of row-parallel weights with rows of 64 and 88 vectors: the side-by-side merge (and the packing of
        // narrower rows out of a pitched source) also exists as gathered tiles, which the woven order launches
        reshard_model_spec g = dense;
        g.L = 1; g.H = 64; g.nq = 8; g.nkv = 2; g.d = 128; g.I = 1408; g.V = 64; g.qkv_bias = 0;
        reshard_tuning blocks{};
        blocks.flags = 31;  // the same plans through the row blocks
        for (const reshard_tuning *tn : {static_cast<const reshard_tuning *>(nullptr), static_cast<const reshard_tuning *>(&woven_small),
                                         static_cast<const reshard_tuning *>(&blocks)}) {
            g.elem_bytes = 2;
            bad += run(g, lay(RESHARD_TRAIN, 2, 1, 1, 0), lay(RESHARD_GEN, 1, 1, 1, 0), tn, false);  // two sources per row
            bad += run(g, lay(RESHARD_TRAIN, 1, 1, 1, 0), lay(RESHARD_GEN, 2, 1, 1, 0), tn, false);  // one pitched source
            g.elem_bytes = 4;
            bad += run(g, lay(RESHARD_TRAIN, 4, 1, 1, 0), lay(RESHARD_GEN, 1, 1, 1, 0), tn, tn == nullptr);  // four
        }
        {   // the plans above do hold gathered tiles
            reshard_plan *plan = nullptr;
            const reshard_layout a = lay(RESHARD_TRAIN, 4, 1, 1, 0), b = lay(RESHARD_GEN, 1, 1, 1, 0);
            reshard_plan_info info{};
            int64_t gathered = 0;
            if (reshard_plan_create(&g, &a, &b, &plan) != RESHARD_OK || reshard_plan_get_info(plan, &info) != RESHARD_OK) bad += 1;
            for (int64_t q = 0; !bad && q < info.num_tiles; ++q) {
                reshard_tile t;
                if (reshard_plan_tile(plan, q, &t) != RESHARD_OK) { bad += 1; break; }
                gathered += t.kind == 2 && t.sources == 4 && t.order == 2;
            }
            if (!gathered) { std::printf("no gathered tiles in the plan meant to have them\n"); bad += 1; }
            reshard_plan_destroy(plan);
        }
        std::printf("gathered tiles done: %ld launches so far\n", host_simt::launches);
    }
    std::printf(bad ? "FAILED %d\n" : "ok\n", bad);
    return bad ? 1 : 0;
}
