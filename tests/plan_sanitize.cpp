// Host-only driver for the plan builder, built by tests/test_plan_sanitizers.py with
// AddressSanitizer and UndefinedBehaviorSanitizer (g++, no GPU code involved).  It builds the
// fragment lists, descriptors and tiles of a set of shapes, valid and invalid, and checks a few
// invariants; the sanitizers abort on any out-of-bounds access, overflow or leak.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "internal.h"

using namespace reshard;

static reshard_model_spec spec(int family, int L, int H, int nq, int nkv, int d, int I, int V, int bias, int emb,
                               int E, int Ie, int shared, int eb, int tied = 0) {
    reshard_model_spec s{};
    s.struct_size = sizeof s;
    s.family = family; s.L = L; s.H = H; s.nq = nq; s.nkv = nkv; s.d = d; s.I = I; s.V = V;
    s.qkv_bias = bias; s.has_embeddings = emb; s.E = E; s.Ie = Ie; s.n_shared = shared; s.elem_bytes = eb;
    s.tied_embeddings = tied;
    return s;
}
static reshard_layout lay(int kind, int tp, int pp, int ep, int grouped = 0, int tf = -1, int ef = -1, int vpp = 1,
                          int first = 0, int last = 0, int vpad = 0, int etp = 1) {
    reshard_layout l{};
    l.struct_size = sizeof l;
    l.kind = kind; l.tp = tp; l.pp = pp; l.ep = ep; l.expert_layout = grouped;
    l.tp_rank_filter = tf; l.ep_rank_filter = ef; l.vpp = vpp; l.first_stage_layers = first; l.last_stage_layers = last; l.vocab_padded = vpad; l.etp = etp;
    return l;
}

// expect: 1 must succeed, 0 must be refused, -1 either (only the sanitizers and the invariants judge)
static int run(const reshard_model_spec &s, const reshard_layout &a, const reshard_layout &b, const Tuning &tn,
               int expect) {
    Side S, D;
    std::vector<reshard_desc> descs;
    int rc = build_side(s, a, true, S);
    if (!rc) rc = build_side(s, b, false, D);
    if (!rc) rc = compile_descriptors(s, S, D, descs);
    int fr = tn.transpose_rows, fc = tn.transpose_cols;
    if (!transpose_shape_ok(s.elem_bytes, fr, fc)) transpose_default_shape(s.elem_bytes, fr, fc);
    std::vector<TileClass> classes;
    if (!rc) rc = cut_tiles(descs, int(S.buf_bytes.size()), tn, fr, fc, classes);
    if (expect >= 0 && (rc == 0) != (expect == 1)) {
        std::printf("unexpected result %d (expected %s)\n", rc, expect ? "ok" : "an error");
        return 1;
    }
    if (rc) return 0;
    // bytes of the tiles equal bytes of the descriptors; every access stays inside its buffer
    long long dbytes = 0, tbytes = 0, again_blocks = 0, again_gathered = 0;
    for (const reshard_desc &d : descs) dbytes += d.rows * d.row_bytes;
    auto check = [&](const TileClass &c) {
        const std::vector<Tile> &v = c.tiles;
        for (size_t i = 0; i < v.size(); ++i) {
            const Tile &t = v[i];
            const long long unit = 1ll << t.vec_log2;
            const long long sb = S.buf_bytes[t.src_buf], db = D.buf_bytes[t.dst_buf - S.buf_bytes.size()];
            if (t.kind == 2) {
                // gathered tiles (behind the row blocks and runs of the copy class): the same bytes as the row
                // blocks they stand for, every unit inside the buffer of the source it comes from
                const uint32_t c0 = t.src_stride & 0xFFFFu, j0 = (t.src_stride >> 16) & 0xFFu, lk = t.src_stride >> 24;
                const bool placed = c.kind == 0 && i >= size_t(c.num_blocks) + c.num_runs && unit == 16 && t.row_units >= 64 &&
                                    c0 < t.row_units && j0 < (1u << lk) && t.src_buf + (1u << lk) <= S.buf_bytes.size();
                if (!placed) { std::printf("a gathered tile of a wrong form or place\n"); std::exit(1); }
                again_gathered += (long long)t.rows * 16;
                for (uint32_t u = 0; u < t.rows; ++u) {
                    const unsigned long long w = (unsigned long long)j0 * t.row_units + c0 + u, seg = w / t.row_units;
                    const long long at = (long long)t.src_off + (long long)(seg >> lk) * t.dst_stride * 16 + (long long)(w % t.row_units) * 16;
                    if (at + 16 > S.buf_bytes[t.src_buf + (seg & ((1u << lk) - 1))]) { std::printf("tile leaves its buffer\n"); std::exit(1); }
                }
                if ((long long)t.dst_off + (long long)t.rows * 16 > db) { std::printf("tile leaves its buffer\n"); std::exit(1); }
                continue;
            }
            tbytes += (long long)t.rows * t.row_units * unit;
            if (c.kind == 0 && i >= size_t(c.num_blocks - c.num_regathered) && i < c.num_blocks) again_blocks += (long long)t.rows * t.row_units * unit;
            long long s_end, d_end;
            if (t.kind == 0) {
                s_end = (long long)t.src_off + (long long)(t.rows - 1) * t.src_stride + t.row_units * unit;
                d_end = (long long)t.dst_off + (long long)(t.rows - 1) * t.dst_stride + t.row_units * unit;
            } else {
                s_end = (long long)t.src_off + (long long)(t.rows - 1) * t.src_stride + t.row_units * unit;
                d_end = (long long)t.dst_off + (long long)(t.row_units - 1) * t.dst_stride + t.rows * unit;
            }
            if (s_end > sb || d_end > db) { std::printf("tile leaves its buffer\n"); std::exit(1); }
        }
    };
    for (const TileClass &c : classes) {
        check(c);
        // register-path tiles are whole tiles of their class's shape, in a shape the kernel is built for
        if (c.kind == 1)
            for (const Tile &t : c.tiles)
                if (int(t.rows) != c.rows || int(t.row_units) != c.cols || !transpose_shape_ok(s.elem_bytes, c.rows, c.cols)) {
                    std::printf("register-path tile of a wrong shape\n");
                    return 1;
                }
    }
    if (again_blocks != again_gathered) { std::printf("gathered bytes %lld != bytes of the row blocks they stand for %lld\n", again_gathered, again_blocks); return 1; }
    if (dbytes != tbytes) { std::printf("tile bytes %lld != descriptor bytes %lld\n", tbytes, dbytes); return 1; }
    return 0;
}

// Cases from a file, one per line: expect, then the 20 spec fields after struct_size in header order,
// then the 12 fields of the source layout and of the destination layout after struct_size.
static int run_file(const char *path, const Tuning &tn) {
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
        bad += run(s, l[0], l[1], tn, v[0]);
        ++n;
    }
    std::fclose(f);
    std::printf("%d cases from file\n", n);
    return bad;
}
static_assert(sizeof(reshard_model_spec) == 21 * 4 && sizeof(reshard_layout) == 13 * 4, "field counts used by run_file");

int main(int argc, char **argv) {
    Tuning def;
    Tuning small; small.tile_bytes = 4096; small.transpose_rows = 64; small.transpose_cols = 128;
    int bad = 0;
    if (argc > 1) {
        bad = run_file(argv[1], def) + run_file(argv[1], small);
        std::printf(bad ? "FAILED %d\n" : "ok\n", bad);
        return bad ? 1 : 0;
    }
    const int TR = RESHARD_TRAIN, GEN = RESHARD_GEN;
    for (const Tuning &tn : {def, small}) {
        // the task's shapes
        bad += run(spec(0, 2, 256, 4, 2, 64, 688, 1024, 0, 1, 0, 0, 0, 2), lay(TR, 2, 1, 1), lay(GEN, 1, 1, 1), tn, 1);
        bad += run(spec(0, 28, 3584, 28, 4, 128, 18944, 152064, 1, 1, 0, 0, 0, 2), lay(TR, 4, 2, 1), lay(GEN, 2, 1, 1), tn, 1);
        bad += run(spec(0, 64, 5120, 40, 8, 128, 27648, 152064, 1, 1, 0, 0, 0, 2), lay(TR, 8, 4, 1), lay(GEN, 4, 1, 1), tn, 1);
        bad += run(spec(1, 48, 2048, 32, 4, 128, 0, 151936, 0, 1, 128, 768, 0, 2), lay(TR, 1, 2, 8, 1), lay(GEN, 2, 1, 4), tn, 1);
        // ragged and odd shapes, every element size, filters, the way back, the layout options
        for (int eb : {1, 2, 4, 8}) {
            bad += run(spec(0, 4, 48, 8, 4, 8, 40, 64, 1, 1, 0, 0, 0, eb), lay(TR, 4, 2, 1), lay(GEN, 2, 1, 1), tn, 1);
            bad += run(spec(1, 2, 320, 4, 2, 16, 0, 64, 0, 1, 4, 200, 1, eb), lay(TR, 1, 1, 2, 1), lay(GEN, 2, 1, 1), tn, 1);
            bad += run(spec(1, 2, 320, 4, 2, 16, 0, 64, 0, 1, 4, 200, 1, eb), lay(GEN, 2, 1, 1), lay(TR, 1, 1, 2, 1), tn, 1);
            bad += run(spec(0, 8, 48, 8, 2, 8, 40, 64, 1, 1, 0, 0, 0, eb, 1), lay(TR, 4, 2, 1, 0, -1, -1, 2), lay(GEN, 8, 1, 1), tn, 1);
            bad += run(spec(0, 8, 32, 8, 2, 8, 24, 48, 0, 1, 0, 0, 0, eb), lay(TR, 4, 4, 1, 0, -1, -1, 1, 3, 1), lay(GEN, 2, 1, 1, 0, 1), tn, 1);
            bad += run(spec(0, 2, 7, 3, 3, 5, 9, 6, 1, 1, 0, 0, 0, 1), lay(TR, 3, 1, 1), lay(GEN, 1, 1, 1), tn, 1);
            bad += run(spec(1, 2, 32, 4, 4, 8, 0, 48, 0, 1, 4, 24, 1, eb), lay(TR, 4, 1, 2, 1, -1, -1, 1, 0, 0, 0, 4),
                       lay(GEN, 2, 1, 1, 0, 1, -1, 1, 0, 0, 0, 2), tn, 1);
            bad += run(spec(0, 2, 24, 4, 4, 8, 24, 50, 0, 1, 0, 0, 0, eb), lay(TR, 4, 2, 1, 0, -1, -1, 1, 0, 0, 64),
                       lay(GEN, 2, 1, 1, 0, -1, -1, 1, 0, 0, 54), tn, 1);
        }
        // invalid requests must be refused, not crash
        // rows just under the 4 GiB pitch limit (64-bit offsets in every tile), and just over it
        bad += run(spec(0, 1, 8, 2, 2, 8, (1 << 29) - 8, 8, 0, 1, 0, 0, 0, 8), lay(TR, 2, 1, 1), lay(GEN, 1, 1, 1), tn, 1);
        bad += run(spec(0, 1, 8, 2, 2, 8, 1 << 29, 8, 0, 1, 0, 0, 0, 8), lay(TR, 2, 1, 1), lay(GEN, 1, 1, 1), tn, 0);
        bad += run(spec(0, 2, 256, 4, 2, 64, 688, 1024, 0, 1, 0, 0, 0, 2), lay(TR, 3, 1, 1), lay(GEN, 1, 1, 1), tn, 0);
        bad += run(spec(0, 2, 256, 4, 2, 64, 688, 1024, 0, 1, 0, 0, 0, 3), lay(TR, 2, 1, 1), lay(GEN, 1, 1, 1), tn, 0);
        bad += run(spec(0, 2, 256, 4, 2, 64, 688, 1024, 0, 1, 0, 0, 0, 2), lay(TR, 2, 1, 1), lay(GEN, 1, 2, 1), tn, 0);
        bad += run(spec(1, 4, 64, 4, 4, 8, 0, 64, 0, 1, 512, 8, 0, 2), lay(TR, 1, 1, 512), lay(GEN, 1, 1, 1), tn, 1);
        bad += run(spec(0, 2, 256, 4, 2, 64, 688, 1024, 0, 1, 0, 0, 0, 2), lay(TR, 2, 1, 1, 0, 0), lay(GEN, 1, 1, 1), tn, 0);
        bad += run(spec(0, 2, 256, 4, 2, 64, 688, 1024, 0, 1, 0, 0, 0, 2), lay(TR, 2, 1, 1, 0, -1, -1, 1, 0, 0, 1000), lay(GEN, 1, 1, 1), tn, 0);
        bad += run(spec(1, 2, 32, 4, 4, 8, 0, 48, 0, 1, 4, 24, 1, 2), lay(TR, 4, 1, 2, 1, -1, -1, 1, 0, 0, 0, 2), lay(GEN, 2, 1, 1), tn, 0);
        bad += run(spec(0, 2, 256, 4, 2, 64, 688, 1024, 0, 1, 0, 0, 0, 2), lay(TR, 2, 1, 1, 0, -1, -1, 1, 0, 0, 1025), lay(GEN, 1, 1, 1), tn, 0);
    }
    std::printf(bad ? "FAILED %d\n" : "ok\n", bad);
    return bad ? 1 : 0;
}
