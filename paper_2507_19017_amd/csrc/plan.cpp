// Host-side plan builder: compiles (model shape, source layout, destination
// layout) into a flat table of copy descriptors and equal-work tiles.
//
// This is the selection half of step 2 of the allgather-swap technique (paper
// section "Allgather-Swap Technique": each device selects and copies the weight
// slices it needs for generation), done once per layout pair instead of per
// iteration.  Formulation: each layout is described as a list of FRAGMENTS
// (rectangles of logical tensors with a storage address); the mapping is the set
// of pairwise intersections of source and destination fragments of the same
// logical tensor.  Nothing here depends on which two layout kinds are paired.
#include <algorithm>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>

#include "internal.h"

namespace reshard {

namespace {

thread_local std::string g_error;

constexpr int64_t kAlign = 256;

uint64_t make_key(int id, int layer, int expert) {
    return (uint64_t(id) << 48) | (uint64_t(uint32_t(layer + 1) & 0xFFFFFF) << 24) |
           uint64_t(uint32_t(expert + 1) & 0xFFFFFF);
}

bool is_replicated(int id) {
    switch (id) {
        case LT_LN1: case LT_LN2: case LT_FINAL_LN: case LT_ROUTER:
        case LT_QA: case LT_QA_LN: case LT_KVA: case LT_KVA_LN:
            return true;
        default:
            return false;
    }
}

// Lays stored tensors out in one buffer and records the fragments they hold.
class BufferBuilder {
  public:
    // A destination records every copy of a tensor.  A source records only the copy that is
    // read: common tensors on tensor rank 0 (`rank0`), other replicas where marked primary.
    BufferBuilder(Side &side, int buf, int eb, bool record_frags, bool is_source, bool rank0,
                  bool expert_buffer = false)
        : side_(side), buf_(buf), eb_(eb), frags_(record_frags), src_(is_source), rank0_(rank0),
          expert_buffer_(expert_buffer) {}

    // Starts a stored tensor of `elems` elements; returns its byte offset.
    int64_t begin(const char *name, int layer, int expert, int64_t elems, bool replicated) {
        off_ = (off_ + kAlign - 1) / kAlign * kAlign;
        reshard_tensor_info ti{};
        std::snprintf(ti.name, sizeof ti.name, "%s", name);
        ti.layer = layer;
        ti.expert = expert;
        ti.buffer = buf_;
        ti.replicated = replicated ? 1 : 0;
        ti.weight_class = expert_buffer_ ? RESHARD_CLASS_EP : replicated ? RESHARD_CLASS_COMMON : RESHARD_CLASS_TP;
        ti.offset = off_;
        ti.bytes = elems * eb_;
        side_.tensors.push_back(ti);
        int64_t at = off_;
        off_ += elems * eb_;
        return at;
    }

    // Rows [r0,r1) x cols [c0,c1) of logical tensor `id` stored row-major (ld elements
    // per row) at byte offset `off`; transposed = stored column-major with that ld.
    // `primary` = false marks a copy that a source never reads (another rank or stage holds
    // the copy that is read); destinations record every copy.
    void frag(int id, int layer, int expert, int64_t r0, int64_t r1, int64_t c0, int64_t c1,
              int64_t off, int64_t ld, bool transposed = false, bool primary = true) {
        if (!frags_) return;
        if (src_ && (!primary || (is_replicated(id) && !rank0_))) return;
        side_.frags.push_back(Fragment{make_key(id, layer, expert), r0, r1, c0, c1, buf_, off, ld, transposed});
    }

    // A vocabulary shard: `rows` stored rows of which only those below `vocab` are logical.
    void vocab_shard(const char *name, int id, int64_t r0, int64_t rows, int64_t vocab, int64_t cols,
                     bool primary = true) {
        int64_t at = begin(name, -1, -1, rows * cols, !primary);
        side_.tensors.back().weight_class = RESHARD_CLASS_TP;
        const int64_t r1 = std::min(r0 + rows, vocab);
        if (r1 > r0) frag(id, -1, -1, r0, r1, 0, cols, at, cols, false, primary);
    }

    // A whole stored tensor that is one fragment.
    void whole(const char *name, int id, int layer, int64_t r0, int64_t rows, int64_t c0,
               int64_t cols, bool primary = true) {
        int64_t at = begin(name, layer, -1, rows * cols, is_replicated(id) || !primary);
        if (!is_replicated(id)) side_.tensors.back().weight_class = RESHARD_CLASS_TP;  // a never-read copy of a shard
        frag(id, layer, -1, r0, r0 + rows, c0, c0 + cols, at, cols, false, primary);
    }

    int64_t finish() const { return (off_ + kAlign - 1) / kAlign * kAlign; }

  private:
    Side &side_;
    int buf_, eb_;
    bool frags_, src_, rank0_, expert_buffer_;
    int64_t off_ = 0;
};

int check_shape(const reshard_model_spec &s, const reshard_layout &l) {
    auto bad = [](const char *what) { return fail(RESHARD_ERR_UNSUPPORTED, what); };
    if (s.family < RESHARD_DENSE_GQA || s.family > RESHARD_MOE_MLA)
        return fail(RESHARD_ERR_INVALID_ARG, "unknown model family");
    if (l.kind != RESHARD_TRAIN && l.kind != RESHARD_GEN)
        return fail(RESHARD_ERR_INVALID_ARG, "unknown layout kind");
    if (l.expert_layout != RESHARD_PER_EXPERT && l.expert_layout != RESHARD_GROUPED)
        return fail(RESHARD_ERR_INVALID_ARG, "unknown expert layout");
    if (s.L <= 0 || s.H <= 0 || s.nq <= 0) return fail(RESHARD_ERR_INVALID_ARG, "L, H, nq must be positive");
    if (s.elem_bytes != 1 && s.elem_bytes != 2 && s.elem_bytes != 4 && s.elem_bytes != 8)
        return fail(RESHARD_ERR_INVALID_ARG, "elem_bytes must be 1, 2, 4 or 8");
    if (l.tp < 1 || l.pp < 1 || l.ep < 1) return fail(RESHARD_ERR_INVALID_ARG, "degrees must be >= 1");
    if (l.kind == RESHARD_GEN && l.pp != 1) return bad("a generation layout has one pipeline stage");
    if (l.vpp < 0 || l.first_stage_layers < 0 || l.last_stage_layers < 0)
        return fail(RESHARD_ERR_INVALID_ARG, "vpp and stage layer counts must be >= 0");
    const int vpp = l.vpp > 0 ? l.vpp : 1;
    if (l.first_stage_layers || l.last_stage_layers) {
        const int mid = s.L - l.first_stage_layers - l.last_stage_layers;
        if (vpp != 1) return bad("an uneven pipeline split cannot be combined with vpp");
        if (l.pp < 2 || !l.first_stage_layers || !l.last_stage_layers)
            return bad("an uneven pipeline split needs pp >= 2 and both first and last stage sizes");
        if (l.pp == 2 ? mid != 0 : (mid <= 0 || mid % (l.pp - 2)))
            return bad("layers between the first and last stage not divisible by pp - 2");
    } else if (s.L % (l.pp * vpp)) {
        return bad("layers not divisible by pp * vpp");
    }
    if (s.nq % l.tp) return bad("query heads not divisible by tp");
    if (s.family != RESHARD_MOE_MLA) {
        if (s.nkv <= 0 || s.d <= 0) return fail(RESHARD_ERR_INVALID_ARG, "nkv, d must be positive");
        if (s.nq % s.nkv) return bad("query heads not divisible by KV heads");
        if (s.nkv % l.tp && l.tp % s.nkv) return bad("KV heads neither divide nor are divided by tp");
    } else if (s.q_lora <= 0 || s.kv_lora <= 0 || s.nope <= 0 || s.rope <= 0 || s.v_dim <= 0) {
        return fail(RESHARD_ERR_INVALID_ARG, "MLA dimensions must be positive");
    }
    if (s.family == RESHARD_DENSE_GQA) {
        if (s.I <= 0) return fail(RESHARD_ERR_INVALID_ARG, "I must be positive");
        if (s.I % l.tp) return bad("feed-forward width not divisible by tp");
        if (l.ep != 1) return bad("a dense model has no expert parallelism");
    } else {
        if (s.E <= 0 || s.Ie <= 0) return fail(RESHARD_ERR_INVALID_ARG, "E, Ie must be positive");
        if (s.E % l.ep) return bad("experts not divisible by ep");
        if (s.n_shared < 0) return fail(RESHARD_ERR_INVALID_ARG, "n_shared must be >= 0");
        if ((int64_t(s.n_shared) * s.Ie) % l.tp) return bad("shared-expert width not divisible by tp");
        if (l.etp < 0) return fail(RESHARD_ERR_INVALID_ARG, "etp must be >= 0");
        if (l.etp > 1 && l.etp != l.tp) return bad("expert tensor parallelism must be 1 or equal to tp");
        if (l.etp > 1 && s.Ie % l.etp) return bad("expert width not divisible by etp");
    }
    if (s.has_embeddings) {
        if (s.V <= 0) return fail(RESHARD_ERR_INVALID_ARG, "V must be positive");
        if (l.vocab_padded < 0 || (l.vocab_padded && l.vocab_padded < s.V))
            return fail(RESHARD_ERR_INVALID_ARG, "vocab_padded must be 0 or at least V");
        if ((l.vocab_padded ? l.vocab_padded : s.V) % l.tp) return bad("(padded) vocabulary not divisible by tp");
    }
    return RESHARD_OK;
}

}  // namespace

void set_error(const std::string &msg) { g_error = msg; }
int fail(int code, const std::string &msg) {
    g_error = msg;
    return code;
}
const char *last_error_cstr() { return g_error.c_str(); }

namespace {
std::mutex g_tuning_mutex;
Tuning g_tuning;
}  // namespace

Tuning current_tuning() {
    std::lock_guard<std::mutex> g(g_tuning_mutex);
    return g_tuning;
}

void set_default_tuning(const Tuning &t) {
    std::lock_guard<std::mutex> g(g_tuning_mutex);
    g_tuning = t;
}

int tuning_from_abi(const reshard_tuning *t, Tuning &out) {
    Tuning n;  // built-in defaults
    if (t) {
        if (t->tile_bytes) {
            if (t->tile_bytes < 4096 || t->tile_bytes > 512 * 1024 || (t->tile_bytes & (t->tile_bytes - 1)))
                return fail(RESHARD_ERR_INVALID_ARG, "tile_bytes must be a power of two in [4 KiB, 512 KiB]");
            n.tile_bytes = t->tile_bytes;
        }
        if (t->block_threads) {
            const int b = t->block_threads;
            if (b != 64 && b != 128 && b != 256 && b != 512 && b != 1024)
                return fail(RESHARD_ERR_INVALID_ARG, "block_threads must be 64, 128, 256, 512 or 1024");
            n.block_threads = b;
        }
        if (t->blocks_per_cu) {
            if (t->blocks_per_cu < 1 || t->blocks_per_cu > 64)
                return fail(RESHARD_ERR_INVALID_ARG, "blocks_per_cu must be in [0, 64]");
            n.blocks_per_cu = t->blocks_per_cu;
        }
        if (t->unroll) {
            const int u = t->unroll;
            if (u != 1 && u != 2 && u != 4 && u != 8) return fail(RESHARD_ERR_INVALID_ARG, "unroll must be 1, 2, 4 or 8");
            n.unroll = u;
        }
        for (int v : {t->transpose_rows, t->transpose_cols})
            if (v != 0 && v != 64 && v != 128 && v != 192 && v != 256 && v != 512)
                return fail(RESHARD_ERR_INVALID_ARG, "transpose_rows / transpose_cols must be 64, 128, 192, 256 or 512");
        if (t->transpose_rows) n.transpose_rows = t->transpose_rows;
        if (t->transpose_cols) n.transpose_cols = t->transpose_cols;
        if (t->flags < -1 || t->flags > 127) return fail(RESHARD_ERR_INVALID_ARG, "flags must be in [-1, 127]");
        // 0 keeps the default like every other field; -1 asks for plain loads and stores, no barrier
        if (t->flags > 0) n.flags = t->flags;
        if (t->flags == -1) n.flags = 0;
        if (t->tail_pool_percent < 0 || t->tail_pool_percent > 50)
            return fail(RESHARD_ERR_INVALID_ARG, "tail_pool_percent must be in [0, 50]");
        n.tail_pool_percent = t->tail_pool_percent;
        if (t->tail_chunk_tiles) {
            if (t->tail_chunk_tiles < 1 || t->tail_chunk_tiles > 1024)
                return fail(RESHARD_ERR_INVALID_ARG, "tail_chunk_tiles must be in [1, 1024]");
            n.tail_chunk_tiles = t->tail_chunk_tiles;
        }
        if (t->table_copies < 0 || t->table_copies > 64) return fail(RESHARD_ERR_INVALID_ARG, "table_copies must be in [0, 64]");
        if (t->table_copies) n.table_copies = t->table_copies;  // 0 keeps what the defaults say (built in: chosen from the table size)
        // the one-tile copy kernel is built for every hint set at unroll 2, for none or all at the others
        const int hints = n.flags & 7;
        if (n.blocks_per_cu == 0 && n.unroll != 2 && hints != 0 && hints != 7)
            return fail(RESHARD_ERR_INVALID_ARG, "with unroll 1, 4 or 8 the hint bits 0-2 must be all set or all clear");
    }
    out = n;
    return RESHARD_OK;
}

void tuning_to_abi(const Tuning &t, reshard_tuning *out) {
    out->tile_bytes = t.tile_bytes;
    out->block_threads = t.block_threads;
    out->blocks_per_cu = t.blocks_per_cu;
    out->unroll = t.unroll;
    out->flags = t.flags;
    out->transpose_rows = t.transpose_rows;
    out->transpose_cols = t.transpose_cols;
    out->tail_pool_percent = t.tail_pool_percent;
    out->tail_chunk_tiles = t.tail_chunk_tiles;
    out->table_copies = t.table_copies;
}

int build_side(const reshard_model_spec &s, const reshard_layout &l, bool is_source, Side &out) {
    if (int rc = check_shape(s, l)) return rc;
    if (is_source && (l.tp_rank_filter >= 0 || l.ep_rank_filter >= 0))
        return fail(RESHARD_ERR_INVALID_ARG, "rank filters apply to the destination only");
    if (l.tp_rank_filter >= l.tp || l.ep_rank_filter >= l.ep)
        return fail(RESHARD_ERR_INVALID_ARG, "rank filter out of range");
    const int T = l.tp, P = l.pp, X = l.ep, eb = s.elem_bytes;
    const bool moe = s.family != RESHARD_DENSE_GQA, mla = s.family == RESHARD_MOE_MLA;
    const bool gen = l.kind == RESHARD_GEN;
    const bool grouped = !gen && l.expert_layout == RESHARD_GROUPED;
    const int64_t H = s.H;
    const bool tied = s.tied_embeddings && s.has_embeddings;
    // layers of every stage in storage order
    std::vector<std::vector<int>> stage_layers(P);
    if (l.first_stage_layers || l.last_stage_layers) {
        const int mid = P > 2 ? (s.L - l.first_stage_layers - l.last_stage_layers) / (P - 2) : 0;
        int next = 0;
        for (int p = 0; p < P; ++p) {
            const int n = p == 0 ? l.first_stage_layers : p == P - 1 ? l.last_stage_layers : mid;
            for (int i = 0; i < n; ++i) stage_layers[p].push_back(next++);
        }
    } else {
        const int v = l.vpp > 0 ? l.vpp : 1, chunk = s.L / (P * v);
        for (int c = 0; c < P * v; ++c)  // chunk c -> stage c mod P, appended in chunk order
            for (int i = 0; i < chunk; ++i) stage_layers[c % P].push_back(c * chunk + i);
    }
    out = Side{};
    out.layout = l;
    out.nd = P * T;
    const int Y = moe && l.etp > 0 ? l.etp : 1;  // expert-tensor ranks per expert rank
    out.ne = moe ? P * X * Y : 0;
    if (int64_t(P) * T + (moe ? int64_t(P) * X * Y : 0) > kMaxLayoutBuffers)
        return fail(RESHARD_ERR_UNSUPPORTED, "too many buffers in one layout");
    out.buf_bytes.assign(out.nd + out.ne, 0);
    out.used.assign(out.nd + out.ne, 0);

    for (int p = 0; p < P; ++p) {
        for (int t = 0; t < T; ++t) {
            const int b = p * T + t;
            const bool kept = is_source || l.tp_rank_filter < 0 || l.tp_rank_filter == t;
            // a source reads replicated tensors from tensor rank 0 only
            BufferBuilder bb(out, b, eb, kept, is_source, t == 0);
            if (!is_source) out.used[b] = kept;
            const int64_t vrows = (l.vocab_padded ? l.vocab_padded : s.V) / T;  // per rank, padding included
            if (s.has_embeddings && p == 0) bb.vocab_shard("emb", LT_EMB, t * vrows, vrows, s.V, H);
            for (const int L_ : stage_layers[p]) {
                bb.whole("ln1", LT_LN1, L_, 0, 1, 0, H);
                if (mla) {
                    const int64_t heads = s.nq / T;
                    const int64_t qrows = heads * (s.nope + s.rope), kvrows = heads * (s.nope + s.v_dim);
                    bb.whole("q_a", LT_QA, L_, 0, s.q_lora, 0, H);
                    bb.whole("q_a_ln", LT_QA_LN, L_, 0, 1, 0, s.q_lora);
                    bb.whole("q_b", LT_QB, L_, t * qrows, qrows, 0, s.q_lora);
                    bb.whole("kv_a", LT_KVA, L_, 0, s.kv_lora + s.rope, 0, H);
                    bb.whole("kv_a_ln", LT_KVA_LN, L_, 0, 1, 0, s.kv_lora);
                    bb.whole("kv_b", LT_KVB, L_, t * kvrows, kvrows, 0, s.kv_lora);
                    bb.whole("wo", LT_WO, L_, 0, H, t * heads * s.v_dim, heads * s.v_dim);
                } else {
                    const int64_t d = s.d, g = s.nq / s.nkv;
                    const bool kv_shared = T > s.nkv;           // each KV head replicated on T/nkv ranks
                    const int64_t groups = kv_shared ? 1 : s.nkv / T;  // KV heads stored by this rank
                    const int64_t qrows = int64_t(s.nq) / T * d, krows = groups * d;
                    for (int pass = 0; pass < (s.qkv_bias ? 2 : 1); ++pass) {
                        const bool bias = pass == 1;
                        const int64_t w = bias ? 1 : H;         // a bias is a one-column matrix
                        const int iq = bias ? LT_BQ : LT_WQ, ik = bias ? LT_BK : LT_WK, iv = bias ? LT_BV : LT_WV;
                        const int64_t at = bb.begin(bias ? "qkv_b" : "qkv_w", L_, -1, (qrows + 2 * krows) * w, false);
                        if (kv_shared) {
                            // both kinds: the rank's query rows, then the shared key and value head;
                            // a source reads the head from the lowest rank holding it
                            const int64_t rep = T / s.nkv, head = t / rep;
                            const bool first_copy = t % rep == 0;
                            bb.frag(iq, L_, -1, t * qrows, (t + 1) * qrows, 0, w, at, w);
                            bb.frag(ik, L_, -1, head * d, (head + 1) * d, 0, w, at + qrows * w * eb, w, false, first_copy);
                            bb.frag(iv, L_, -1, head * d, (head + 1) * d, 0, w, at + (qrows + d) * w * eb, w, false, first_copy);
                        } else if (gen) {
                            // blocked: this rank's query rows, key rows, value rows
                            bb.frag(iq, L_, -1, t * qrows, (t + 1) * qrows, 0, w, at, w);
                            bb.frag(ik, L_, -1, t * krows, (t + 1) * krows, 0, w, at + qrows * w * eb, w);
                            bb.frag(iv, L_, -1, t * krows, (t + 1) * krows, 0, w, at + (qrows + krows) * w * eb, w);
                        } else {
                            // interleaved per KV group: g query heads, key head, value head
                            const int64_t span = (g + 2) * d;
                            for (int64_t j = 0; j < groups; ++j) {
                                const int64_t G = t * groups + j, base = at + j * span * w * eb;
                                bb.frag(iq, L_, -1, G * g * d, (G + 1) * g * d, 0, w, base, w);
                                bb.frag(ik, L_, -1, G * d, (G + 1) * d, 0, w, base + g * d * w * eb, w);
                                bb.frag(iv, L_, -1, G * d, (G + 1) * d, 0, w, base + (g + 1) * d * w * eb, w);
                            }
                        }
                    }
                    const int64_t ocols = int64_t(s.nq) * d / T;
                    bb.whole("wo", LT_WO, L_, 0, H, t * ocols, ocols);
                }
                bb.whole("ln2", LT_LN2, L_, 0, 1, 0, H);
                // fused gate/up (column-parallel halves) and down (row-parallel)
                auto ffn = [&](const char *n1, const char *n2, int ig, int iu, int idn, int64_t width) {
                    const int64_t n = width / T;
                    const int64_t at = bb.begin(n1, L_, -1, 2 * n * H, false);
                    bb.frag(ig, L_, -1, t * n, (t + 1) * n, 0, H, at, H);
                    bb.frag(iu, L_, -1, t * n, (t + 1) * n, 0, H, at + n * H * eb, H);
                    bb.whole(n2, idn, L_, 0, H, t * n, n);
                };
                if (!moe) {
                    ffn("gate_up", "down", LT_GATE, LT_UP, LT_DOWN, s.I);
                } else {
                    bb.whole("router", LT_ROUTER, L_, 0, s.E, 0, H);
                    if (s.n_shared) ffn("sh_fc1", "sh_fc2", LT_SH_GATE, LT_SH_UP, LT_SH_DOWN, int64_t(s.n_shared) * s.Ie);
                }
            }
            if (s.has_embeddings && p == P - 1) {
                bb.whole("final_ln", LT_FINAL_LN, -1, 0, 1, 0, H);
                if (!tied)
                    bb.vocab_shard("lm_head", LT_LM_HEAD, t * vrows, vrows, s.V, H);
                else if (P > 1)  // the tied output layer's own copy; never the one a source reads
                    bb.vocab_shard("emb_tied", LT_EMB, t * vrows, vrows, s.V, H, false);
            }
            out.buf_bytes[b] = bb.finish();
        }
        if (!moe) continue;
        // Expert buffer (p, x, y): whole experts x*E/X .. when Y == 1; with expert tensor parallelism
        // (Y == T) expert-tensor rank y holds rows y*n.. of gate and up and columns y*n.. of down.
        const int64_t n = s.Ie / Y, El = s.E / X;
        for (int x = 0; x < X; ++x)
            for (int y = 0; y < Y; ++y) {
                const int b = out.nd + (p * X + x) * Y + y;
                const bool kept = is_source || ((l.ep_rank_filter < 0 || l.ep_rank_filter == x) &&
                                                (Y == 1 || l.tp_rank_filter < 0 || l.tp_rank_filter == y));
                BufferBuilder bb(out, b, eb, kept, is_source, true, true);
                if (!is_source) out.used[b] = kept;
                const int64_t r0 = y * n, r1 = (y + 1) * n;  // this buffer's slice of the expert width
                for (const int L_ : stage_layers[p]) {
                    if (gen || grouped) {
                        const int64_t a1 = bb.begin(gen ? "w13" : "w1", L_, -1, El * 2 * n * H, false);
                        const int64_t a2 = bb.begin("w2", L_, -1, El * n * H, false);
                        for (int64_t j = 0; j < El; ++j) {
                            const int e = int(x * El + j);
                            if (gen) {
                                const int64_t base = a1 + j * 2 * n * H * eb;
                                bb.frag(LT_EX_GATE, L_, e, r0, r1, 0, H, base, H);
                                bb.frag(LT_EX_UP, L_, e, r0, r1, 0, H, base + n * H * eb, H);
                                bb.frag(LT_EX_DOWN, L_, e, 0, H, r0, r1, a2 + j * H * n * eb, n);
                            } else {
                                // [expert][in][out]: logical (out r, in c) sits at column-major position
                                const int64_t base = a1 + j * H * 2 * n * eb;
                                bb.frag(LT_EX_GATE, L_, e, r0, r1, 0, H, base, 2 * n, true);
                                bb.frag(LT_EX_UP, L_, e, r0, r1, 0, H, base + n * eb, 2 * n, true);
                                bb.frag(LT_EX_DOWN, L_, e, 0, H, r0, r1, a2 + j * n * H * eb, H, true);
                            }
                        }
                    } else {
                        for (int64_t j = 0; j < El; ++j) {
                            const int e = int(x * El + j);
                            const int64_t a1 = bb.begin("fc1", L_, e, 2 * n * H, false);
                            bb.frag(LT_EX_GATE, L_, e, r0, r1, 0, H, a1, H);
                            bb.frag(LT_EX_UP, L_, e, r0, r1, 0, H, a1 + n * H * eb, H);
                            const int64_t a2 = bb.begin("fc2", L_, e, H * n, false);
                            bb.frag(LT_EX_DOWN, L_, e, 0, H, r0, r1, a2, n);
                        }
                    }
                }
                out.buf_bytes[b] = bb.finish();
            }
    }
    std::stable_sort(out.tensors.begin(), out.tensors.end(),
                     [](const reshard_tensor_info &a, const reshard_tensor_info &b) { return a.buffer < b.buffer; });
    return RESHARD_OK;
}

namespace {

// Folds a descriptor whose rows are back to back on both sides into one long row.
void normalise(reshard_desc &d) {
    if (d.kind == 0 && d.rows > 1 && d.src_stride == d.row_bytes && d.dst_stride == d.row_bytes) {
        d.row_bytes *= d.rows;
        d.rows = 1;
    }
    if (d.kind == 0 && d.rows == 1) d.src_stride = d.dst_stride = d.row_bytes;
    if (d.kind == 1) {
        // a one-row or one-column transpose is a strided copy of single elements; a
        // 1 x n or n x 1 block with unit strides is a plain run
        const int64_t cols = d.row_bytes / d.elem_bytes;
        if (d.rows == 1 && d.dst_stride == d.elem_bytes) {
            d.kind = 0;
            d.src_stride = d.dst_stride = d.row_bytes;
        } else if (cols == 1 && d.src_stride == d.elem_bytes) {
            d.kind = 0;
            d.row_bytes = d.rows * d.elem_bytes;
            d.rows = 1;
            d.src_stride = d.dst_stride = d.row_bytes;
        }
    }
}

// Appends `d` to the table, merging it into the previous descriptor when the two
// are adjacent on both sides.
void append_merged(std::vector<reshard_desc> &out, reshard_desc d) {
    normalise(d);
    if (!out.empty()) {
        reshard_desc &p = out.back();
        if (p.kind == 0 && d.kind == 0 && p.src_buf == d.src_buf && p.dst_buf == d.dst_buf) {
            if (p.rows == 1 && d.rows == 1 && p.src_off + p.row_bytes == d.src_off &&
                p.dst_off + p.row_bytes == d.dst_off) {
                p.row_bytes += d.row_bytes;
                p.src_stride = p.dst_stride = p.row_bytes;
                return;
            }
            if (p.row_bytes == d.row_bytes && p.rows >= 1 && d.rows >= 1) {
                // stack row blocks with equal pitch
                const bool p_multi = p.rows > 1, d_multi = d.rows > 1;
                int64_t ss = p_multi ? p.src_stride : d_multi ? d.src_stride : d.src_off - p.src_off;
                int64_t ds = p_multi ? p.dst_stride : d_multi ? d.dst_stride : d.dst_off - p.dst_off;
                // a tile record holds 32-bit pitches: rows further apart stay separate descriptors
                const bool pitch_ok = ss >= p.row_bytes && ds >= p.row_bytes && ss <= 0xFFFFFFFFll && ds <= 0xFFFFFFFFll &&
                                      (!p_multi || (p.src_stride == ss && p.dst_stride == ds)) &&
                                      (!d_multi || (d.src_stride == ss && d.dst_stride == ds));
                if (pitch_ok && d.src_off == p.src_off + p.rows * ss && d.dst_off == p.dst_off + p.rows * ds &&
                    !(ss == p.row_bytes && ds == p.row_bytes)) {
                    p.rows += d.rows;
                    p.src_stride = ss;
                    p.dst_stride = ds;
                    return;
                }
            }
        }
    }
    out.push_back(d);
}

}  // namespace

int compile_descriptors(const reshard_model_spec &spec, Side &src, Side &dst,
                        std::vector<reshard_desc> &descs) {
    const int64_t eb = spec.elem_bytes;
    // index the source fragments by logical tensor
    std::vector<uint32_t> order(src.frags.size());
    for (uint32_t i = 0; i < order.size(); ++i) order[i] = i;
    std::stable_sort(order.begin(), order.end(),
                     [&](uint32_t a, uint32_t b) { return src.frags[a].key < src.frags[b].key; });
    auto first_of = [&](uint64_t key) {
        return std::lower_bound(order.begin(), order.end(), key,
                                [&](uint32_t a, uint64_t k) { return src.frags[a].key < k; });
    };
    std::fill(src.used.begin(), src.used.end(), 0);
    descs.clear();
    for (const Fragment &D : dst.frags) {
        int64_t covered = 0;
        for (auto it = first_of(D.key); it != order.end() && src.frags[*it].key == D.key; ++it) {
            const Fragment &S = src.frags[*it];
            const int64_t ra = std::max(S.r0, D.r0), rb = std::min(S.r1, D.r1);
            const int64_t ca = std::max(S.c0, D.c0), cb = std::min(S.c1, D.c1);
            if (ra >= rb || ca >= cb) continue;
            covered += (rb - ra) * (cb - ca);
            auto address = [&](const Fragment &F) {
                return F.transposed ? F.off + ((ca - F.c0) * F.ld + (ra - F.r0)) * eb
                                    : F.off + ((ra - F.r0) * F.ld + (ca - F.c0)) * eb;
            };
            reshard_desc d{};
            d.src_buf = S.buf;
            d.dst_buf = D.buf;
            d.elem_bytes = int32_t(eb);
            d.src_off = address(S);
            d.dst_off = address(D);
            d.src_stride = S.ld * eb;
            d.dst_stride = D.ld * eb;
            if (S.transposed == D.transposed) {
                d.kind = 0;
                // walk along whichever logical axis is contiguous on both sides
                d.rows = S.transposed ? cb - ca : rb - ra;
                d.row_bytes = (S.transposed ? rb - ra : cb - ca) * eb;
            } else {
                d.kind = 1;
                // i runs along the source's slow axis, k along its fast axis
                d.rows = S.transposed ? cb - ca : rb - ra;
                d.row_bytes = (S.transposed ? rb - ra : cb - ca) * eb;
            }
            src.used[S.buf] = 1;
            append_merged(descs, d);
        }
        if (covered != (D.r1 - D.r0) * (D.c1 - D.c0))
            return fail(RESHARD_ERR_UNSUPPORTED, "internal: a destination fragment is not covered exactly once");
    }
    return RESHARD_OK;
}

int cut_tiles(const std::vector<reshard_desc> &descs, int num_src_bufs, const Tuning &tuning,
              int fast_rows, int fast_cols, std::vector<TileClass> &classes) {
    const int tile_bytes = tuning.tile_bytes;
    classes.clear();
    classes.resize(2);
    classes[0].kind = 0;
    classes[1].kind = 1;
    classes[1].rows = fast_rows;
    classes[1].cols = fast_cols;
    TileClass generic;
    generic.kind = 2;
    // copy tiles of one contiguous row / of several pitched rows / pitched rows that also have a gathered form / that form
    std::vector<Tile> run_tiles, block_tiles, regathered_tiles, gathered_tiles;
    size_t group_left = 0;  // descriptors still to come of the gathered group being cut
    auto reg_class = [&](int ti, int tk) -> std::vector<Tile> & {
        for (size_t c = 1; c < classes.size(); ++c)
            if (classes[c].rows == ti && classes[c].cols == tk) return classes[c].tiles;
        TileClass n;
        n.kind = 1;
        n.rows = ti;
        n.cols = tk;
        classes.push_back(n);
        return classes.back().tiles;
    };
    auto fits32 = [](int64_t v) { return v >= 0 && v <= 0xFFFFFFFFll; };
    // Descriptors di .. di + k - 1 (k = 2^n, 1 <= k <= 256) whose rows of `units` 16-byte units interleave into ONE
    // contiguous stretch of the destination: row r of the stretch is row r of source j0, j0 + 1, ... in turn (the
    // shards of a row-parallel weight merged side by side; k == 1: rows packed from a pitched source).  Returns k,
    // or 0 when the descriptors at di do not have that form.
    auto gather_group = [&](size_t di, int64_t units) -> size_t {
        const reshard_desc &d = descs[di];
        const int64_t S = d.row_bytes;
        if (units < 64 || S != units * 16 || d.dst_stride % S || d.src_stride < S) return 0;
        const int64_t k = d.dst_stride / S;
        if (k < 1 || k > 256 || (k & (k - 1)) || di + size_t(k) > descs.size()) return 0;
        if (k == 1 && d.src_stride == S) return 0;
        for (int64_t j = 1; j < k; ++j) {
            const reshard_desc &e = descs[di + size_t(j)];
            if (e.kind != 0 || e.rows != d.rows || e.row_bytes != S || e.src_stride != d.src_stride ||
                e.dst_stride != d.dst_stride || e.dst_buf != d.dst_buf || e.src_buf != d.src_buf + j ||
                e.src_off != d.src_off || e.dst_off != d.dst_off + j * S)
                return 0;
        }
        return size_t(k);
    };
    for (size_t di = 0; di < descs.size(); ++di) {
        const reshard_desc &d = descs[di];
        // a single row (a contiguous run of any length) has no pitch
        const bool pitched = d.rows > 1 || d.kind == 1;
        if (pitched && (!fits32(d.src_stride) || !fits32(d.dst_stride)))
            return fail(RESHARD_ERR_UNSUPPORTED, "a row pitch exceeds 4 GiB");
        Tile t{};
        t.src_buf = uint16_t(d.src_buf);
        t.dst_buf = uint16_t(num_src_bufs + d.dst_buf);
        t.src_stride = pitched ? uint32_t(d.src_stride) : 0;
        t.dst_stride = pitched ? uint32_t(d.dst_stride) : 0;
        if (d.kind == 1) {
            if (group_left) return fail(RESHARD_ERR_UNSUPPORTED, "internal: a gathered group ends early");
            int lg = 0;
            while ((1 << lg) < d.elem_bytes) ++lg;
            const int E = d.elem_bytes;
            const int64_t cols = d.row_bytes / d.elem_bytes;
            t.kind = 1;
            t.vec_log2 = uint8_t(lg);
            auto emit = [&](int64_t i, int64_t k, int64_t ni, int64_t nk, std::vector<Tile> &out) {
                t.rows = uint32_t(ni);
                t.row_units = uint32_t(nk);
                t.src_off = uint64_t(d.src_off + i * d.src_stride + k * d.elem_bytes);
                t.dst_off = uint64_t(d.dst_off + k * d.dst_stride + i * d.elem_bytes);
                out.push_back(t);
            };
            // generic tiles: any extent, cut at kTransposeDim
            auto generic_rect = [&](int64_t i0, int64_t i1, int64_t k0, int64_t k1) {
                for (int64_t i = i0; i < i1; i += kTransposeDim)
                    for (int64_t k = k0; k < k1; k += kTransposeDim)
                        emit(i, k, std::min<int64_t>(kTransposeDim, i1 - i), std::min<int64_t>(kTransposeDim, k1 - k),
                             generic.tiles);
            };
            const bool reg_path = (d.src_off | d.dst_off | d.src_stride | d.dst_stride) % 16 == 0;
            // Largest register-path shape that fits an R x C rectangle: the preferred shape if it
            // fits, else the fitting shape of the largest area (the longer source rows on a tie).
            auto best_shape = [&](int64_t R, int64_t C, int &ti, int &tk) {
                if (fast_rows <= R && fast_cols <= C && transpose_shape_ok(E, fast_rows, fast_cols)) {
                    ti = fast_rows;
                    tk = fast_cols;
                    return true;
                }
                int64_t best = 0;
                for (int a : {512, 256, 192, 128, 64})
                    for (int b : {512, 256, 192, 128, 64})
                        if (a <= R && b <= C && transpose_shape_ok(E, a, b) && int64_t(a) * b > best) {
                            best = int64_t(a) * b;
                            ti = a;
                            tk = b;
                        }
                return best > 0;
            };
            // Full tiles of the best shape from the rectangle's corner, then the same again for the
            // strip to the right of them and the strip below; what no shape fits goes to the generic kernel.
            struct Rect { int64_t i0, i1, k0, k1; };
            std::vector<Rect> todo{{0, d.rows, 0, cols}};
            while (!todo.empty()) {
                const Rect r = todo.back();
                todo.pop_back();
                if (r.i0 >= r.i1 || r.k0 >= r.k1) continue;
                int ti = 0, tk = 0;
                if (!reg_path || !best_shape(r.i1 - r.i0, r.k1 - r.k0, ti, tk)) {
                    generic_rect(r.i0, r.i1, r.k0, r.k1);
                    continue;
                }
                const int64_t ci = (r.i1 - r.i0) / ti * ti, ck = (r.k1 - r.k0) / tk * tk;
                std::vector<Tile> &out = reg_class(ti, tk);
                for (int64_t i = r.i0; i < r.i0 + ci; i += ti)
                    for (int64_t k = r.k0; k < r.k0 + ck; k += tk) emit(i, k, ti, tk, out);
                todo.push_back({r.i0 + ci, r.i1, r.k0, r.k1});       // below
                todo.push_back({r.i0, r.i0 + ci, r.k0 + ck, r.k1});  // right of the tiles
            }
            continue;
        }
        // single rows (contiguous runs) and row blocks are kept apart: the copy class lists the row blocks first
        // widest vector that every row start and the row length allow
        int vec = 16;
        auto misfit = [&](int v) {
            if (d.row_bytes % v || d.src_off % v || d.dst_off % v) return true;
            return d.rows > 1 && (d.src_stride % v || d.dst_stride % v);
        };
        while (vec > 1 && misfit(vec)) vec >>= 1;
        int64_t units = d.row_bytes / vec;
        if (units == 1 && d.rows > 1 && vec > 1) {  // keep the row split well defined
            vec >>= 1;
            units = 2;
        }
        int lg = 0;
        while ((1 << lg) < vec) ++lg;
        t.kind = 0;
        t.vec_log2 = uint8_t(lg);
        const int64_t max_units = std::max<int64_t>(1, std::min<int64_t>(tile_bytes / vec, kMaxTileUnits));
        if (d.rows == 1 || units >= max_units || units == 1) {
            // long rows: cut every row into runs.  The cuts fall on multiples of the tile size in the DESTINATION
            // buffer (a short first piece brings the row there), so that in the woven order, where the XCD on
            // which a 1 KiB granule lands is its index in the tile modulo 8, an XCD always writes the same
            // 1 KiB residues of every 8 KiB of the buffer, whatever run the tile belongs to.
            if (group_left) return fail(RESHARD_ERR_UNSUPPORTED, "internal: a gathered group ends early");
            const int64_t tile_span = max_units * vec;
            for (int64_t r = 0; r < d.rows; ++r) {
                const int64_t row_dst = d.dst_off + r * d.dst_stride;
                int64_t head = ((tile_span - row_dst % tile_span) % tile_span) / vec;
                if (head >= units) head = 0;
                for (int64_t u = 0; u < units;) {
                    const int64_t len = (u == 0 && head > 0) ? head : std::min(max_units, units - u);
                    t.rows = 1;
                    t.row_units = uint32_t(len);
                    t.magic = 0;
                    t.src_off = uint64_t(d.src_off + r * d.src_stride + u * vec);
                    t.dst_off = uint64_t(row_dst + u * vec);
                    run_tiles.push_back(t);
                    u += len;
                }
            }
        } else {
            // short rows.  Where the rows of this descriptor (and of the k - 1 that follow) fill one contiguous
            // stretch of the destination, that stretch is ALSO cut like a run, into gathered tiles (same cuts on
            // destination multiples of the tile size): the woven order takes those, the other orders the row blocks.
            if (!group_left && vec == 16) {
                const size_t k = gather_group(di, units);
                if (k) {
                    group_left = k;
                    int lk = 0;
                    while ((size_t(1) << lk) < k) ++lk;
                    const int64_t total = d.rows * int64_t(k) * units, tile_span = max_units * 16;
                    int64_t head = ((tile_span - d.dst_off % tile_span) % tile_span) / 16;
                    if (head >= total) head = 0;
                    Tile g = t;
                    g.kind = 2;
                    g.row_units = uint32_t(units);
                    g.magic = uint32_t((uint64_t(1) << 32) / uint64_t(units)) + 1u;
                    g.dst_stride = uint32_t(d.src_stride / 16);
                    for (int64_t u = 0; u < total;) {
                        const int64_t len = (u == 0 && head > 0) ? head : std::min(max_units, total - u);
                        const int64_t seg = u / units, c0 = u % units, j0 = seg % int64_t(k), r0 = seg / int64_t(k);
                        g.rows = uint32_t(len);
                        g.src_stride = uint32_t(c0) | uint32_t(j0) << 16 | uint32_t(lk) << 24;
                        g.src_off = uint64_t(d.src_off + r0 * d.src_stride);
                        g.dst_off = uint64_t(d.dst_off + u * 16);
                        gathered_tiles.push_back(g);
                        u += len;
                    }
                }
            }
            // several whole rows per tile
            const int64_t rows_per_tile = std::max<int64_t>(1, max_units / units);
            for (int64_t r = 0; r < d.rows; r += rows_per_tile) {
                t.rows = uint32_t(std::min(rows_per_tile, d.rows - r));
                t.row_units = uint32_t(units);
                t.magic = t.rows == 1 ? 0u : uint32_t((uint64_t(1) << 32) / uint64_t(units)) + 1u;
                t.src_off = uint64_t(d.src_off + r * d.src_stride);
                t.dst_off = uint64_t(d.dst_off + r * d.dst_stride);
                (group_left ? regathered_tiles : t.rows == 1 ? run_tiles : block_tiles).push_back(t);
            }
            if (group_left) --group_left;
        }
    }
    {
        TileClass &c = classes[0];
        c.num_regathered = uint32_t(regathered_tiles.size());
        c.num_blocks = uint32_t(block_tiles.size()) + c.num_regathered;
        c.num_runs = uint32_t(run_tiles.size());
        c.num_gathered = uint32_t(gathered_tiles.size());
        c.tiles = std::move(block_tiles);
        c.tiles.insert(c.tiles.end(), regathered_tiles.begin(), regathered_tiles.end());
        c.tiles.insert(c.tiles.end(), run_tiles.begin(), run_tiles.end());
        c.tiles.insert(c.tiles.end(), gathered_tiles.begin(), gathered_tiles.end());
        for (size_t i = 0; i < c.tiles.size(); ++i) {
            const Tile &t = c.tiles[i];
            c.max_units = std::max(c.max_units, t.kind == 2 ? t.rows : t.rows * t.row_units);
            if (i >= c.num_blocks) c.runs_wide = c.runs_wide && t.vec_log2 == 4;
        }
    }
    classes.push_back(std::move(generic));
    return RESHARD_OK;
}

}  // namespace reshard
