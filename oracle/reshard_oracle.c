/*
 * Loop oracle for the weight-resharding step.  TEST INFRASTRUCTURE ONLY: the
 * product library never links, loads or calls this file; the tests, the smoke
 * check and the benchmark's CPU-baseline leg do.
 *
 * What it computes (Allgather-Swap Technique section, step 2: select and copy
 * the weight slices needed for generation): every weight element is moved,
 * bit for bit, from its place in the source-side shards to its place in the
 * destination-side shards.  The paper prints no layout; the conventions are
 * the Megatron-style ones fixed by this repository (tensor-parallel column and
 * row splits, pipeline stages, fused QKV interleaved per KV-head group on the
 * training side and blocked Q|K|V on the generation side, fused gate/up,
 * expert-parallel blocks; weight classes T / E / C as in the paper's
 * redundant-memory example).
 *
 * Formulation: walk every destination buffer in storage order; each stored
 * tensor is a handful of rectangular pieces of logical tensors; each piece is
 * filled row by row, asking the source layout "where is logical (row, col) and
 * how many further columns are contiguous there", and memcpy-ing that run.
 * No blocking, fusion or reordering beyond that.  A second, independent
 * statement of the same mapping lives in locate.py; tests compare the two.
 *
 * Parity status: pinned, by element tracing, per-element write counts,
 * closed-form byte totals, the per-device bytes the paper's ablation prints
 * and numpy constructions in tests/.  The paper prints no worked example of
 * the mapping itself, so none of the pins is an element-level value from the
 * authors; the layout conventions are the public Megatron ones.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int family; /* 0 dense GQA, 1 MoE GQA, 2 MoE MLA */
    int L, H, nq, nkv, d, I, V, qkv_bias, has_embeddings;
    int E, Ie, n_shared, q_lora, kv_lora, nope, rope, v_dim, elem_bytes;
    int tied_embeddings; /* 1: no lm_head; with pp > 1 the last training stage keeps an embedding copy */
} orc_spec;

typedef struct {
    int kind;          /* 0 train, 1 gen */
    int tp, pp, ep;
    int expert_layout; /* 0 per-expert [out][in], 1 grouped [expert][in][out] */
    int tp_filter, ep_filter;
    int vpp;                /* virtual pipeline size: layer chunks dealt round-robin to the stages */
    int first_stage_layers; /* uneven split: layers on the first / last stage (0 = even) */
    int last_stage_layers;
    int vocab_padded;       /* rows the embedding / lm_head are padded to before the split (0 = V) */
    int etp;                /* expert tensor parallelism: 1 (whole experts) or tp */
} orc_layout;

enum { FAM_DENSE = 0, FAM_MOE = 1, FAM_MLA = 2 };
enum { K_TRAIN = 0, K_GEN = 1 };

/* logical tensors */
enum {
    T_EMB, T_FINAL_LN, T_LM_HEAD, T_LN1, T_WQ, T_WK, T_WV, T_BQ, T_BK, T_BV, T_WO, T_LN2,
    T_GATE, T_UP, T_DOWN, T_ROUTER, T_SH_GATE, T_SH_UP, T_SH_DOWN, T_EX_GATE, T_EX_UP,
    T_EX_DOWN, T_QA, T_QA_LN, T_QB, T_KVA, T_KVA_LN, T_KVB
};

/* stored tensors of a dense buffer, per layer */
enum {
    S_LN1, S_QKV_W, S_QKV_B, S_WO, S_LN2, S_GATE_UP, S_DOWN, S_ROUTER, S_SH_FC1, S_SH_FC2,
    S_QA, S_QA_LN, S_QB, S_KVA, S_KVA_LN, S_KVB, NSLOT
};

typedef struct {
    orc_spec s;
    orc_layout l;
    int T, P, X, Y, El, nd, ne, moe, grouped, tied; /* Y: expert-tensor ranks per expert rank */
    int64_t Vp;      /* vocabulary rows including padding */
    int *stage_of;   /* [L] stage holding a layer */
    int *order;      /* [L] layers sorted by (stage, storage position) */
    int *first;      /* [P+1] range of `order` belonging to a stage */
    int64_t eb;
    int64_t *doff;   /* [L][NSLOT] byte offset of a stored tensor in its stage's dense buffers */
    int64_t *eoff;   /* [L][El][2] byte offset in its stage's expert buffers (stacked: j = 0) */
    int64_t emb_off, final_ln_off, lm_head_off, emb_tied_off;
    int64_t *dense_bytes, *expert_bytes; /* [P] */
} ctx_t;

static int64_t up256(int64_t x) { return (x + 255) / 256 * 256; }

static int valid(const orc_spec *s, const orc_layout *l)
{
    if (s->family < 0 || s->family > 2) return 0;
    if (s->L <= 0 || s->H <= 0 || s->nq <= 0) return 0;
    if (s->elem_bytes != 1 && s->elem_bytes != 2 && s->elem_bytes != 4 && s->elem_bytes != 8) return 0;
    if (l->tp < 1 || l->pp < 1 || l->ep < 1) return 0;
    if (l->kind == K_GEN && l->pp != 1) return 0;
    if (l->vpp < 1) return 0;
    if (l->first_stage_layers || l->last_stage_layers) {
        int mid = s->L - l->first_stage_layers - l->last_stage_layers;
        if (l->vpp != 1 || l->pp < 2 || l->first_stage_layers <= 0 || l->last_stage_layers <= 0) return 0;
        if (l->pp == 2 ? mid != 0 : (mid <= 0 || mid % (l->pp - 2))) return 0;
    } else if (s->L % (l->pp * l->vpp)) return 0;
    if (s->nq % l->tp) return 0;
    if (s->family != FAM_MLA) {
        if (s->nkv <= 0 || s->d <= 0 || s->nq % s->nkv) return 0;
        if (s->nkv % l->tp && l->tp % s->nkv) return 0;
    } else if (s->q_lora <= 0 || s->kv_lora <= 0 || s->nope <= 0 || s->rope <= 0 || s->v_dim <= 0)
        return 0;
    if (s->family == FAM_DENSE) {
        if (s->I <= 0 || s->I % l->tp || l->ep != 1) return 0;
    } else {
        if (s->E <= 0 || s->Ie <= 0 || s->E % l->ep) return 0;
        if (l->etp != 1 && l->etp != l->tp) return 0;
        if (s->Ie % l->etp) return 0;
        if ((s->n_shared * s->Ie) % l->tp) return 0;
    }
    if (s->has_embeddings) {
        int vp = l->vocab_padded ? l->vocab_padded : s->V;
        if (s->V <= 0 || vp < s->V || vp % l->tp) return 0;
    }
    return 1;
}

static void ctx_free(ctx_t *c)
{
    free(c->doff); free(c->eoff); free(c->dense_bytes); free(c->expert_bytes);
    free(c->stage_of); free(c->order); free(c->first);
}

/* Lay the stored tensors of every stage out in order, each on a 256-byte boundary. */
static int ctx_init(ctx_t *c, const orc_spec *s, const orc_layout *l)
{
    memset(c, 0, sizeof *c);
    if (!valid(s, l)) return -1;
    c->s = *s; c->l = *l;
    c->T = l->tp; c->P = l->pp; c->X = l->ep;
    c->moe = s->family != FAM_DENSE;
    c->tied = s->tied_embeddings && s->has_embeddings;
    c->Vp = l->vocab_padded ? l->vocab_padded : s->V;
    /* which stage holds which layers, and in which order they are stored there */
    c->stage_of = calloc(s->L, sizeof(int));
    c->order = calloc(s->L, sizeof(int));
    c->first = calloc(c->P + 1, sizeof(int));
    {
        int n = 0;
        if (l->first_stage_layers || l->last_stage_layers) {
            int mid = c->P > 2 ? (s->L - l->first_stage_layers - l->last_stage_layers) / (c->P - 2) : 0;
            for (int p = 0; p < c->P; p++) {
                int cnt = p == 0 ? l->first_stage_layers : p == c->P - 1 ? l->last_stage_layers : mid;
                c->first[p] = n;
                for (int i = 0; i < cnt; i++) { c->stage_of[n] = p; c->order[n] = n; n++; }
            }
        } else {
            int lc = s->L / (c->P * l->vpp);
            for (int p = 0; p < c->P; p++) {
                c->first[p] = n;
                for (int k = 0; k < l->vpp; k++)          /* chunk k*P + p */
                    for (int i = 0; i < lc; i++) {
                        int ly = (k * c->P + p) * lc + i;
                        c->stage_of[ly] = p;
                        c->order[n++] = ly;
                    }
            }
        }
        c->first[c->P] = n;
    }
    c->El = c->moe ? s->E / c->X : 0;
    c->Y = c->moe ? l->etp : 1;
    c->nd = c->P * c->T;
    c->ne = c->moe ? c->P * c->X * c->Y : 0; /* expert buffer (p, x, y): nd + (p*X + x)*Y + y */
    c->grouped = l->kind == K_TRAIN && l->expert_layout == 1;
    c->eb = s->elem_bytes;
    c->doff = calloc((size_t)s->L * NSLOT, sizeof(int64_t));
    c->eoff = calloc((size_t)s->L * (c->El ? c->El : 1) * 2, sizeof(int64_t));
    c->dense_bytes = calloc(c->P, sizeof(int64_t));
    c->expert_bytes = calloc(c->P, sizeof(int64_t));
    const int64_t H = s->H, T = c->T, eb = c->eb;
    for (int p = 0; p < c->P; p++) {
        int64_t off = 0;
#define PUT(dst, nelem) do { off = up256(off); (dst) = off; off += (int64_t)(nelem) * eb; } while (0)
        if (s->has_embeddings && p == 0) PUT(c->emb_off, c->Vp / T * H);
        for (int at = c->first[p]; at < c->first[p + 1]; at++) {
            int ly = c->order[at];
            int64_t *o = c->doff + (size_t)ly * NSLOT;
            PUT(o[S_LN1], H);
            if (s->family == FAM_MLA) {
                int64_t nql = s->nq / T;
                PUT(o[S_QA], (int64_t)s->q_lora * H);
                PUT(o[S_QA_LN], s->q_lora);
                PUT(o[S_QB], nql * (s->nope + s->rope) * s->q_lora);
                PUT(o[S_KVA], (int64_t)(s->kv_lora + s->rope) * H);
                PUT(o[S_KVA_LN], s->kv_lora);
                PUT(o[S_KVB], nql * (s->nope + s->v_dim) * s->kv_lora);
                PUT(o[S_WO], H * nql * s->v_dim);
            } else {
                int64_t kvl = s->nkv / T > 0 ? s->nkv / T : 1; /* a replicated KV head when T > nkv */
                int64_t rows = (s->nq / T + 2 * kvl) * s->d;
                PUT(o[S_QKV_W], rows * H);
                if (s->qkv_bias) PUT(o[S_QKV_B], rows);
                PUT(o[S_WO], H * ((int64_t)s->nq * s->d / T));
            }
            PUT(o[S_LN2], H);
            if (s->family == FAM_DENSE) {
                PUT(o[S_GATE_UP], 2 * (s->I / T) * H);
                PUT(o[S_DOWN], H * (s->I / T));
            } else {
                PUT(o[S_ROUTER], (int64_t)s->E * H);
                if (s->n_shared) {
                    int64_t Is = (int64_t)s->n_shared * s->Ie;
                    PUT(o[S_SH_FC1], 2 * (Is / T) * H);
                    PUT(o[S_SH_FC2], H * (Is / T));
                }
            }
        }
        if (s->has_embeddings && p == c->P - 1) {
            PUT(c->final_ln_off, H);
            if (!c->tied) PUT(c->lm_head_off, c->Vp / T * H);
            else if (c->P > 1) PUT(c->emb_tied_off, c->Vp / T * H);
        }
        c->dense_bytes[p] = up256(off);
        if (c->moe) {
            off = 0;
            int64_t Ie = s->Ie / c->Y, El = c->El; /* Ie: the expert width one buffer holds */
            for (int at = c->first[p]; at < c->first[p + 1]; at++) {
                int ly = c->order[at];
                int64_t *o = c->eoff + (size_t)ly * El * 2;
                if (l->kind == K_GEN || c->grouped) {
                    PUT(o[0], El * 2 * Ie * H);
                    PUT(o[1], El * Ie * H);
                } else {
                    for (int64_t j = 0; j < El; j++) {
                        PUT(o[2 * j], 2 * Ie * H);
                        PUT(o[2 * j + 1], H * Ie);
                    }
                }
            }
            c->expert_bytes[p] = up256(off);
        }
#undef PUT
    }
    return 0;
}

static int buf_used(const ctx_t *c, int b)
{
    if (b < c->nd) return c->l.tp_filter < 0 || b % c->T == c->l.tp_filter;
    int x = (b - c->nd) / c->Y % c->X, y = (b - c->nd) % c->Y;
    return (c->l.ep_filter < 0 || x == c->l.ep_filter) && (c->Y == 1 || c->l.tp_filter < 0 || y == c->l.tp_filter);
}

/*
 * Source lookup: logical element (r, col) of tensor `tid` -> buffer, byte
 * offset, and the number of columns from `col` on that are contiguous there.
 * Replicated tensors are read from tensor rank 0 of the owning stage.
 */
static void src_find(const ctx_t *c, int tid, int ly, int ex, int64_t r, int64_t col,
                     int *buf, int64_t *off, int64_t *run)
{
    const orc_spec *s = &c->s;
    const int64_t H = s->H, T = c->T, eb = c->eb;
    int p = tid == T_EMB ? 0 : (tid == T_FINAL_LN || tid == T_LM_HEAD) ? c->P - 1 : c->stage_of[ly];
    const int64_t *o = ly >= 0 ? c->doff + (size_t)ly * NSLOT : NULL;
    int64_t t = 0, e = 0, ncols = H;
    switch (tid) {
    case T_EMB: case T_LM_HEAD: {
        int64_t n = c->Vp / T; /* rows per rank, padding rows included */
        t = r / n;
        e = (tid == T_EMB ? c->emb_off : c->lm_head_off) / eb + (r % n) * H + col;
        break;
    }
    case T_FINAL_LN: e = c->final_ln_off / eb + col; break;
    case T_LN1: e = o[S_LN1] / eb + col; break;
    case T_LN2: e = o[S_LN2] / eb + col; break;
    case T_ROUTER: e = o[S_ROUTER] / eb + r * H + col; break;
    case T_QA: e = o[S_QA] / eb + r * H + col; break;
    case T_KVA: e = o[S_KVA] / eb + r * H + col; break;
    case T_QA_LN: ncols = s->q_lora; e = o[S_QA_LN] / eb + col; break;
    case T_KVA_LN: ncols = s->kv_lora; e = o[S_KVA_LN] / eb + col; break;
    case T_WQ: case T_WK: case T_WV: case T_BQ: case T_BK: case T_BV: {
        int bias = tid == T_BQ || tid == T_BK || tid == T_BV;
        int isq = tid == T_WQ || tid == T_BQ, isk = tid == T_WK || tid == T_BK;
        int64_t g = s->nq / s->nkv, d = s->d, row;
        if (T > s->nkv) {
            /* one replicated KV head per rank: read the copy on the lowest rank holding it */
            int64_t rep = T / s->nkv, hq = s->nq / T;
            if (isq) { t = r / (hq * d); row = r % (hq * d); }
            else { t = (r / d) * rep; row = hq * d + r % d + (isk ? 0 : d); }
        } else if (c->l.kind == K_TRAIN) {
            int64_t per = s->nkv / T, G, w;
            if (isq) { G = r / (g * d); w = r % (g * d); }
            else { G = r / d; w = r % d; w += isk ? g * d : (g + 1) * d; }
            t = G / per;
            row = (G % per) * (g + 2) * d + w;
        } else {
            int64_t nql = (int64_t)s->nq * d / T, nkl = (int64_t)s->nkv * d / T;
            if (isq) { t = r / nql; row = r % nql; }
            else { t = r / nkl; row = nql + r % nkl + (isk ? 0 : nkl); }
        }
        ncols = bias ? 1 : H;
        e = o[bias ? S_QKV_B : S_QKV_W] / eb + row * ncols + col;
        break;
    }
    case T_WO: {
        int64_t wid = (int64_t)s->nq * (s->family == FAM_MLA ? s->v_dim : s->d), n = wid / T;
        t = col / n;
        e = o[S_WO] / eb + r * n + col % n;
        *run = n - col % n;
        goto done;
    }
    case T_GATE: case T_UP: case T_SH_GATE: case T_SH_UP: {
        int sh = tid == T_SH_GATE || tid == T_SH_UP;
        int64_t wid = sh ? (int64_t)s->n_shared * s->Ie : s->I, n = wid / T;
        int64_t row = r % n + ((tid == T_UP || tid == T_SH_UP) ? n : 0);
        t = r / n;
        e = o[sh ? S_SH_FC1 : S_GATE_UP] / eb + row * H + col;
        break;
    }
    case T_DOWN: case T_SH_DOWN: {
        int sh = tid == T_SH_DOWN;
        int64_t wid = sh ? (int64_t)s->n_shared * s->Ie : s->I, n = wid / T;
        t = col / n;
        e = o[sh ? S_SH_FC2 : S_DOWN] / eb + r * n + col % n;
        *run = n - col % n;
        goto done;
    }
    case T_QB: case T_KVB: {
        int64_t per_head = s->nope + (tid == T_QB ? s->rope : s->v_dim);
        int64_t n = s->nq / T * per_head;
        ncols = tid == T_QB ? s->q_lora : s->kv_lora;
        t = r / n;
        e = o[tid == T_QB ? S_QB : S_KVB] / eb + (r % n) * ncols + col;
        break;
    }
    case T_EX_GATE: case T_EX_UP: case T_EX_DOWN: {
        /* n: the expert width one buffer holds; gate/up rows and down columns are split over Y ranks */
        int64_t n = s->Ie / c->Y, El = c->El, x = ex / El, j = ex % El, y, rl = r, cl = col;
        const int64_t *eo = c->eoff + (size_t)ly * El * 2;
        if (tid == T_EX_DOWN) { y = col / n; cl = col % n; } else { y = r / n; rl = r % n; }
        int64_t upo = tid == T_EX_UP ? n : 0;
        *buf = c->nd + (p * c->X + (int)x) * c->Y + (int)y;
        if (c->l.kind == K_GEN) {
            if (tid == T_EX_DOWN) { *off = eo[1] + ((j * H + rl) * n + cl) * eb; *run = n - cl; }
            else { *off = eo[0] + ((j * 2 * n + upo + rl) * H + cl) * eb; *run = H - cl; }
        } else if (c->grouped) {
            if (tid == T_EX_DOWN) *off = eo[1] + ((j * n + cl) * H + rl) * eb;
            else *off = eo[0] + ((j * H + cl) * 2 * n + upo + rl) * eb;
            *run = 1;
        } else {
            if (tid == T_EX_DOWN) { *off = eo[2 * j + 1] + (rl * n + cl) * eb; *run = n - cl; }
            else { *off = eo[2 * j] + ((upo + rl) * H + cl) * eb; *run = H - cl; }
        }
        return;
    }
    default: abort();
    }
    *run = ncols - col;
done:
    *buf = p * c->T + (int)t;
    *off = e * eb;
}

/* One rectangular piece of a logical tensor and where it goes in a destination buffer. */
typedef struct {
    int tid, ly, ex;
    int64_t r0, nr, c0, nc;
    int dbuf;
    int64_t doff; /* byte offset of element (r0, c0) */
    int64_t ld;   /* elements between consecutive rows (or consecutive columns if transposed) */
    int transposed;
} piece_t;

typedef struct { piece_t *v; size_t n, cap; } pieces_t;

static void add_piece(pieces_t *ps, int tid, int ly, int ex, int64_t r0, int64_t nr, int64_t c0,
                      int64_t nc, int dbuf, int64_t doff, int64_t ld, int tr)
{
    if (ps->n == ps->cap) {
        ps->cap = ps->cap ? ps->cap * 2 : 1024;
        ps->v = realloc(ps->v, ps->cap * sizeof(piece_t));
    }
    piece_t q = { tid, ly, ex, r0, nr, c0, nc, dbuf, doff, ld, tr };
    ps->v[ps->n++] = q;
}

/* Fill one piece: row by row, run by run. */
static void fill_piece(const ctx_t *S, const piece_t *q, const void *const *src, void *const *dst,
                       int64_t eb)
{
    char *dbase = (char *)dst[q->dbuf] + q->doff;
    for (int64_t i = 0; i < q->nr; i++) {
        int64_t r = q->r0 + i, k = 0;
        while (k < q->nc) {
            int sb; int64_t so, run;
            src_find(S, q->tid, q->ly, q->ex, r, q->c0 + k, &sb, &so, &run);
            const char *sp = (const char *)src[sb] + so;
            if (q->transposed) {
                memcpy(dbase + (k * q->ld + i) * eb, sp, eb);
                k += 1;
            } else {
                int64_t n = run < q->nc - k ? run : q->nc - k;
                memcpy(dbase + (i * q->ld + k) * eb, sp, n * eb);
                k += n;
            }
        }
    }
}

/* Enumerate the pieces that make up every used destination buffer, in storage order. */
static void dst_pieces(const ctx_t *D, pieces_t *ps)
{
    const orc_spec *s = &D->s;
    const int64_t H = s->H, T = D->T, eb = D->eb;
    for (int b = 0; b < D->nd; b++) {
        if (!buf_used(D, b)) continue;
        int p = b / D->T;
        int64_t t = b % D->T;
        /* real vocabulary rows of this rank: the shard minus padding rows (possibly none) */
        int64_t vn = D->Vp / T, vreal = s->V - t * vn < vn ? s->V - t * vn : vn;
        if (s->has_embeddings && p == 0 && vreal > 0)
            add_piece(ps, T_EMB, -1, -1, t * vn, vreal, 0, H, b, D->emb_off, H, 0);
        for (int at = D->first[p]; at < D->first[p + 1]; at++) {
            int ly = D->order[at];
            const int64_t *o = D->doff + (size_t)ly * NSLOT;
            add_piece(ps, T_LN1, ly, -1, 0, 1, 0, H, b, o[S_LN1], H, 0);
            if (s->family == FAM_MLA) {
                int64_t nql = s->nq / T;
                int64_t nqb = nql * (s->nope + s->rope), nkb = nql * (s->nope + s->v_dim);
                int64_t now = nql * s->v_dim;
                add_piece(ps, T_QA, ly, -1, 0, s->q_lora, 0, H, b, o[S_QA], H, 0);
                add_piece(ps, T_QA_LN, ly, -1, 0, 1, 0, s->q_lora, b, o[S_QA_LN], s->q_lora, 0);
                add_piece(ps, T_QB, ly, -1, t * nqb, nqb, 0, s->q_lora, b, o[S_QB], s->q_lora, 0);
                add_piece(ps, T_KVA, ly, -1, 0, s->kv_lora + s->rope, 0, H, b, o[S_KVA], H, 0);
                add_piece(ps, T_KVA_LN, ly, -1, 0, 1, 0, s->kv_lora, b, o[S_KVA_LN], s->kv_lora, 0);
                add_piece(ps, T_KVB, ly, -1, t * nkb, nkb, 0, s->kv_lora, b, o[S_KVB], s->kv_lora, 0);
                add_piece(ps, T_WO, ly, -1, 0, H, t * now, now, b, o[S_WO], now, 0);
            } else {
                int64_t g = s->nq / s->nkv, d = s->d;
                for (int bias = 0; bias <= (s->qkv_bias ? 1 : 0); bias++) {
                    int64_t w = bias ? 1 : H, base = o[bias ? S_QKV_B : S_QKV_W];
                    int tq = bias ? T_BQ : T_WQ, tk = bias ? T_BK : T_WK, tv = bias ? T_BV : T_WV;
                    if (T > s->nkv) {
                        /* this rank's query heads, then the KV head it shares with T/nkv - 1 others */
                        int64_t rep = T / s->nkv, hq = s->nq / T, kvh = t / rep;
                        add_piece(ps, tq, ly, -1, t * hq * d, hq * d, 0, w, b, base, w, 0);
                        add_piece(ps, tk, ly, -1, kvh * d, d, 0, w, b, base + hq * d * w * eb, w, 0);
                        add_piece(ps, tv, ly, -1, kvh * d, d, 0, w, b, base + (hq + 1) * d * w * eb, w, 0);
                    } else if (D->l.kind == K_TRAIN) {
                        int64_t per = s->nkv / T;
                        for (int64_t j = 0; j < per; j++) {
                            int64_t G = t * per + j, row = j * (g + 2) * d;
                            add_piece(ps, tq, ly, -1, G * g * d, g * d, 0, w, b, base + row * w * eb, w, 0);
                            add_piece(ps, tk, ly, -1, G * d, d, 0, w, b, base + (row + g * d) * w * eb, w, 0);
                            add_piece(ps, tv, ly, -1, G * d, d, 0, w, b, base + (row + (g + 1) * d) * w * eb, w, 0);
                        }
                    } else {
                        int64_t nql = (int64_t)s->nq * d / T, nkl = (int64_t)s->nkv * d / T;
                        add_piece(ps, tq, ly, -1, t * nql, nql, 0, w, b, base, w, 0);
                        add_piece(ps, tk, ly, -1, t * nkl, nkl, 0, w, b, base + nql * w * eb, w, 0);
                        add_piece(ps, tv, ly, -1, t * nkl, nkl, 0, w, b, base + (nql + nkl) * w * eb, w, 0);
                    }
                }
                int64_t now = (int64_t)s->nq * d / T;
                add_piece(ps, T_WO, ly, -1, 0, H, t * now, now, b, o[S_WO], now, 0);
            }
            add_piece(ps, T_LN2, ly, -1, 0, 1, 0, H, b, o[S_LN2], H, 0);
            if (s->family == FAM_DENSE) {
                int64_t n = s->I / T;
                add_piece(ps, T_GATE, ly, -1, t * n, n, 0, H, b, o[S_GATE_UP], H, 0);
                add_piece(ps, T_UP, ly, -1, t * n, n, 0, H, b, o[S_GATE_UP] + n * H * eb, H, 0);
                add_piece(ps, T_DOWN, ly, -1, 0, H, t * n, n, b, o[S_DOWN], n, 0);
            } else {
                add_piece(ps, T_ROUTER, ly, -1, 0, s->E, 0, H, b, o[S_ROUTER], H, 0);
                if (s->n_shared) {
                    int64_t n = (int64_t)s->n_shared * s->Ie / T;
                    add_piece(ps, T_SH_GATE, ly, -1, t * n, n, 0, H, b, o[S_SH_FC1], H, 0);
                    add_piece(ps, T_SH_UP, ly, -1, t * n, n, 0, H, b, o[S_SH_FC1] + n * H * eb, H, 0);
                    add_piece(ps, T_SH_DOWN, ly, -1, 0, H, t * n, n, b, o[S_SH_FC2], n, 0);
                }
            }
        }
        if (s->has_embeddings && p == D->P - 1) {
            add_piece(ps, T_FINAL_LN, -1, -1, 0, 1, 0, H, b, D->final_ln_off, H, 0);
            if (vreal > 0) {
                if (!D->tied) add_piece(ps, T_LM_HEAD, -1, -1, t * vn, vreal, 0, H, b, D->lm_head_off, H, 0);
                else if (D->P > 1) add_piece(ps, T_EMB, -1, -1, t * vn, vreal, 0, H, b, D->emb_tied_off, H, 0);
            }
        }
    }
    for (int b = D->nd; b < D->nd + D->ne; b++) {
        if (!buf_used(D, b)) continue;
        int p = (b - D->nd) / (D->X * D->Y);
        int64_t x = (b - D->nd) / D->Y % D->X, y = (b - D->nd) % D->Y;
        int64_t n = s->Ie / D->Y, El = D->El; /* this buffer holds rows / columns y*n .. of every local expert */
        for (int at = D->first[p]; at < D->first[p + 1]; at++) {
            int ly = D->order[at];
            const int64_t *eo = D->eoff + (size_t)ly * El * 2;
            for (int64_t j = 0; j < El; j++) {
                int ex = (int)(x * El + j);
                if (D->l.kind == K_GEN) {
                    int64_t b13 = eo[0] + j * 2 * n * H * eb;
                    add_piece(ps, T_EX_GATE, ly, ex, y * n, n, 0, H, b, b13, H, 0);
                    add_piece(ps, T_EX_UP, ly, ex, y * n, n, 0, H, b, b13 + n * H * eb, H, 0);
                    add_piece(ps, T_EX_DOWN, ly, ex, 0, H, y * n, n, b, eo[1] + j * H * n * eb, n, 0);
                } else if (D->grouped) {
                    int64_t b1 = eo[0] + j * H * 2 * n * eb;
                    add_piece(ps, T_EX_GATE, ly, ex, y * n, n, 0, H, b, b1, 2 * n, 1);
                    add_piece(ps, T_EX_UP, ly, ex, y * n, n, 0, H, b, b1 + n * eb, 2 * n, 1);
                    add_piece(ps, T_EX_DOWN, ly, ex, 0, H, y * n, n, b, eo[1] + j * n * H * eb, H, 1);
                } else {
                    add_piece(ps, T_EX_GATE, ly, ex, y * n, n, 0, H, b, eo[2 * j], H, 0);
                    add_piece(ps, T_EX_UP, ly, ex, y * n, n, 0, H, b, eo[2 * j] + n * H * eb, H, 0);
                    add_piece(ps, T_EX_DOWN, ly, ex, 0, H, y * n, n, b, eo[2 * j + 1], n, 0);
                }
            }
        }
    }
}

/* ------------------------------------------------------------------ API -- */

int orc_num_bufs(const orc_spec *s, const orc_layout *l)
{
    ctx_t c;
    if (ctx_init(&c, s, l)) return -1;
    int n = c.nd + c.ne;
    ctx_free(&c);
    return n;
}

int64_t orc_buf_bytes(const orc_spec *s, const orc_layout *l, int i)
{
    ctx_t c;
    if (ctx_init(&c, s, l)) return -1;
    int64_t n = -1;
    if (i >= 0 && i < c.nd) n = c.dense_bytes[i / c.T];
    else if (i >= c.nd && i < c.nd + c.ne) n = c.expert_bytes[(i - c.nd) / (c.X * c.Y)];
    ctx_free(&c);
    return n;
}

int orc_buf_used(const orc_spec *s, const orc_layout *l, int i)
{
    ctx_t c;
    if (ctx_init(&c, s, l)) return -1;
    int u = (i >= 0 && i < c.nd + c.ne) ? buf_used(&c, i) : -1;
    ctx_free(&c);
    return u;
}

/*
 * Fill every used destination buffer from the source buffers.  Pieces larger
 * than `chunk_rows` rows are cut by rows so threads share the work evenly.
 * Returns 0, or -1 for an invalid spec/layout pair.  total_bytes (optional)
 * receives the number of destination bytes written.
 */
int orc_reshard(const orc_spec *s, const orc_layout *sl, const orc_layout *dl,
                const void *const *src, void *const *dst, int nthreads, int64_t *total_bytes)
{
    ctx_t S, D;
    if (sl->tp_filter >= 0 || sl->ep_filter >= 0) return -1;
    if (ctx_init(&S, s, sl)) return -1;
    if (ctx_init(&D, s, dl)) { ctx_free(&S); return -1; }
    pieces_t ps = { 0, 0, 0 }, cut = { 0, 0, 0 };
    dst_pieces(&D, &ps);
    const int64_t eb = S.eb, target = 1 << 20; /* about 1 MiB of elements per work item */
    int64_t bytes = 0;
    for (size_t i = 0; i < ps.n; i++) {
        piece_t q = ps.v[i];
        bytes += q.nr * q.nc * eb;
        int64_t rows = target / (q.nc > 0 ? q.nc : 1);
        if (rows < 1) rows = 1;
        for (int64_t r = 0; r < q.nr; r += rows) {
            int64_t n = q.nr - r < rows ? q.nr - r : rows;
            int64_t doff = q.doff + (q.transposed ? r : r * q.ld) * eb;
            add_piece(&cut, q.tid, q.ly, q.ex, q.r0 + r, n, q.c0, q.nc, q.dbuf, doff, q.ld, q.transposed);
        }
    }
    if (nthreads < 1) nthreads = 1;
    long n = (long)cut.n;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads)
    for (long i = 0; i < n; i++) fill_piece(&S, &cut.v[i], src, dst, eb);
    if (total_bytes) *total_bytes = bytes;
    free(ps.v); free(cut.v);
    ctx_free(&S); ctx_free(&D);
    return 0;
}

int orc_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
