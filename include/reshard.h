/*
 * reshard.h - C ABI of the MI355X weight-resharding library.
 *
 * Scope: the on-device part of the resharding flow of MindSpeed RL (paper
 * sections "Allgather-Swap Technique" and "Problem Statement", redundant-memory
 * example).  After an actor update the training-layout weight shards (already
 * gathered in HBM: step 1 of the technique) are repacked into the generation
 * engine's layout at a different tensor/expert-parallel degree (step 2: slice
 * selection and copy), the training-side buffers are swapped to pinned host memory so
 * their HBM can be released for generation (step 3, device-to-host), and swapped
 * back before the next update (host-to-device) instead of resharding again.
 *
 * Conventions shared by every call
 *   - All pointers named *_ptrs / spec / layout / out are HOST pointers.  The
 *     entries of src_ptrs[] / dst_ptrs[] are DEVICE pointers owned by the caller.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   - Every function returns RESHARD_OK (0) or a negative RESHARD_ERR_* code and
 *     never throws.  reshard_last_error() returns a thread-local message for the
 *     last failing call on the calling thread.
 *   - A plan is not thread-safe: calls on one plan must be serialised by the
 *     caller.  Different plans are independent.
 *
 * Layouts (the paper prints none; these are the Megatron-style conventions this
 * library fixes).  Logical matrices are row-major [out, in]; elements are
 * opaque words of elem_bytes bytes (2 for bf16) and are moved bit for bit.
 *   Buffers.  A layout with tensor-parallel degree T, pipeline degree P and
 *   expert-parallel degree X owns P*T "dense" buffers, index p*T + t, followed
 *   (MoE families) by P*X "expert" buffers, index P*T + p*X + x.  Replicas along
 *   data parallelism are not represented.  Every stored tensor starts on a
 *   256-byte boundary; gap bytes are never read or written.
 *   Dense buffer (p, t), in order: [embedding rows t*V/T..] (stage 0 only); per
 *   layer of the stage: ln1, attention block, ln2, feed-forward block;
 *   [final_ln, lm_head rows t*V/T..] (last stage only).
 *     attention, GQA families: qkv weight, [qkv bias], o_proj columns
 *       t*nq*d/T.. stored [H, nq*d/T].  TRAIN qkv: rank t owns KV groups
 *       t*nkv/T.. ; each group is stored as its nq/nkv query heads, then its key
 *       head, then its value head.  GEN qkv: rank t stores its query rows, then
 *       its key rows, then its value rows.
 *     attention, MLA family: q_a, q_a_ln, q_b (rows of heads t*nq/T..), kv_a,
 *       kv_a_ln, kv_b (rows of heads t*nq/T..), o_proj columns t*nq*v_dim/T.. .
 *     feed-forward, dense family: gate_up = gate rows t*I/T.. then up rows of the
 *       same range; down = columns t*I/T.. stored [H, I/T].
 *     feed-forward, MoE families: router [E, H] (replicated); if n_shared > 0 the
 *       shared expert of width n_shared*Ie as fused gate_up and down, split like
 *       the dense feed-forward.
 *     fewer KV heads than tensor ranks (T a multiple of nkv), both kinds: rank t
 *       stores its nq/T query heads, then KV head t / (T/nkv): each KV head is
 *       replicated on T/nkv ranks.
 *   Replicated ("common") tensors: ln1, ln2, final_ln, router, q_a, q_a_ln, kv_a,
 *     kv_a_ln.  They are READ from tensor rank 0 of the owning stage and WRITTEN
 *     to every destination tensor rank.  Likewise a replicated KV head is read from
 *     the lowest rank holding it, a tied embedding from the first stage.
 *   Pipeline stages hold contiguous, equal blocks of layers unless the layout asks
 *     for interleaved chunks (vpp) or an uneven first / last stage.
 *   Expert buffer (p, x) holds whole experts x*E/X .. (unless etp > 1, see reshard_layout:
 *   then buffer (p, x, y) holds gate/up rows and down columns y*Ie/etp.. of each of them, and
 *   Ie below reads Ie/etp), per layer of the stage:
 *     TRAIN, RESHARD_PER_EXPERT: for each local expert fc1 = [gate; up] stored
 *       [2*Ie, H], then fc2 = down stored [H, Ie].
 *     TRAIN, RESHARD_GROUPED (grouped-matmul orientation): w1[E/X][H][2*Ie] with
 *       w1[e][h][c] = (c < Ie ? gate_e[c][h] : up_e[c-Ie][h]), then
 *       w2[E/X][Ie][H] with w2[e][i][h] = down_e[h][i].
 *     GEN: w13[E/X][2*Ie][H] (gate rows then up rows), then w2[E/X][H][Ie].
 */
#ifndef RESHARD_H
#define RESHARD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct reshard_plan reshard_plan;

enum {
    RESHARD_OK = 0,
    RESHARD_ERR_INVALID_ARG = -1, /* NULL/misaligned pointer, bad struct_size, bad index */
    RESHARD_ERR_UNSUPPORTED = -2, /* shape not divisible by a degree, too many buffers */
    RESHARD_ERR_OOM = -3,         /* host or device allocation for the plan failed */
    RESHARD_ERR_HOST_OOM = -4,    /* pinned host memory for the swap could not be allocated */
    RESHARD_ERR_BAD_STATE = -5,   /* call not allowed in the plan's current swap state */
    RESHARD_ERR_HIP = -6          /* a HIP runtime call failed; message has the HIP error */
};

enum { RESHARD_DENSE_GQA = 0, RESHARD_MOE_GQA = 1, RESHARD_MOE_MLA = 2 };
enum { RESHARD_TRAIN = 0, RESHARD_GEN = 1 };
enum { RESHARD_PER_EXPERT = 0, RESHARD_GROUPED = 1 };

/* Shape of the model whose weights are resharded.  Set struct_size = sizeof. */
typedef struct reshard_model_spec {
    uint32_t struct_size;
    int32_t family;         /* RESHARD_DENSE_GQA / MOE_GQA / MOE_MLA */
    int32_t L, H;           /* decoder layers, hidden size */
    int32_t nq, nkv, d;     /* query heads, KV heads, head dim (GQA families) */
    int32_t I;              /* dense feed-forward width (dense family) */
    int32_t V;              /* vocabulary rows (when has_embeddings) */
    int32_t qkv_bias;       /* 1: fused qkv bias present (GQA families) */
    int32_t has_embeddings; /* 1: embedding, final norm and lm_head present (untied) */
    int32_t E, Ie;          /* routed experts per layer, expert feed-forward width */
    int32_t n_shared;       /* shared experts (0 = none); shared width = n_shared*Ie */
    int32_t q_lora, kv_lora, nope, rope, v_dim; /* MLA family */
    int32_t elem_bytes;     /* bytes per weight element: 1, 2, 4 or 8 */
    int32_t tied_embeddings; /* 1: no lm_head; a TRAIN layout with pp > 1 keeps a copy of the
                                embedding shard on its last stage (after final_ln) */
} reshard_model_spec;

/* One side of the resharding.  Set struct_size = sizeof. */
typedef struct reshard_layout {
    uint32_t struct_size;
    int32_t kind;           /* RESHARD_TRAIN or RESHARD_GEN (GEN requires pp == 1) */
    int32_t tp, pp, ep;     /* degrees, each >= 1 (ep must be 1 for the dense family) */
    int32_t expert_layout;  /* TRAIN only: RESHARD_PER_EXPERT or RESHARD_GROUPED */
    int32_t tp_rank_filter; /* destination only: keep this tensor rank's dense buffers (-1 = all) */
    int32_t ep_rank_filter; /* destination only: keep this expert rank's buffers (-1 = all) */
    int32_t vpp;            /* virtual pipeline size (0 or 1 = none): layers are cut into pp*vpp
                               chunks, chunk c lives on stage c mod pp, stored in chunk order */
    int32_t first_stage_layers; /* uneven pipeline split: layers on the first stage (0 = even) */
    int32_t last_stage_layers;  /* ... and on the last; the stages between share the rest evenly */
    int32_t vocab_padded;   /* rows the embedding / lm_head are padded to before the tensor-parallel
                               split (0 = V; else >= V and divisible by tp).  Rank t stores
                               vocab_padded/tp rows; rows at or beyond V are padding: never read, never
                               written */
    int32_t etp;            /* expert tensor parallelism: 0 or 1 = whole experts; tp = every expert is
                               split over the tensor ranks like a dense feed-forward.  Expert buffers
                               are then indexed P*T + (p*X + x)*etp + y, and tp_rank_filter also
                               selects y */
} reshard_layout;

/* Weight classes of the paper's redundant-memory example (Problem Statement): tensor-parallel
 * weights T, expert-parallel weights E, common (replicated) weights C. */
enum { RESHARD_CLASS_TP = 0, RESHARD_CLASS_EP = 1, RESHARD_CLASS_COMMON = 2 };

/* One stored tensor of a layout (for loading weights into / reading them out of the buffers). */
typedef struct reshard_tensor_info {
    char name[24];          /* "ln1", "qkv_w", "qkv_b", "wo", "gate_up", "down", "fc1", "w13", ... */
    int32_t layer;          /* -1 for embedding / final norm / lm_head */
    int32_t expert;         /* global expert index of a per-expert tensor, else -1 */
    int32_t buffer;         /* index into src_ptrs / dst_ptrs */
    int32_t replicated;     /* 1 for a common (replicated) tensor or a never-read copy */
    int64_t offset, bytes;  /* placement inside the buffer */
    int32_t weight_class;   /* RESHARD_CLASS_TP / EP / COMMON */
    int32_t reserved_;
} reshard_tensor_info;

/*
 * One copy descriptor of a plan (host-side view, for inspection and tests).
 * kind 0 (strided copy): for i in [0, rows):
 *     memcpy(dst + dst_off + i*dst_stride, src + src_off + i*src_stride, row_bytes)
 * kind 1 (transposing copy of elem_bytes words): for i in [0, rows), k in [0, row_bytes/elem_bytes):
 *     dst[dst_off + k*dst_stride + i*elem_bytes] = src[src_off + i*src_stride + k*elem_bytes]
 * All offsets and strides are bytes.
 */
typedef struct reshard_desc {
    int32_t src_buf, dst_buf;
    int32_t kind, elem_bytes;
    int64_t src_off, dst_off;
    int64_t rows, row_bytes;
    int64_t src_stride, dst_stride;
} reshard_desc;

/*
 * One device work item (host-side view of the tile table, for inspection and tests).
 * kind 0: `rows` rows of `row_units` vectors of `vec_bytes` bytes each, row pitches as given.
 * kind 1: transposing tile of `rows` source rows x `row_units` elements of `vec_bytes` bytes:
 *     dst[dst_off + k*dst_stride + i*vec_bytes] = src[src_off + i*src_stride + k*vec_bytes]
 * kind 2: gathering tile: `rows` consecutive vectors of `vec_bytes` bytes of the destination, made of
 *     segments of `row_units` vectors taken from `sources` consecutive source buffers in turn
 *     (the shards of a weight split along its rows' direction, merged side by side):
 *     for u in [0, rows): w = phase + u, seg = w / row_units, c = w % row_units,
 *         dst[dst_off + u*vec_bytes] = src(src_buf + seg % sources)[src_off + (seg / sources)*src_stride + c*vec_bytes]
 *     (vec_bytes bytes each; dst_stride is 0).
 * tile_class: 0 copy kernel; 1 register-transpose kernel, a whole tile of the plan's preferred
 * shape; 2 register-transpose kernel, a whole tile of another shape the kernel is built for
 * (rows x row_units says which); 3 generic transpose kernel (at most 64 x 64, any extent).
 * order: some bytes are in the table twice, cut two ways, and an execute launches one of the two:
 *     0 launched by every execute; 1 launched unless the plan gathers; 2 launched only when it
 *     does (the kind 2 tiles).  A plan gathers when its tuning has flags bits 5 and 6 set,
 *     block_threads 1024 and blocks_per_cu 0.  The tiles of order 0 and 1
 *     together, and those of order 0 and 2 together, each write every destination byte exactly once.
 */
typedef struct reshard_tile {
    int32_t src_buf, dst_buf;
    int32_t kind, tile_class;
    int64_t src_off, dst_off;
    int64_t rows, row_units;
    int64_t src_stride, dst_stride;
    int32_t vec_bytes, order;
    int64_t sources, phase; /* kind 2 only (else 1 and 0) */
} reshard_tile;

typedef struct reshard_plan_info {
    int32_t num_src_bufs, num_dst_bufs;
    int64_t num_descs;      /* copy descriptors after merging */
    int64_t num_tiles;      /* records of the tile table (device work items; see reshard_tile.order) */
    int64_t num_transpose_tiles; /* of which transposing tiles (register path + generic path) */
    int64_t bytes_moved;    /* destination bytes written by one execute (== bytes read) */
    int64_t table_bytes;    /* bytes of one copy of the tile table; the plan holds reshard_tuning.table_copies copies
                               (see there) of table_bytes + 256 bytes each on the device once it is prepared */
} reshard_plan_info;

/* Swap / residency state of the source (training-side) buffers of a plan. */
enum {
    RESHARD_SRC_UNBOUND = 0,      /* no source pointers known yet */
    RESHARD_SRC_RESIDENT = 1,     /* bound, valid in HBM */
    RESHARD_SRC_SWAPPING_OUT = 2, /* device-to-host copies in flight */
    RESHARD_SRC_ON_HOST = 3,      /* host copy complete; device copy may be released */
    RESHARD_SRC_RELEASED = 4,     /* caller freed the device copy; rebind before swap-in */
    RESHARD_SRC_SWAPPING_IN = 5,  /* host-to-device copies in flight */
    RESHARD_SRC_MIXED = 6         /* plan level only: the source buffers are in different states (streaming) */
};

/* Byte ledger of a plan (pure host bookkeeping of what the caller told the plan). */
typedef struct reshard_mem_stats_t {
    int64_t src_live;     /* bytes of bound, not released source buffers */
    int64_t dst_live;     /* bytes of bound, not released destination buffers */
    int64_t host_pinned;  /* pinned host bytes the plan currently owns */
    int64_t peak_device;  /* max over time of src_live + dst_live (the plan's own table is in plan_info) */
    int64_t released;     /* bytes of source buffers currently marked released */
    int32_t state;        /* RESHARD_SRC_* */
} reshard_mem_stats_t;

/* Knobs of the repack kernels; zero fields keep the built-in default.  Every plan holds its own
 * copy: tile_bytes and the transposing tile shape decide how the plan's tiles are cut and are fixed
 * at creation, the other fields are the launch shape and may be changed between executes. */
typedef struct reshard_tuning {
    int32_t tile_bytes;     /* bytes of work per tile (power of two, 4 KiB .. 512 KiB; default 32 KiB) */
    int32_t block_threads;  /* 64, 128, 256, 512 or 1024 (default 1024) */
    int32_t blocks_per_cu;  /* 0 (default): one tile per workgroup; n > 0: persistent grid of n per CU */
    int32_t unroll;         /* 16-byte loads in flight per lane: 1, 2, 4 or 8 (default 2) */
    int32_t flags;          /* bit 0: non-temporal loads, bit 1: non-temporal stores, bit 2: workgroup
                               barrier between a tile's load burst and its store burst, bit 3: each XCD
                               walks a contiguous eighth of the tile table, bit 4: the one-tile copy kernel issues
                               its loads at raised wave priority (with bits 0-2 all set), bit 5: woven order for the
                               copy tiles that are one contiguous run: the eight XCDs share every group of 8
                               tiles, 1 KiB apart, instead of walking an eighth of the table each (1024-lane
                               workgroups, two loads per lane whatever `unroll` says; tiles of several pitched
                               rows keep the order bit 3 selects and go out in a launch of their own),
                               bit 6 (with bit 5): where shards are merged side by side, or narrower rows packed
                               out of a wider source, into one contiguous stretch of the destination (rows of
                               at least 1 KiB), that stretch goes out in the woven order as well, as gathered
                               tiles that read the sources in turn, instead of as tiles of pitched rows.
                               Default 127 (all); -1 = none.
                               With unroll 1, 4 or 8 bits 0-2 must be all set or all clear.  A persistent
                               grid moves 2 loads per lane, has no barrier and no raised priority, and its
                               accesses are non-temporal when bits 0 and 1 are both set */
    int32_t transpose_rows; /* shape of a register-transposed tile in elements: source rows ... */
    int32_t transpose_cols; /* ... and source columns; each 64, 128, 192, 256 or 512.  0, or a shape the plan's
                             * element size does not allow (the tile must fit 128 KiB): the default for
                             * that size (1 byte 512 x 256, 2 bytes 256 x 256, 4 bytes 128 x 256, 8 bytes 128 x 128) */
    int32_t tail_pool_percent; /* 0 (default): every XCD walks its whole eighth of the copy tiles.  1..50: that share of
                                  every eighth goes to a pool that the last workgroups of the grid drain in chunks, so
                                  XCDs that finish early take over work of the slower ones (default launch shape only) */
    int32_t tail_chunk_tiles;  /* tiles a pool workgroup takes per fetch, 1..1024 (default 16) */
    int32_t table_copies;      /* copies of the tile table the plan keeps on the device, 1..64; execute number n reads copy
                                  n mod table_copies.  Why: the woven copy kernel runs 3 to 4 % slower when the records it
                                  reads are still in the 256 MB memory-side cache from the execute before, which happens
                                  when executes follow each other with less than that much other cached traffic in
                                  between.  0 (default): as many copies as make 512 MiB of tables, and one for a table
                                  under 16 MiB (32 copies would not get there, and fewer than that buy nothing).  Fixed once the table is on the device (first execute or
                                  prepare); reshard_execute_source and reshard_execute_noalloc read a single copy, and an
                                  execute recorded into a HIP graph reads, at every replay, the copy it was recorded with */
} reshard_tuning;

/* Thread-local message of the last failing call on this thread ("" if none). */
const char *reshard_last_error(void);

/*
 * The process-wide default tuning: plans created afterwards by reshard_plan_create start from a
 * copy of it; existing plans are not affected.  NULL restores the built-in defaults.
 * Returns INVALID_ARG for a value outside the ranges above.
 */
int reshard_set_tuning(const reshard_tuning *t);
int reshard_get_tuning(reshard_tuning *out);

/*
 * Step 2 (slice selection and copy), compile time (host only, no GPU needed): validates the
 * shape against both layouts and compiles the src -> dst mapping into a flat
 * table of copy descriptors, cut into equal-work tiles.  Any (kind, degrees)
 * pair is allowed, so TRAIN -> GEN is the resharding, TRAIN -> TRAIN with equal
 * degrees is the identity and GEN -> TRAIN is the way back.  Rank filters must
 * be -1 on the source.  *out is owned by the library until reshard_plan_destroy.
 * Errors: INVALID_ARG (NULL, struct_size), UNSUPPORTED (divisibility, more than
 * RESHARD_MAX_BUFFERS USED source plus destination buffers, i.e. buffers the plan reads or
 * writes once the destination's rank filters are applied, more than 16384 buffers in one
 * layout, sizes beyond 32-bit strides), OOM.
 */
#define RESHARD_MAX_BUFFERS 384
int reshard_plan_create(const reshard_model_spec *spec, const reshard_layout *src,
                        const reshard_layout *dst, reshard_plan **out);

/*
 * The same with the plan's tuning given explicitly (NULL: the process-wide default; otherwise the
 * non-zero fields of *tuning over the built-in defaults), so that plans with different tile sizes
 * and launch shapes live side by side in one process.
 */
int reshard_plan_create_tuned(const reshard_model_spec *spec, const reshard_layout *src,
                              const reshard_layout *dst, const reshard_tuning *tuning, reshard_plan **out);

/*
 * Changes the launch shape of an existing plan (block_threads, blocks_per_cu, unroll, flags) for the
 * executes issued afterwards; NULL or zero fields select the built-in defaults.  tile_bytes and
 * transpose_rows / transpose_cols must be zero or what the plan was created with (INVALID_ARG
 * otherwise): the tiles are already cut.  reshard_plan_get_tuning reads the plan's copy.
 */
int reshard_plan_set_tuning(reshard_plan *plan, const reshard_tuning *tuning);
int reshard_plan_get_tuning(const reshard_plan *plan, reshard_tuning *out);

/* Frees the plan, its device tile table and its pinned host memory.  Waits for
 * swap copies still in flight.  NULL is allowed. */
int reshard_plan_destroy(reshard_plan *plan);

/* Buffer tables.  side: 0 = source, 1 = destination.  Counts are >= 0; a negative
 * return is an error code.  `used` is 0 for a buffer the plan never touches (its
 * pointer may then be NULL): destination buffers removed by a rank filter, source
 * buffers that no kept destination needs. */
int reshard_plan_num_bufs(const reshard_plan *plan, int side);
int64_t reshard_plan_buf_bytes(const reshard_plan *plan, int side, int index);
int reshard_plan_buf_used(const reshard_plan *plan, int side, int index);

/* Stored-tensor table of one side, in (buffer, offset) order. */
int64_t reshard_plan_num_tensors(const reshard_plan *plan, int side);
int reshard_plan_tensor(const reshard_plan *plan, int side, int64_t index, reshard_tensor_info *out);

/* Bytes one side stores per weight class, over all its buffers (every copy counted):
 * out[RESHARD_CLASS_TP], out[RESHARD_CLASS_EP], out[RESHARD_CLASS_COMMON]. */
int reshard_plan_class_bytes(const reshard_plan *plan, int side, int64_t out[3]);

/*
 * Redundant memory of a resharding WITHOUT the swap (paper Eq. 3, Problem Statement):
 *   R = GDP * (TW / UTP + EW / GEP)
 * with GDP / GEP the generation-side DP and EP sizes, UTP the update-side TP size, TW / EW
 * the total bytes of the tensor-parallel and expert-parallel weights.  Pure arithmetic;
 * returns -1 for a non-positive degree.
 */
double reshard_redundant_memory_bytes(int gen_dp, double tp_weight_bytes, int update_tp,
                                      double ep_weight_bytes, int gen_ep);

/* Plan statistics and the descriptor table (copied into caller memory). */
int reshard_plan_get_info(const reshard_plan *plan, reshard_plan_info *out);
int reshard_plan_desc(const reshard_plan *plan, int64_t index, reshard_desc *out);
/* Record `index` of the tile table, in table order (0 <= index < num_tiles): the copy tiles (tiles of
 * pitched rows, then contiguous runs, then gathered tiles), then the transposing tiles by shape.
 * See reshard_tile.order for which records an execute launches. */
int reshard_plan_tile(const reshard_plan *plan, int64_t index, reshard_tile *out);

/*
 * Step 2 (slice selection and copy), run time: asynchronous kernel launches on `stream` (one for the
 * copy tiles of several pitched rows, one for the contiguous runs, one for the gathered tiles, one
 * per transposing tile shape in use, each only where the plan has such tiles; three or fewer for
 * most plans, a dozen at most) that fill every used destination buffer from the source buffers.
 * src_ptrs[num_src_bufs], dst_ptrs[num_dst_bufs]: device pointers, each aligned to
 * 256 bytes and at least buf_bytes long; NULL allowed only where used == 0.  The
 * two sets must not overlap.  The memory stays caller-owned and must remain valid
 * until `stream` has run the launch.  On the first call the tile table is uploaded
 * to device memory owned by the plan (a synchronous copy).  Remembers both pointer
 * sets for the swap calls and the ledger (source state becomes RESIDENT).  Also
 * allowed while a swap-out of the same source pointers is in flight (state stays
 * SWAPPING_OUT): both only read the sources.
 * Errors: INVALID_ARG, BAD_STATE (sources are on the host, released, or being
 * swapped in), OOM, HIP.
 */
int reshard_execute(reshard_plan *plan, const void *const *src_ptrs, void *const *dst_ptrs,
                    void *stream);

/*
 * For callers that cannot allocate device memory (set-up code of a HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): reshard_execute with the kernels' tile table in a
 * static device array of RESHARD_STATIC_TABLE_BYTES (32 MiB = 699,050 tiles; each GPU the library
 * runs on holds that array until the process ends) instead of device memory owned by the plan.
 * The call, and everything it calls, allocates and frees nothing: no hipMalloc, no hipFree, no
 * pinned memory.  Arguments, checks, launches, state changes and results are those of
 * reshard_execute; inputs and outputs stay caller-owned.
 * The array is shared by every plan on that GPU and keeps the last call's table: when it does not
 * already hold this plan's table (the first call for the plan, or another plan has used it since),
 * the table is copied there from the plan's host memory with hipMemcpyAsync on `stream`, ahead of
 * the kernels; later calls for the same plan are kernel launches only.  Calls for DIFFERENT plans
 * that overlap on one GPU (other streams, other threads) race for the array: serialise them, e.g. by
 * issuing them on one stream.
 * Errors: those of reshard_execute, and UNSUPPORTED when the plan's table_bytes (reshard_plan_info)
 * exceed RESHARD_STATIC_TABLE_BYTES: cut the plan into larger tiles (tile_bytes of
 * reshard_plan_create_tuned) or use reshard_execute.
 */
#define RESHARD_STATIC_TABLE_BYTES (32u << 20)
int reshard_execute_noalloc(reshard_plan *plan, const void *const *src_ptrs, void *const *dst_ptrs,
                            void *stream);

/*
 * Optional: uploads the tile table to the current device now (hipMalloc + a
 * synchronous copy) instead of inside the first reshard_execute.  After it, an
 * execute is kernel launches only: no allocation, no copy, no synchronisation, so
 * it may be recorded into a HIP graph (the pointer sets are baked into the
 * recorded launches).  Errors: OOM, HIP.
 */
int reshard_plan_prepare(reshard_plan *plan);

/*
 * Streaming form of the repack, for callers that never hold all source buffers at once (the
 * gathered shards arrive, are repacked and are swapped out or dropped one buffer at a time, so
 * the peak is the destination plus the buffers in flight instead of source plus destination):
 * runs the part of the plan that READS source buffer `src_index` (device pointer `src_ptr`,
 * 256-byte aligned) and writes into dst_ptrs (all used destination buffers must be given every
 * time).  After it has been called once for every used source buffer the destination is
 * complete and bit-identical to one reshard_execute.  The first call uploads a second copy of
 * the tile table, regrouped by source buffer.  The buffer becomes RESIDENT; the plan-level
 * state is RESHARD_SRC_MIXED while buffers differ.
 * Errors: INVALID_ARG, BAD_STATE (this buffer is swapped out / in flight), OOM, HIP.
 */
int reshard_execute_source(reshard_plan *plan, int src_index, const void *src_ptr, void *const *dst_ptrs,
                           void *stream);

/* Per-buffer forms of swap-out and release for the streaming flow.  reshard_swap_out_source needs
 * the buffer RESIDENT (-> SWAPPING_OUT; complete it with reshard_swap_wait_buffer(host_wait = 1) or
 * reshard_swap_wait); reshard_mark_src_buffer_released needs it ON_HOST (-> RELEASED).  When every
 * used buffer is RELEASED the plan is RELEASED and continues with reshard_bind_src / reshard_swap_in. */
int reshard_swap_out_source(reshard_plan *plan, int src_index, void *stream);
int reshard_mark_src_buffer_released(reshard_plan *plan, int src_index);
/* Per-buffer swap-in (the host-to-device copy "in advance", one buffer at a time, so the trainer's
 * memory can come back stage by stage): the buffer must be ON_HOST or RELEASED.  `src_ptr` is its
 * new device home (256-byte aligned); NULL keeps the pointer still bound (ON_HOST only).  The copy
 * is ordered after work already queued on `stream`, and `stream` waits for it; the buffer becomes
 * SWAPPING_IN (complete it with reshard_swap_wait_buffer(host_wait = 1) or reshard_swap_wait).
 * Errors: INVALID_ARG, BAD_STATE, HIP. */
int reshard_swap_in_source(reshard_plan *plan, int src_index, void *src_ptr, void *stream);
/* RESHARD_SRC_* of one source buffer (negative = error). */
int reshard_src_buffer_state(const reshard_plan *plan, int src_index);

/* Bind (or re-bind, after the caller re-allocated) the source pointers without
 * running the repack.  Allowed in UNBOUND, RESIDENT, ON_HOST and RELEASED; from
 * RELEASED the state becomes ON_HOST again (a device home for swap-in exists). */
int reshard_bind_src(reshard_plan *plan, const void *const *src_ptrs);

/*
 * Step 3, device-to-host: copies every used source buffer into pinned host
 * memory owned by the plan (allocated on first use, one block per buffer) with
 * hipMemcpyAsync on the plan's own side stream.  The side stream first waits for
 * the work already queued on `stream` at the time of the call (which may have
 * written the sources), and for nothing queued later: call reshard_swap_out
 * first and reshard_execute second (or use two streams) and the copies overlap
 * the repack, which only reads the sources.
 * State RESIDENT -> SWAPPING_OUT.  Call reshard_swap_wait before freeing the
 * device buffers: it returns once the copies are done AND every reshard_execute
 * issued on this plan while they were in flight has finished reading the sources.
 * Errors: BAD_STATE, HOST_OOM (state unchanged), HIP.
 */
int reshard_swap_out(reshard_plan *plan, void *stream);

/*
 * Step 3, second half (section "Allgather-Swap Technique": before the next update stage the
 * update weights are swapped from the host back to the device instead of being resharded
 * again; the paper notes that this copy can be issued ahead of time and hidden under the
 * inference stage): copies the pinned host copy back into
 * the currently bound source pointers on the side stream and makes `stream` wait
 * for it, so work queued on `stream` afterwards sees the weights.
 * State ON_HOST -> SWAPPING_IN.  Errors: BAD_STATE (not swapped out, or the
 * device copy was released and not re-bound), HIP.
 */
int reshard_swap_in(reshard_plan *plan, void *stream);

/*
 * Finer-grained wait: the copy of source buffer `index` alone (the copies of one swap run in
 * buffer order).  With host_wait != 0 the host blocks until that buffer's copy of the swap in
 * flight (or the last finished one) is done; otherwise `stream` is made to wait for it, so a
 * consumer can start on the first pipeline stage's weights while later buffers still stream
 * in.  A host wait also completes that buffer's state change (SWAPPING_OUT -> ON_HOST,
 * SWAPPING_IN -> RESIDENT); reshard_swap_wait completes the rest.
 * Errors: INVALID_ARG (index, unused buffer), BAD_STATE (no swap was ever started), HIP.
 */
int reshard_swap_wait_buffer(reshard_plan *plan, int index, void *stream, int host_wait);

/* Blocks the host until the swap copies in flight are done (and, for a swap-out, until every
 * repack launched on this plan meanwhile has finished: only then may the sources go) and
 * completes the state change (SWAPPING_OUT -> ON_HOST, SWAPPING_IN -> RESIDENT).  A no-op in
 * any other state. */
int reshard_swap_wait(reshard_plan *plan);

/* Ledger of step 3's release (section "Allgather-Swap Technique": once the update weights are on
 * the host their device buffer is released completely, so generation gets that memory; step 4
 * releases the temporary gather buffer, which on one device is the same memory): the caller has
 * freed the device copy of the sources (allowed in ON_HOST) / of the destinations.  The source
 * pointers are forgotten. */
int reshard_mark_src_released(reshard_plan *plan);
int reshard_mark_dst_released(reshard_plan *plan);

/* Host side of step 3 (the host buffer the update weights are swapped into).
 * Allocates the pinned host copies now (all or nothing) instead of inside the first swap-out,
 * which otherwise pays for pinning the pages (about one second for 65 GB).  Allowed in any state.
 * Errors: HOST_OOM. */
int reshard_reserve_host(reshard_plan *plan);

/* Frees the pinned host copy of step 3 once the weights are back on the device (allowed in
 * UNBOUND, RESIDENT: in every other state the host copy is the only one, or a copy is in flight). */
int reshard_release_host(reshard_plan *plan);

/* Host pointer of the pinned copy of source buffer `index` (NULL before the first
 * swap-out).  The memory is owned by the plan; valid until release/destroy. */
const void *reshard_host_copy(const reshard_plan *plan, int index);

/* Test hook: refuse pinned allocations once the plan would own more than `limit`
 * pinned bytes (negative = no limit).  Process-wide. */
void reshard_set_host_limit(int64_t limit);

/* The byte ledger (section "Allgather-Swap Technique", steps 3 and 4, and the memory-profiling
 * ablation, which reports about 8 GB released per device for the 32B dense model going from TP8 to
 * TP4): src_live + dst_live is the peak while both copies exist, and `released` is what the swap-out
 * gave back.  Pure host bookkeeping of what the caller told the plan. */
int reshard_mem_stats(const reshard_plan *plan, reshard_mem_stats_t *out);

/*
 * Plain device-to-device copy of `bytes` (multiple of 16, pointers 16-byte
 * aligned) with the same load/store code path as the repack kernel, one launch on
 * `stream`.  Used as the bandwidth ceiling next to the repack and to calibrate
 * hardware byte counters against a transfer of known size.
 */
int reshard_copy_baseline(void *dst, const void *src, int64_t bytes, void *stream);

/*
 * One-way bandwidth probes with the copy kernel's tile shape, launch shape and access hints:
 * reshard_read_baseline only loads `bytes` from `src` (the data is folded into a checksum that
 * is never stored), reshard_write_baseline only stores `bytes` of a fixed pattern to `dst`
 * (the buffer's contents are lost).  `bytes` a multiple of 32 KiB, pointers 16-byte aligned,
 * one launch on `stream`.  With R and W the two rates, a copy that moves equal bytes both ways
 * over the same memory is bounded by 2 / (1/R + 1/W).
 */
int reshard_read_baseline(const void *src, int64_t bytes, void *stream);
int reshard_write_baseline(void *dst, int64_t bytes, void *stream);

/* Library build tag, e.g. "reshard 0.1 gfx950". */
const char *reshard_version(void);

#ifdef __cplusplus
}
#endif
#endif /* RESHARD_H */
