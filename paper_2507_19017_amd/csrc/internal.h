// Internal structures of the resharding library (not part of the C ABI).
#pragma once

#include <cstdint>
#include <string>
#include <vector>

#include "reshard.h"

namespace reshard {

// Logical weight tensors (row-major [out, in]).
enum LogicalId : int {
    LT_EMB, LT_FINAL_LN, LT_LM_HEAD, LT_LN1, LT_LN2,
    LT_WQ, LT_WK, LT_WV, LT_BQ, LT_BK, LT_BV, LT_WO,
    LT_GATE, LT_UP, LT_DOWN, LT_ROUTER, LT_SH_GATE, LT_SH_UP, LT_SH_DOWN,
    LT_EX_GATE, LT_EX_UP, LT_EX_DOWN,
    LT_QA, LT_QA_LN, LT_QB, LT_KVA, LT_KVA_LN, LT_KVB
};

// A rectangle [r0,r1) x [c0,c1) of a logical tensor and where a layout stores it.
// Element (r, c) lives at byte  off + ((r-r0)*ld + (c-c0))*eb   (transposed == false)
//                          or   off + ((c-c0)*ld + (r-r0))*eb   (transposed == true).
struct Fragment {
    uint64_t key;  // (logical id, layer, expert) packed; equal keys = same logical tensor
    int64_t r0, r1, c0, c1;
    int32_t buf;
    int64_t off;
    int64_t ld;
    bool transposed;
};

struct Side {
    reshard_layout layout{};
    int nd = 0, ne = 0;  // dense / expert buffer counts
    std::vector<int64_t> buf_bytes;
    std::vector<uint8_t> used;
    std::vector<reshard_tensor_info> tensors;
    std::vector<Fragment> frags;
};

// Device work item: 48 bytes, read with scalar loads by a whole workgroup.
struct alignas(16) Tile {
    uint64_t src_off;     // bytes from the start of the source buffer
    uint64_t dst_off;     // bytes from the start of the destination buffer
    uint32_t src_stride;  // bytes between rows.  gather: c0 | j0 << 16 | log2(k) << 24 (see below)
    uint32_t dst_stride;  //                      gather: 16-byte units between consecutive segments of one source
    uint32_t rows;        // copy: rows of the tile.  transpose: source rows (i extent).  gather: units of the tile
    uint32_t row_units;   // copy: vector units per row.  transpose: elements per source row (k extent).  gather: units per segment
    uint32_t magic;       // copy and gather: floor(2^32/row_units)+1, or 0 when rows == 1
    uint16_t src_buf;     // gather: the first of k consecutive entries of the pointer table
    uint16_t dst_buf;     // index into the pointer table (already offset past the sources)
    uint8_t kind;         // 0 strided copy, 1 transposing copy, 2 gathering copy: the tile is `rows` consecutive 16-byte
                          // units of the destination, made of segments of row_units units that come from k = 2^n
                          // sources in turn (source j of a group of k, then the next segment of every source);
                          // the tile starts c0 units into a segment of source j0, and src_off is that segment's row
    uint8_t vec_log2;     // copy: log2 of the vector width in bytes.  transpose: log2(elem_bytes)
    uint8_t pad_[2];
};
static_assert(sizeof(Tile) == 48, "tile record layout");

constexpr int kMaxTileUnits = 32768;  // keeps the multiply-high row split exact
constexpr int kMaxLayoutBuffers = 16384;  // buffers of one layout, used or not (tile records hold 16-bit indices)
constexpr int kTransposeDim = 64;     // transposing tiles are at most 64 x 64 elements

struct Tuning {
    int tile_bytes = 32 * 1024;   // one round of block_threads * unroll * 16 bytes
    int block_threads = 1024;
    int blocks_per_cu = 0;        // 0: one tile per workgroup; > 0: persistent grid
    int unroll = 2;               // 22 VGPRs: two 1024-lane workgroups fit a compute unit (8 takes 69: one)
    int flags = 127;              // bit 0/1: non-temporal loads/stores, bit 2: barrier between bursts,
                                  // bit 3: each XCD walks a contiguous eighth of the tile table,
                                  // bit 4: the one-tile copy kernel's load bursts run at raised wave priority,
                                  // bit 5: copy tiles in the woven order (the XCDs share every group of 8 tiles),
                                  // bit 6: with it, side-by-side merges as gathered tiles
    int transpose_rows = 0;       // register-transposed tiles: rows x cols of the source, in elements;
    int transpose_cols = 0;       // 0 (or a shape the element size does not allow): the default for that size
    int tail_pool_percent = 0;    // copy kernel: share of every XCD's eighth of the table left to the shared tail pool
    int tail_chunk_tiles = 16;    // tiles a pool workgroup takes per fetch
    int table_copies = 0;         // copies of the tile table on the device that successive executes rotate through
                                  // (0: as many as make 512 MiB; one for a table under 16 MiB, where 32 would not)
};
// The process-wide default that new plans copy (every plan then keeps its own).
Tuning current_tuning();
void set_default_tuning(const Tuning &t);
// Validates the ABI struct and overlays its non-zero fields on the built-in defaults
// (t == nullptr: the built-in defaults).  Returns RESHARD_OK or INVALID_ARG.
int tuning_from_abi(const reshard_tuning *t, Tuning &out);
void tuning_to_abi(const Tuning &t, reshard_tuning *out);

// Shapes the register-transpose kernel is built for: E-byte elements, ti x tk elements per tile.
// (16 / E) x (16 / E) blocks, one per lane and round; at least eight 16-byte chunks per
// destination row (the LDS swizzle needs them); whole waves; at most 128 KiB of LDS.
// Lanes of the workgroup that handles a ti x tk tile: the largest whole number of waves, at most
// 1024 lanes, that divides the tile's blocks (0 if there is none).
constexpr int transpose_threads(int E, int ti, int tk) {
    const int ve = 16 / E, blocks = (ti / ve) * (tk / ve);
    for (int t = 1024; t >= 64; t -= 64)
        if (blocks % t == 0) return t;
    return 0;
}
constexpr bool transpose_shape_ok(int E, int ti, int tk) {
    // 192 (2-byte elements, with 256 or 192 on the other side) serves experts of width 768 split four ways
    auto listed = [](int v) { return v == 64 || v == 128 || v == 192 || v == 256 || v == 512; };
    if (!listed(ti) || !listed(tk) || (E != 1 && E != 2 && E != 4 && E != 8)) return false;
    if ((ti == 192 || tk == 192) && (E != 2 || ti < 192 || tk < 192)) return false;
    const int ve = 16 / E;
    if (E == 1 ? tk < 128 : (ti > 256 || tk > 256)) return false;  // shapes nobody needs are not built
    return ti / ve >= 8 && (ti / ve) % 8 == 0 && transpose_threads(E, ti, tk) > 0 && ti * tk * E <= 128 * 1024;
}
// Shape used when the tuning names none (or one the element size does not allow).
inline void transpose_default_shape(int E, int &ti, int &tk) {
    ti = E == 8 ? 128 : E == 4 ? 128 : E == 1 ? 512 : 256;
    tk = E == 8 ? 128 : 256;
}

// Workgroups (of 256 lanes) for `n` generic transposing tiles: the kernel strides over the table, so
// the grid only has to stay within the 2^32 - 1 lanes of one launch.
constexpr uint32_t generic_transpose_grid(uint32_t n, uint32_t wanted) {
    const uint32_t cap = 0xFFFFFFFFu / 256u;
    return (n < wanted ? n : wanted) < cap ? (n < wanted ? n : wanted) : cap;
}
static_assert(uint64_t(generic_transpose_grid(0x7FFFFFF0u, 0xFFFFFFFFu)) * 256 <= 0xFFFFFFFFull &&
              generic_transpose_grid(1000, 0xFFFFFFFFu) == 1000 && generic_transpose_grid(1000, 512) == 512, "launch limit");

// Tiles of one kind that go out in one launch.
struct TileClass {
    int kind = 0;            // 0 strided copy, 1 register transpose of rows x cols elements, 2 generic transpose
    int rows = 0, cols = 0;  // kind 1 only
    // kind 0 only: tiles = [row blocks | row blocks that have a gathered form | runs | gathered].  The first
    // num_blocks tiles hold pitched rows, the next num_runs one contiguous row each; those two parts are the
    // whole work.  The last num_gathered tiles (Tile::kind 2) are the same bytes as the num_regathered last
    // row blocks, cut along the contiguous destination instead: the woven order launches them in their place.
    uint32_t max_units = 0;  // the most vector units any of the tiles holds
    uint32_t num_blocks = 0, num_regathered = 0, num_runs = 0, num_gathered = 0;
    bool runs_wide = true;   // every tile behind the row blocks moves 16-byte units
    std::vector<Tile> tiles;
};

void set_error(const std::string &msg);
int fail(int code, const std::string &msg);

// Host plan builder.
int build_side(const reshard_model_spec &spec, const reshard_layout &lay, bool is_source, Side &out);
int compile_descriptors(const reshard_model_spec &spec, Side &src, Side &dst,
                        std::vector<reshard_desc> &descs);
// classes[0]: copy tiles; classes[1]: register-transposed tiles of the preferred shape
// (fast_rows x fast_cols); then one class per other register shape used; last: generic transposes.
int cut_tiles(const std::vector<reshard_desc> &descs, int num_src_bufs, const Tuning &tuning,
              int fast_rows, int fast_cols, std::vector<TileClass> &classes);

}  // namespace reshard

struct reshard_plan {
    reshard_model_spec spec{};
    reshard::Side src, dst;
    std::vector<reshard_desc> descs;
    // copy tiles; register-transposed tiles by shape (the preferred shape first); generic transposes
    std::vector<reshard::TileClass> classes;
    int fast_rows = 0, fast_cols = 0;  // preferred shape of the register-transposed tiles
    reshard::Tuning tuning;            // this plan's own knobs: tile_bytes and the transposing shape are fixed
                                       // once the tiles are cut, the launch shape may change between executes
    // Tile records index a pointer table of the USED buffers only (used sources first, then used
    // destinations; at most RESHARD_MAX_BUFFERS): slot of every buffer (-1 unused) and the way back.
    std::vector<int> src_slot, dst_slot, slot_buf;
    int num_src_slots = 0;
    reshard_plan_info info{};
    uint64_t serial = 0;  // unique per plan in this process (tells whose table a shared device array holds)

    // device side (created lazily by the first execute)
    int device = -1;
    void *d_tiles = nullptr;  // the classes' tiles one after another
    int num_cus = 0;
    // streaming (created by the first execute_source): the tiles regrouped by source buffer
    struct SrcSlice { std::vector<uint32_t> first, count; uint32_t copy_blocks = 0; };  // per class; row-block tiles leading the copy class
                                                                                        // (gathered tiles read several sources: not here)
    std::vector<SrcSlice> src_slices;
    std::vector<reshard::Tile> by_src_tiles;
    void *d_by_src = nullptr;
    // d_tiles holds table_copies copies of the table, table_stride bytes apart; execute number n reads copy
    // n mod table_copies, so that the records an execute reads are not still in the memory-side cache from the
    // execute before (the woven kernel runs 3 to 4 % slower when they are)
    int table_copies = 1;
    size_t table_stride = 0;
    uint64_t executes = 0;

    // bound pointers
    std::vector<const void *> src_ptrs;
    std::vector<void *> dst_ptrs;
    bool dst_bound = false;

    // swap path
    int state = RESHARD_SRC_UNBOUND;
    std::vector<void *> host_copy;  // pinned, one per used source buffer (else nullptr)
    int64_t host_pinned = 0;
    void *side_stream = nullptr;
    void *ev_ready = nullptr;  // recorded on the caller's stream
    void *ev_exec = nullptr;   // recorded on the caller's stream behind a repack launched during a swap-out
    bool exec_during_swap = false;  // such a repack is (or may be) still reading the sources
    std::vector<void *> ev_buf; // per source buffer: recorded on the side stream after that buffer's copy
    std::vector<int> buf_state; // per source buffer: RESHARD_SRC_*; `state` is their common value or MIXED
    bool swapped_once = false;

    // ledger
    int64_t src_live = 0, dst_live = 0, peak_device = 0, released = 0;
    void touch_peak() {
        int64_t now = src_live + dst_live;
        if (now > peak_device) peak_device = now;
    }
};
