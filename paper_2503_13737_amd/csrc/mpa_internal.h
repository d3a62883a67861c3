// Internal declarations shared by the host planner, the C ABI and the kernel launchers.
#pragma once
#include <cstddef>
#include <cstdint>
#include <vector>

namespace mpa {

// The kernels walk the cache in pages of 16 tokens.  A KV block holds 1, 2, 4 or 8 pages
// (block sizes 16, 32, 64, 128); page j of a sequence is page j % pages_per_block of the block
// in table entry j / pages_per_block.  In registers a page is named by one word,
// (block id << kPageBits) | page inside the block; -1 = none.
constexpr int kPage = 16;
constexpr int kPageBits = 3;
constexpr int kTileRows = 128;   // query rows of one prompt tile (matrix-core body)
constexpr int kKvTile = 64;      // keys staged per step of the matrix-core body
constexpr int kThreads = 256;    // work-group size of the attention kernel (4 wavefronts)
constexpr int kWaves = kThreads / 64;
// Wide launches: work-groups of 8 wavefronts, one per compute unit.  A prompt tile then has 256
// query rows (32 per wavefront) over one shared K/V tile, which lives in a ring of kRingBufs
// buffers: the loads of step s + kRingAhead are issued during step s and the wavefronts meet at a
// barrier every kRingBarrier steps only.
constexpr int kWideWaves = 8;
constexpr int kWideTileRows = 256;
constexpr int kRingBufs = 5;
constexpr int kRingAhead = 3;
constexpr int kRingBarrier = 2;
static_assert(kRingAhead >= kRingBarrier && kRingBufs >= kRingAhead + kRingBarrier, "ring hazards");

// kGroupItem: a generation row of a grouped-K/V-head layer on the matrix-core body -- the "rows" of
// the tile are the H/HK query heads that share one K/V head (its index sits in kind >> 8), all at
// the position of the one token q_row0; q_rows stays 1 (one token) in the work list.
enum ItemKind : int32_t { kRowItem = 0, kTileItem = 1, kGroupItem = 2 };
// Flag in the kind of a tile item: no other tile reads its keys (a chunk of one tile, or the ranges
// only the chunk's last tile reaches) and no other head does (every query head has its own K/V
// head), so its K/V passes through the caches once.
constexpr int32_t kSoloTile = 1 << 8;
// Above it, the kind of a tile item carries the tile's first row counted from the first row of its
// chunk: q_pos0 minus that is the first position of the sequence whose K/V arrives with this very
// iteration (needed when the append runs inside the attention launch).
constexpr int kTileRowShift = 9;
constexpr int32_t kTileRowMax = 1 << (31 - kTileRowShift);

// One unit of work.  A tile item is executed by one work-group per head; a row item by one
// wavefront per head (a work-group covers kWaves consecutive heads).
struct WorkItem {
    int32_t seq;       // sequence index = row of the block table
    int32_t q_row0;    // first row in q / out
    int32_t q_rows;    // rows of this item (1 for a row item)
    int32_t q_pos0;    // absolute position of row 0 inside its sequence
    int32_t kv_begin;  // first key position covered (multiple of the KV tile / block)
    int32_t kv_end;    // one past the last key position covered (<= q_pos0 + q_rows)
    int32_t part_row;  // first row in the partial buffers, or -1: write `out` directly
    int32_t kind;      // ItemKind
};
static_assert(sizeof(WorkItem) == 32, "work item layout");

// Tile items that walk the same keys of the same sequence (the q-tiles of a chunk over one key
// range) form a team per head: while they stay within a few steps of each other one fetch of a
// K/V tile from HBM serves all of them through L2.  Each member publishes the number of steps it
// has finished in progress[base + head * stride + member] (kNotRunning before its first and after
// its last step), and members that get ahead of a running team mate pause briefly.
struct TeamRef {
    int32_t base;      // first word of the team's [heads][stride] progress array, or -1: no pacing
    int32_t member;    // this item's index in its run of tiles over the same keys (set with or without pacing)
    int32_t size;      // tiles of the run (<= kTeamMax)
    int32_t stride;    // words per head
};
constexpr uint32_t kNotRunning = 0xFFFFFFFFu;
constexpr int kTeamMax = 64;   // one progress word per lane of the checking wavefront

// One output row whose keys were split over several items.
struct MergeRow {
    int32_t out_row;   // row in out
    int32_t part_row;  // partial row of split 0
    int32_t stride;    // partial rows between consecutive splits
    int32_t nsplit;
};
static_assert(sizeof(MergeRow) == 16, "merge row layout");

struct PlanOptions {
    int32_t heads = 0;
    int32_t kv_heads = 0;
    int32_t head_dim = 0;
    int32_t block_size = 16;      // tokens per KV block
    int64_t tg_split_blocks = 0;  // 0 = automatic
    int64_t pp_split_tokens = 0;  // 0 = automatic
    int64_t pp_rowstream = 0;
    int64_t pp_resident_wgs = 0;  // 0 = automatic
    int64_t pp_team_min_steps = 0; // shortest key range (in 64-key steps) whose q-tiles form a team; 0 = automatic
    int64_t tile_mode = 0;        // 0, 1 = work-groups of 4 wavefronts, 2 = of 8 (wide)
};

struct Plan {
    std::vector<WorkItem> items;  // tile items, then group items, then row items; each kind longest first
    std::vector<MergeRow> merge;
    std::vector<TeamRef> teams;   // one per tile item
    int64_t progress_words = 0;   // all set to kNotRunning before every launch
    int32_t n_tile_items = 0;
    int32_t n_group_items = 0;
    int32_t n_row_items = 0;
    int32_t n_tile_wgs = 0;       // work-groups that share the n_tile_items * heads tile units
    bool wide = false;            // work-groups of kWideWaves wavefronts, tiles of kWideTileRows rows
    bool fusable = true;          // the append may run inside the attention launch (see AttnParams::k_new)
    int64_t part_rows = 0;

    // workspace layout (byte offsets)
    // [items | merge | teams | progress] are written by the host before every launch
    size_t off_items = 0, off_merge = 0, off_teams = 0, off_progress = 0, off_acc = 0, off_ml = 0, total_bytes = 0;
};

// Returns MPA_OK or MPA_ERR_BAD_BATCH.
int build_plan(const PlanOptions &opt, const int32_t *chunk_starts, const int32_t *context_lens,
               int32_t num_seqs, Plan *plan);
size_t plan_bytes_upper_bound(const PlanOptions &opt, int64_t max_seqs, int64_t max_tokens,
                              int64_t max_ctx);

struct AttnParams {
    const uint16_t *q;
    const uint16_t *k_cache;
    const uint16_t *v_cache;
    const int32_t *block_table;
    int32_t table_stride;
    int32_t page_shift; // log2(pages per KV block)
    int32_t heads;      // query heads
    int32_t kv_heads;   // K/V heads; query head h reads K/V head h / (heads / kv_heads)
    int32_t group;      // heads / kv_heads
    float scale_log2e;  // scale * log2(e): scores are kept in base-2 exponent units
    uint16_t *out;
    const WorkItem *items;
    int32_t n_tile_items;
    int32_t n_group_items;
    int32_t n_row_items;
    int32_t n_tile_wgs;  // the first n_tile_wgs work-groups take tile units wg, wg + n_tile_wgs, ...
    float *part_acc;  // [part_rows, H, D]
    float *part_ml;   // [part_rows, H, 2]  (running max in base-2 units, running sum)
    const MergeRow *merge;
    int32_t n_merge;
    const TeamRef *teams;   // [n_tile_items]
    uint32_t *progress;
    int32_t wide;           // Plan::wide
    // Append inside the launch (k_new != nullptr): the iteration's new K/V [n_new, kv_heads, D] is
    // stored to the caches by n_append_wgs extra work-groups (between the tiles' and the rows'), and every reader
    // takes the keys of its own sequence's new positions from k_new / v_new instead of the cache.
    const uint16_t *k_new;
    const uint16_t *v_new;
    const int64_t *slot_map;
    int32_t n_new;
    int32_t block_size;
    int32_t n_append_wgs;
};

// The entry point that allocates nothing keeps work list and partial results in a device array of
// this size that is part of the library; the list travels there as kernel arguments.
constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
constexpr int kListChunkBytes = 3584;
// Device address of that array on the current device (looked up once per device).
int static_scratch(void **ptr);
// bytes: a multiple of 16; host_src is read before the call returns
int launch_list_chunks(const void *host_src, void *dst, size_t bytes, void *stream);

// Kernel launchers (kernels.hip).  Return the raw hipError_t as int.
int launch_kv_append(const void *k_new, const void *v_new, const int64_t *slot_map, int32_t T,
                     int32_t H, int32_t D, int32_t block_size, void *k_cache, void *v_cache, void *stream);
// bytes: a multiple of 16; *pinned_flag (host memory the GPU can write) receives `ticket` once pinned_src has been read
int launch_upload(const void *pinned_src, void *dst, size_t bytes, uint64_t *pinned_flag, uint64_t ticket, void *stream);
int launch_append_upload(const void *k_new, const void *v_new, const int64_t *slot_map, int32_t T, int32_t H, int32_t D,
                         int32_t block_size, void *k_cache, void *v_cache, const void *pinned_src, void *dst,
                         size_t bytes, uint64_t *pinned_flag, uint64_t ticket, void *stream);
int launch_copy_blocks(const void *src_k, const void *src_v, void *dst_k, void *dst_v, const int64_t *pairs,
                       int32_t n, int64_t block_bytes, void *stream);
int launch_attention(const AttnParams &p, int32_t D, bool fp16, void *stream);
int launch_merge(const AttnParams &p, int32_t D, bool fp16, void *stream);

}  // namespace mpa
