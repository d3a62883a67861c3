// Host planner: turns the ragged batch description (row offsets + context lengths) into the
// work list the attention kernel consumes.  Pure host code, no HIP.
//
// A sequence with one row (generation task) becomes row items: its keys are cut into
// contiguous ranges of whole KV blocks so that the chip sees several thousand equally sized
// streams.  A sequence with several rows (prompt chunk; Sec. 2.3 / 4.2 of the paper: rows
// prior..prior+q_len-1 of the prompt, attending to everything before them) becomes tile items
// of up to kTileRows rows, each tile's key range [0, last row's position] again cut into
// ranges when it is long.  Every item that is one of several over the same rows writes a
// partial result, and the rows are listed for the merge pass.
#include <algorithm>
#include <cmath>
#include <functional>
#include <map>
#include <numeric>
#include <queue>

#include "../../include/mpa.h"
#include "mpa_internal.h"

namespace mpa {

namespace {
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// What depends on the launch's work-group shape: four wavefronts and 128-row prompt tiles, two
// work-groups resident per compute unit -- or (wide) eight wavefronts and 256-row tiles, one
// work-group per compute unit, so that a compute unit runs either prompt tiles or generation rows.
struct Shape {
    int64_t waves, tile_rows, slots;   // slots: work-groups resident on the chip at a time
};
constexpr Shape kNarrow = {kWaves, kTileRows, 512};
constexpr Shape kWide = {kWideWaves, kWideTileRows, 256};
constexpr int64_t kComputeUnits = 256;

// Row items wanted from a batch: two per wavefront slot (256 compute units, 8 wavefronts each).
// Every item costs a partial result and a share of the merge, so few long ranges beat many short
// ones as long as the slots stay filled; beyond kMaxRowSplitTokens a range's own tail shows
// (measured over configs 2-5: best at 3.4-6 K items, ranges of 40-128 blocks of 16).
constexpr int64_t kRowItemTarget = 256 * 8 * 2;
constexpr int64_t kMaxRowSplitTokens = 1536;
constexpr int64_t kMinRowSplitTokens = 128;
constexpr int64_t kMinTileSplitSteps = 8;   // 512 keys
constexpr int64_t kTeamMinSteps = 16;       // shorter ranges do not drift apart far enough to matter
// Grouped K/V heads: from this group size on a generation row runs on the matrix-core body, one
// work-group per (row, K/V head, key range) with the group's query heads as the rows of the tile;
// below it the streaming body (one wavefront per query head) is cheaper.
constexpr int64_t kGroupMin = 4;
constexpr int64_t kGroupItemTarget = 1024;  // work-groups wanted from the group items of a batch
constexpr int64_t kMinGroupSplitSteps = 4;

// Key range of a row item in tokens: whole KV blocks, at least kMinRowSplitTokens, few enough
// items for every wavefront slot to see several.
//
// Around that length the one is taken whose work-groups fill whole rounds of the resident slots
// best: the rows are bandwidth-bound, so a last round with few work-groups in it streams at a
// fraction of the chip's rate for a whole range's time (measured on configs 2 and 3: kernel times
// follow this fill factor, 2 % between good and bad lengths).
int64_t auto_row_split_tokens(const PlanOptions &opt, const Shape &sh, int64_t total_tokens, const std::vector<int64_t> &row_keys)
{
    const int64_t kRowSlots = sh.slots;
    const int64_t bs = opt.block_size;
    if (opt.tg_split_blocks > 0) return opt.tg_split_blocks * bs;
    const int64_t want = std::min(std::max<int64_t>(ceil_div(total_tokens * opt.heads, kRowItemTarget), kMinRowSplitTokens),
                                  kMaxRowSplitTokens);
    const int64_t want_blocks = ceil_div(want, bs);
    if (row_keys.empty() || row_keys.size() > 512) return want_blocks * bs;   // keeps the search to a few microseconds
    const int64_t lo = std::max<int64_t>(ceil_div(kMinRowSplitTokens, bs), want_blocks * 2 / 3);
    const int64_t hi = std::max(lo, std::min<int64_t>(kMaxRowSplitTokens / bs, want_blocks * 3 / 2));
    const int64_t wgs_per_item = ceil_div(opt.heads, sh.waves);
    {   // with many rounds the last one weighs little, and the longest ranges are the cheapest
        int64_t items = 0;
        for (int64_t keys : row_keys) items += ceil_div(keys, want_blocks * bs);
        if (items * wgs_per_item > 4 * kRowSlots) return want_blocks * bs;
    }
    int64_t best = want_blocks;
    double best_fill = -1.0;
    for (int64_t nb = lo; nb <= hi; ++nb) {
        int64_t items = 0;
        for (int64_t keys : row_keys) items += ceil_div(keys, nb * bs);
        const int64_t wgs = items * wgs_per_item;
        const double fill = (double)wgs / (double)(ceil_div(wgs, kRowSlots) * kRowSlots);
        const bool nearer = std::llabs(nb - want_blocks) < std::llabs(best - want_blocks);
        if (fill > best_fill + 1e-9 || (fill > best_fill - 1e-9 && nearer)) {
            best_fill = fill;
            best = nb;
        }
    }
    return best * bs;
}

// Key range of a group item (a generation row of grouped K/V heads: one work-group per K/V head and
// range), in keys: whole 64-key steps, enough items for the chip, and -- like the row items' length,
// for batches of generation rows alone and few rounds -- the length near that whose work-groups
// fill whole rounds of the resident slots best (measured on 8 query / 1 K/V head, 256 rows at 2-8 K:
// 1092 work-groups 62 %, 990 work-groups 69 % of the HBM peak).
int64_t auto_group_split_keys(const PlanOptions &opt, const Shape &sh, int64_t total_tokens, const std::vector<int64_t> &row_keys)
{
    const int64_t kRowSlots = sh.slots;
    const int64_t want = std::max<int64_t>(ceil_div(ceil_div(total_tokens * opt.kv_heads, kGroupItemTarget), kKvTile),
                                           kMinGroupSplitSteps);
    if (row_keys.empty() || row_keys.size() > 512) return want * kKvTile;
    auto items_at = [&](int64_t steps) {
        int64_t items = 0;
        for (int64_t keys : row_keys) items += ceil_div(keys, steps * kKvTile);
        return items * opt.kv_heads;
    };
    if (items_at(want) > 4 * kRowSlots) return want * kKvTile;
    const int64_t lo = std::max<int64_t>(kMinGroupSplitSteps, want * 2 / 3), hi = std::max(lo, want * 3 / 2);
    int64_t best = want;
    double best_fill = -1.0;
    for (int64_t steps = lo; steps <= hi; ++steps) {
        const int64_t wgs = items_at(steps);
        const double fill = (double)wgs / (double)(ceil_div(wgs, kRowSlots) * kRowSlots);
        const bool nearer = std::llabs(steps - want) < std::llabs(best - want);
        if (fill > best_fill + 1e-9 || (fill > best_fill - 1e-9 && nearer)) {
            best_fill = fill;
            best = steps;
        }
    }
    return best * kKvTile;
}

// Key-range length for prompt tiles.  `tile_steps` holds, per tile, the number of 64-key steps
// of its full key range.  Splitting a tile's range costs a partial-result round trip, so the
// ranges are kept as long as the launch allows: candidates are tried from "no split" downwards,
// each scored by a list-scheduling estimate of the launch (every piece exists once per head and
// occupies one of the kTileSlots resident work-groups; generation rows keep the memory pipe busy
// for `row_us` anyway), and the longest range within a few percent of the best score wins.
constexpr double kStepUs = 1.9;          // one 64-key step of a 128-row tile with the chip full, measured
constexpr double kPieceOverheadSteps = 5.0;  // item and Q loads, first tile, partial result, its share of the merge
constexpr double kRowBytesPerUs = 6.0e6; // generation rows stream at about 6 TB/s

constexpr double kRowUnitBytesPerUs = 5.0e4;   // one compute unit streams generation rows at about 50 GB/s

// Pieces of one candidate, longest first: (length in steps incl. overhead, how many).
typedef std::vector<std::pair<double, int64_t>> PieceList;

void pieces_of(const std::vector<int64_t> &tile_steps_desc, int64_t len_steps, PieceList *out)
{
    out->clear();
    PieceList tails;
    for (int64_t st : tile_steps_desc) {   // descending, so the full-length pieces come out sorted
        const int64_t n = ceil_div(st, len_steps);
        const int64_t each = ceil_div(st, n);
        const int64_t last = st - (n - 1) * each;
        const int64_t n_full = last == each ? n : n - 1;
        if (n_full > 0) {
            if (!out->empty() && out->back().first == (double)each + kPieceOverheadSteps) out->back().second += n_full;
            else out->push_back({(double)each + kPieceOverheadSteps, n_full});
        }
        if (last != each) tails.push_back({(double)last + kPieceOverheadSteps, 1});
    }
    // `each` shrinks with st only up to rounding (ceil(st/n) with n growing): restore the order
    out->insert(out->end(), tails.begin(), tails.end());
    std::sort(out->begin(), out->end(), [](const std::pair<double, int64_t> &a, const std::pair<double, int64_t> &b) {
        return a.first > b.first;
    });
}

// Estimate of the launch's length for one candidate.  Every piece exists once per head and
// occupies one of kTileSlots resident work-groups.  Longest-first list scheduling of nearly
// equal pieces proceeds in rounds of kTileSlots pieces, and a round lasts as long as its longest
// piece: the estimate is the sum of the round leaders (exact for equal pieces, an upper bound of
// the greedy schedule otherwise) but never less than the mean load.  O(pieces), no simulation:
// the planner runs on the host in front of every launch.
double tile_makespan_us(const PieceList &pieces, int64_t heads, int64_t kTileSlots)
{
    double sum = 0.0, rounds = 0.0;
    int64_t placed = 0;   // pieces (x heads) placed so far
    for (const auto &pc : pieces) {
        const int64_t n = pc.second * heads;
        sum += pc.first * (double)n;
        // rounds that start inside this run of equal pieces: at positions that are multiples of kTileSlots
        const int64_t first = ceil_div(placed, kTileSlots), last = ceil_div(placed + n, kTileSlots);
        rounds += pc.first * (double)(last - first);
        placed += n;
    }
    return std::max(rounds, sum / (double)kTileSlots) * kStepUs;
}

int64_t auto_tile_split_tokens(const PlanOptions &opt, const Shape &sh, std::vector<int64_t> tile_steps, double row_us)
{
    const int64_t kTileSlots = sh.slots;
    if (opt.pp_split_tokens > 0) return ceil_div(opt.pp_split_tokens, kKvTile) * kKvTile;
    if (tile_steps.empty()) return kKvTile;
    std::sort(tile_steps.begin(), tile_steps.end(), std::greater<int64_t>());
    const int64_t longest = tile_steps.front();
    // Candidate range lengths: the longest tile cut into 1, 2, 3, 4, 6, 8, 12, 16, ... ranges
    // (steps of about 1.4 x), and the shortest lengths that still fit all pieces into exactly
    // 1, 2, 3, 4, 6, 8 rounds of resident work-groups -- the launch's length jumps there.
    std::vector<int64_t> cands;
    for (int64_t n = 1; n <= 64; n = (n < 4) ? n + 1 : ((n & (n - 1)) == 0 ? n + n / 2 : (n / 3) * 4)) {
        const int64_t len = std::max<int64_t>(ceil_div(longest, n), kMinTileSplitSteps);
        cands.push_back(len);
        if (len == kMinTileSplitSteps) break;
    }
    auto pieces_at = [&](int64_t len) {
        int64_t n = 0;
        for (int64_t st : tile_steps) n += ceil_div(st, len);
        return n * opt.heads;
    };
    for (int64_t rounds : {1, 2, 3, 4, 6, 8}) {
        int64_t lo = kMinTileSplitSteps, hi = longest;   // smallest len with pieces_at(len) <= rounds * slots
        if (pieces_at(hi) > rounds * kTileSlots) continue;
        while (lo < hi) {
            const int64_t mid = (lo + hi) / 2;
            if (pieces_at(mid) <= rounds * kTileSlots) hi = mid; else lo = mid + 1;
        }
        cands.push_back(lo);
    }
    std::sort(cands.begin(), cands.end(), std::greater<int64_t>());
    cands.erase(std::unique(cands.begin(), cands.end()), cands.end());
    std::vector<double> score(cands.size());
    PieceList pieces;
    double best = 1e300;
    for (size_t i = 0; i < cands.size(); ++i) {
        pieces_of(tile_steps, cands[i], &pieces);
        score[i] = std::max(tile_makespan_us(pieces, opt.heads, kTileSlots), row_us);
        best = std::min(best, score[i]);
    }
    for (size_t i = 0; i < cands.size(); ++i)
        if (score[i] <= best * 1.05) return cands[i] * kKvTile;
    return cands.back() * kKvTile;
}

void finish_layout(const PlanOptions &opt, Plan *p)
{
    size_t off = 0;
    p->off_items = off;
    off = align_up(off + p->items.size() * sizeof(WorkItem), 256);
    p->off_merge = off;
    off = align_up(off + p->merge.size() * sizeof(MergeRow), 256);
    p->off_teams = off;
    off = align_up(off + p->teams.size() * sizeof(TeamRef), 256);
    p->off_progress = off;
    off = align_up(off + (size_t)p->progress_words * sizeof(uint32_t), 256);
    p->off_acc = off;
    off = align_up(off + (size_t)p->part_rows * opt.heads * opt.head_dim * sizeof(float), 256);
    p->off_ml = off;
    off = align_up(off + (size_t)p->part_rows * opt.heads * 2 * sizeof(float), 256);
    p->total_bytes = off;
}
}  // namespace

int build_plan(const PlanOptions &opt, const int32_t *cs, const int32_t *ctx, int32_t S, Plan *plan)
{
    plan->items.clear();
    plan->merge.clear();
    plan->teams.clear();
    plan->fusable = !opt.pp_rowstream;   // a prompt row on the streaming body would need several new keys
    plan->progress_words = 0;
    plan->part_rows = 0;
    if (S < 0) return MPA_ERR_BAD_BATCH;
    if (S == 0) {
        plan->n_tile_items = plan->n_group_items = plan->n_row_items = plan->n_tile_wgs = 0;
        finish_layout(opt, plan);
        return MPA_OK;
    }
    if (cs[0] != 0) return MPA_ERR_BAD_BATCH;
    const int64_t bs = opt.block_size;
    // Work-group shape of the launch: wide only on request.  Measured, the wide shape is within 2 % of
    // the narrow one on prompts alone (better on long chunks, where it halves the K/V loads per row),
    // and loses on mixed batches and on generation rows of grouped K/V heads, so nothing selects it
    // by itself.
    const bool wide = opt.tile_mode == 2 && !opt.pp_rowstream;
    plan->wide = wide;
    const Shape &sh = wide ? kWide : kNarrow;
    const int64_t kTileRows = sh.tile_rows;   // (shadows the constant of the narrow shape)
    const int64_t kTileSlots = sh.slots;
    int64_t row_tokens = 0;   // keys visited by generation rows, in whole blocks
    std::vector<int64_t> row_keys;   // the same per row
    std::vector<int64_t> tile_steps;
    for (int32_t i = 0; i < S; ++i) {
        int64_t q_len = (int64_t)cs[i + 1] - cs[i];
        if (q_len < 1 || ctx[i] < q_len) return MPA_ERR_BAD_BATCH;
        int64_t prior = ctx[i] - q_len;
        if (q_len == 1 || opt.pp_rowstream) {
            for (int64_t j = 0; j < q_len; ++j) {
                row_tokens += ceil_div(prior + j + 1, bs) * bs;
                row_keys.push_back(prior + j + 1);
            }
        } else {
            for (int64_t r0 = 0; r0 < q_len; r0 += kTileRows) {
                int64_t rows = std::min<int64_t>(kTileRows, q_len - r0);
                tile_steps.push_back(ceil_div(prior + r0 + rows, kKvTile));
            }
        }
    }
    const int64_t group = opt.heads / opt.kv_heads;
    // generation rows become group items (one tile holds the whole group)
    const bool rows_on_tiles = group >= kGroupMin && group <= kTileRows && !opt.pp_rowstream;
    // (next to prompt tiles, which hold slots of their own for part of the launch, the rounds do
    // not come out as counted: there the plain target length stays)
    static const std::vector<int64_t> kNoRows;
    const int64_t row_split = auto_row_split_tokens(opt, sh, row_tokens, tile_steps.empty() ? row_keys : kNoRows);
    // key range of a group item, in keys: enough items for the chip, whole 64-key steps
    const int64_t group_split = auto_group_split_keys(opt, sh, row_tokens, tile_steps.empty() ? row_keys : kNoRows);
    const double row_us = (double)row_tokens * 4.0 * opt.head_dim * opt.kv_heads / kRowBytesPerUs;
    const int64_t tile_split = auto_tile_split_tokens(opt, sh, tile_steps, row_us);

    std::vector<WorkItem> tiles, groups, rows;
    auto emit = [&](std::vector<WorkItem> &dst, int32_t kind, int32_t seq, int32_t q_row0,
                    int32_t q_rows, int32_t q_pos0, int64_t split_len, int64_t granule, bool fixed_len) {
        const int64_t kv_len = (int64_t)q_pos0 + q_rows;  // keys visible to the last row
        int64_t nsplit = ceil_div(kv_len, split_len);
        // equal ranges, each a whole number of granules -- or the given length as it is
        int64_t len = fixed_len ? split_len : ceil_div(ceil_div(kv_len, nsplit), granule) * granule;
        nsplit = ceil_div(kv_len, len);
        int32_t part0 = -1;
        if (nsplit > 1) {
            part0 = (int32_t)plan->part_rows;
            plan->part_rows += nsplit * q_rows;
            for (int32_t r = 0; r < q_rows; ++r) {
                // a row only has partials from the ranges that start at or below its position
                int64_t ns_r = std::min<int64_t>(nsplit, ((int64_t)q_pos0 + r) / len + 1);
                plan->merge.push_back(MergeRow{q_row0 + r, part0 + r, q_rows, (int32_t)ns_r});
            }
        }
        for (int64_t s = 0; s < nsplit; ++s) {
            WorkItem it;
            it.seq = seq;
            it.q_row0 = q_row0;
            it.q_rows = q_rows;
            it.q_pos0 = q_pos0;
            it.kv_begin = (int32_t)(s * len);
            it.kv_end = (int32_t)std::min<int64_t>(kv_len, (s + 1) * len);
            it.part_row = nsplit > 1 ? (int32_t)(part0 + s * q_rows) : -1;
            it.kind = kind;
            dst.push_back(it);
        }
    };

    for (int32_t i = 0; i < S; ++i) {
        int32_t q_len = cs[i + 1] - cs[i];
        int32_t prior = ctx[i] - q_len;
        if (q_len == 1 && rows_on_tiles) {
            // ranges, partial rows and the merge row once; one item per K/V head over each range
            std::vector<WorkItem> one;
            const int64_t len = opt.tg_split_blocks > 0 ? ceil_div(opt.tg_split_blocks * bs, kKvTile) * kKvTile
                                                        : group_split;
            emit(one, kGroupItem, i, cs[i], 1, prior, len, kKvTile, false);
            for (int32_t kvh = 0; kvh < opt.kv_heads; ++kvh)
                for (WorkItem w : one) {
                    w.kind = kGroupItem | (kvh << 8);
                    groups.push_back(w);
                }
        } else if (q_len == 1 || opt.pp_rowstream) {
            for (int32_t j = 0; j < q_len; ++j)
                emit(rows, kRowItem, i, cs[i] + j, 1, prior + j, row_split, bs, false);
        } else {
            // All tiles of a chunk cut their keys at the same positions (equal ranges of the
            // chunk's whole context), so that the tiles over one range walk the same K/V blocks
            // from the same first key and can share them (see TeamRef); a tile simply has fewer
            // ranges when its rows end earlier.
            const int64_t n_seq = ceil_div((int64_t)ctx[i], tile_split);
            const int64_t len_seq = ceil_div(ceil_div((int64_t)ctx[i], n_seq), kKvTile) * kKvTile;
            for (int32_t r0 = 0; r0 < q_len; r0 += (int32_t)kTileRows) {
                int32_t nr = (int32_t)std::min<int64_t>(kTileRows, q_len - r0);
                if (r0 >= kTileRowMax) plan->fusable = false;   // (a chunk of 4 M rows)
                emit(tiles, kTileItem | (r0 < kTileRowMax ? r0 << kTileRowShift : 0), i, cs[i] + r0, nr, prior + r0, len_seq,
                     kKvTile, true);
            }
        }
    }
    auto cost = [](const WorkItem &w) {
        // keys actually visited, summed over rows (upper triangle of the last range excluded)
        int64_t full = (int64_t)(w.kv_end - w.kv_begin) * w.q_rows;
        return full;
    };
    auto longer = [&](const WorkItem &a, const WorkItem &b) { return cost(a) > cost(b); };
    // Tiles: all query tiles of one (sequence, key range) read the same K/V blocks.  They are kept
    // adjacent (one launch position apart per head, hence on the same XCD and resident together)
    // so that one tile's fetch serves the others from L2; groups go longest first.
    {
        // emit() produced the tiles sequence by sequence, tile by tile, range by range
        struct Key { int64_t group_cost; int32_t seq, kv_begin, q_row0; WorkItem w; };
        std::map<std::pair<int32_t, int32_t>, int64_t> group_cost;
        for (const WorkItem &w : tiles) group_cost[{w.seq, w.kv_begin}] += cost(w);
        std::vector<Key> keyed;
        keyed.reserve(tiles.size());
        for (const WorkItem &w : tiles) keyed.push_back(Key{group_cost[{w.seq, w.kv_begin}], w.seq, w.kv_begin, w.q_row0, w});
        std::sort(keyed.begin(), keyed.end(), [](const Key &a, const Key &b) {
            if (a.group_cost != b.group_cost) return a.group_cost > b.group_cost;
            if (a.seq != b.seq) return a.seq < b.seq;
            if (a.kv_begin != b.kv_begin) return a.kv_begin < b.kv_begin;
            return a.q_row0 < b.q_row0;
        });
        for (size_t i = 0; i < tiles.size(); ++i) tiles[i] = keyed[i].w;
        // a tile that is alone on its (sequence, key range) reads K/V nobody else reads -- unless
        // query heads share K/V heads: then the tile's units for those heads read it again
        for (size_t i = 0; i < tiles.size() && group == 1; ++i) {
            auto same = [&](size_t j) { return tiles[j].seq == tiles[i].seq && tiles[j].kv_begin == tiles[i].kv_begin; };
            const bool shared = (i > 0 && same(i - 1)) || (i + 1 < tiles.size() && same(i + 1));
            if (!shared) tiles[i].kind |= kSoloTile;
        }
    }
    std::stable_sort(rows.begin(), rows.end(), longer);
    std::stable_sort(groups.begin(), groups.end(), longer);
    plan->n_tile_items = (int32_t)tiles.size();
    plan->n_group_items = (int32_t)groups.size();
    plan->n_row_items = (int32_t)rows.size();
    // Work-groups for the tile units.  Alone, every unit gets its own and the hardware deals them
    // out as slots free up.  Next to a substantial amount of generation rows the tiles get a part
    // of the resident slots and keep them for the whole launch, while the rows stream through
    // the rest from the first microsecond: measured 8-15 % shorter launches on prompt-heavy
    // mixed batches than tiles first, rows after.
    {
        const int64_t units = (int64_t)tiles.size() * opt.heads;   // group items have work-groups of their own
        int64_t steps = 0;
        for (int64_t st : tile_steps) steps += st;
        const double tile_us = (double)steps * opt.heads * kStepUs / (double)kTileSlots;
        int64_t wgs = units;
        if (opt.pp_resident_wgs > 0) wgs = std::min(units, opt.pp_resident_wgs);
        else if (wide && (!rows.empty() || !groups.empty())) {
            // One work-group per compute unit: the tiles get n compute units for the whole launch and
            // the generation rows stream on the others, at kRowUnitBytesPerUs each up to the chip's
            // rate; when the tiles are done first their compute units take rows as well.  n is the
            // count with the shortest launch by that estimate, a multiple of the number of XCDs.
            const double row_bytes = row_us * kRowBytesPerUs;
            const double tile_unit_us = tile_us * (double)kTileSlots;   // on one compute unit
            auto rate = [&](int64_t cus) { return std::min(kRowBytesPerUs, (double)cus * kRowUnitBytesPerUs); };
            double best = 1e300;
            for (int64_t n = 8; n <= kComputeUnits - 8; n += 8) {
                const double t_tiles = tile_unit_us / (double)std::min(n, units);
                const double t_rows = row_bytes / rate(kComputeUnits - n);
                const double t = t_tiles >= t_rows ? t_tiles
                                                   : t_tiles + (row_bytes - t_tiles * rate(kComputeUnits - n)) / rate(kComputeUnits);
                if (t < best * 0.999) {
                    best = t;
                    wgs = std::min(n, units);
                }
            }
        } else if ((!rows.empty() || !groups.empty()) && row_us > 0.15 * tile_us) {
            // The more prompt work there is for the generation rows' streaming time, the more of
            // the slots the tiles keep: 256 (one per compute unit, a row work-group beside each)
            // when the tiles alone would take half the rows' time, 64 more per doubling of that
            // ratio.  Fitted to the best counts measured (config 3: 128, config 5 at iteration 8:
            // 192-256, config 4 and config 5 at iteration 24: 320, iteration 47: 384-448; grouped K/V
            // heads, 512 rows beside a 2048-token chunk: 128, 256 rows beside a 4096-token chunk:
            // 384-448); with too few the tiles outlast the rows (half the best count costs 20-70 %),
            // with too many the rows start late (all slots: 7-10 %).
            const double rho = tile_us / row_us;
            // (a multiple of 32: team mates sit heads * k units apart, and a count that is not a
            // multiple of the number of XCDs moves them to different XCDs from the second turn on)
            const int64_t by_ratio = 32 * (int64_t)std::llround((256.0 + 64.0 * std::log2(2.0 * rho)) / 32.0);
            wgs = std::min(units, std::min<int64_t>(kTileSlots * 7 / 8, std::max<int64_t>(by_ratio, 128)));
        }
        plan->n_tile_wgs = (int32_t)wgs;
    }
    // Teams: runs of adjacent tiles with the same (sequence, first key) -- see TeamRef.
    // Pacing is on request only: since a run's units are launched next to each other the tiles
    // stay together by themselves (K/V fetched 1.08 x), and the pauses only cost (measured with
    // pacing in every mixed launch: 2-4 % longer on configs 4 and 5, up to 8 % on grouped-head
    // mixes; 1.5 % longer on prompts alone).
    {
        const int64_t min_steps = opt.pp_team_min_steps > 0 ? opt.pp_team_min_steps : kTeamMinSteps;
        const bool want = opt.pp_team_min_steps > 0;
        plan->teams.assign(tiles.size(), TeamRef{-1, 0, 1, 0});
        // Every run of tiles over one (sequence, first key) is recorded (member, size): the
        // kernel keeps a run's units for one head next to each other in launch order.  Only where
        // pacing is wanted does the run get progress words (base >= 0).
        for (size_t i = 0; i < tiles.size();) {
            size_t j = i + 1;
            while (j < tiles.size() && j - i < (size_t)kTeamMax && tiles[j].seq == tiles[i].seq &&
                   tiles[j].kv_begin == tiles[i].kv_begin)
                ++j;
            const int64_t steps = ceil_div((int64_t)tiles[i].kv_end - tiles[i].kv_begin, kKvTile);
            const int32_t size = (int32_t)(j - i), stride = (size + 15) / 16 * 16;
            const bool paced = want && size >= 2 && steps >= min_steps;
            for (size_t k = i; k < j; ++k)
                plan->teams[k] = TeamRef{paced ? (int32_t)plan->progress_words : -1, (int32_t)(k - i), size, paced ? stride : 0};
            if (paced) plan->progress_words += (int64_t)stride * opt.heads;
            i = j;
        }
    }
    plan->items = std::move(tiles);
    plan->items.insert(plan->items.end(), groups.begin(), groups.end());
    plan->items.insert(plan->items.end(), rows.begin(), rows.end());
    finish_layout(opt, plan);
    return MPA_OK;
}

size_t plan_bytes_upper_bound(const PlanOptions &opt, int64_t max_seqs, int64_t max_tokens,
                              int64_t max_ctx)
{
    if (max_seqs <= 0 || max_tokens <= 0 || max_ctx <= 0) return 256;
    // Ranges are never shorter than the minimum split (or the forced one), so:
    const int64_t bs = opt.block_size;
    const int64_t row_split = opt.tg_split_blocks > 0 ? opt.tg_split_blocks * bs : ceil_div(kMinRowSplitTokens, bs) * bs;
    const int64_t tile_split = opt.pp_split_tokens > 0
                                   ? ceil_div(opt.pp_split_tokens, kKvTile) * kKvTile
                                   : kMinTileSplitSteps * kKvTile;
    const int64_t row_ns = ceil_div(max_ctx, row_split);
    const int64_t tile_ns = ceil_div(max_ctx, tile_split);
    // every row may be a generation task; alternatively rows group into tiles
    const int64_t n_rows_as_items = std::max(max_seqs, max_tokens);
    const int64_t n_tiles = max_tokens / 2 + max_seqs;  // a tile has >= 2 rows unless it is a remainder
    // as group items a row has one item per K/V head and 256-key range (fewer keys per range only if forced)
    const int64_t group_len = opt.tg_split_blocks > 0
                                  ? ceil_div(opt.tg_split_blocks * bs, kKvTile) * kKvTile
                                  : kMinGroupSplitSteps * kKvTile;
    const int64_t group_ns = opt.heads / opt.kv_heads >= kGroupMin ? ceil_div(max_ctx, group_len) * opt.kv_heads : 0;
    const int64_t items = n_rows_as_items * std::max(row_ns, group_ns) + n_tiles * tile_ns;
    const int64_t group_ranges = group_ns > 0 ? ceil_div(max_ctx, group_len) : 0;   // partial rows per token
    const int64_t part_rows = n_rows_as_items * std::max(row_ns, group_ranges) + (max_tokens + 0) * tile_ns;
    const int64_t merge_rows = max_tokens;
    Plan p;
    size_t off = 0;
    off = align_up(off + (size_t)items * sizeof(WorkItem), 256);
    off = align_up(off + (size_t)merge_rows * sizeof(MergeRow), 256);
    off = align_up(off + (size_t)n_tiles * tile_ns * sizeof(TeamRef), 256);
    // a team of n tiles holds heads * round_up(n, 16) words; teams have at least two members
    off = align_up(off + (size_t)n_tiles * tile_ns * opt.heads * 8 * sizeof(uint32_t), 256);
    off = align_up(off + (size_t)part_rows * opt.heads * opt.head_dim * sizeof(float), 256);
    off = align_up(off + (size_t)part_rows * opt.heads * 2 * sizeof(float), 256);
    return off;
}

}  // namespace mpa
