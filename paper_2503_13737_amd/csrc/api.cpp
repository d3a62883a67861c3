// C ABI of libmpa.so: argument checks, planning, upload of the work list, kernel launches.
#include <hip/hip_runtime.h>

#include <cmath>
#include <chrono>
#include <cstdlib>
#include <cstring>
#include <thread>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/mpa.h"
#include "mpa_internal.h"

using namespace mpa;

namespace {
constexpr int kStagingSlots = 8;

constexpr size_t kStagingHeader = 256;   // the completion word sits in front of the data

// One slot of the ring through which work lists travel: pinned host memory that the upload kernel
// reads, and a word in front of it to which that kernel writes the slot's ticket when it is done
// reading.  The slot is refilled only after its ticket has shown up.
struct Staging {
    void *host = nullptr;  // pinned: [completion word, padding | data]
    size_t bytes = 0;      // of data
    uint64_t ticket = 0;   // of the upload in flight from this slot
    bool in_flight = false;

    volatile uint64_t *flag() const { return static_cast<volatile uint64_t *>(host); }
    char *data() const { return static_cast<char *>(host) + kStagingHeader; }
    bool pinned = true;    // false: ordinary host memory (the stuck slot that a test plants; no GPU reads it)

    // The upload kernel of a slot finishes long before the ring comes round.  Returns true once
    // the slot's ticket has shown up (or nothing was in flight); false when it has not after
    // `timeout_ms` -- a launch that failed after it was queued, or a device that has stopped.  The
    // slot then stays marked as in flight: its memory may still be read and is not touched.
    bool wait(int64_t timeout_ms) {
        if (!in_flight || !host) return true;
        const auto t0 = std::chrono::steady_clock::now();
        while (*flag() < ticket) {
            if (std::chrono::steady_clock::now() - t0 > std::chrono::milliseconds(timeout_ms)) return false;
            std::this_thread::yield();
        }
        in_flight = false;
        return true;
    }
    void release() {
        if (!host) return;
        if (pinned) (void)hipHostFree(host);
        else std::free(host);
        host = nullptr;
        bytes = 0;
    }
};
}  // namespace

struct mpa_ctx {
    mpa_config cfg;
    PlanOptions opt;
    int last_hip = 0;
    Staging staging[kStagingSlots];
    int next_slot = 0;
    uint64_t next_ticket = 1;
    int64_t staging_timeout_ms = 5000;   // MPA_OPT_STAGING_TIMEOUT_MS
    Plan plan;  // the plan of the last batch; reused as it is when the next batch is the same
                // (all layers of one model iteration present the same batch)
    std::vector<int32_t> plan_key;   // chunk_starts then context_lens of that batch
    std::vector<char> list_host;     // the work list as the entry point that allocates nothing sends it
    bool plan_valid = false;         // cleared by mpa_set_option
    bool plan_cache = true;
    bool keep_upload = false;            // MPA_OPT_PLAN_CACHE == 2
    bool fuse_append = false;            // MPA_OPT_FUSE_APPEND
    const void *uploaded_ws = nullptr;   // where, and on which stream, the cached plan's work list was last uploaded
    const void *uploaded_stream = nullptr;
    bool uploaded_valid = false;
    std::vector<hipEvent_t> prof_events;  // start/stop pairs
    int32_t prof_used = 0;                // pairs recorded in the current series
    int32_t prof_every = 1;               // MPA_OPT_PROFILE_EVERY
    int32_t prof_repeat = 1;              // MPA_OPT_PROFILE_REPEAT
    int64_t prof_calls = 0;               // attention calls since profiling was enabled
    std::mutex mu;
};

static bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// No C++ exception leaves the library: host containers may fail to grow.
template <class F>
static auto guarded(F &&f, decltype(f()) on_no_memory) noexcept -> decltype(f())
{
    try {
        return f();
    } catch (...) {
        return on_no_memory;
    }
}

extern "C" {

int mpa_abi_version(void) { return MPA_ABI_VERSION; }

const char *mpa_status_string(int status)
{
    switch (status) {
    case MPA_OK: return "ok";
    case MPA_ERR_INVALID_ARG: return "invalid argument";
    case MPA_ERR_UNSUPPORTED: return "unsupported configuration";
    case MPA_ERR_WORKSPACE: return "workspace missing or too small";
    case MPA_ERR_BAD_BATCH: return "malformed batch description";
    case MPA_ERR_HIP: return "HIP runtime error";
    case MPA_ERR_NO_MEMORY: return "out of host memory";
    default: return "unknown status";
    }
}

int mpa_create(mpa_ctx **out, const mpa_config *cfg)
{
    if (!out || !cfg) return MPA_ERR_INVALID_ARG;
    *out = nullptr;
    if (cfg->num_heads <= 0) return MPA_ERR_INVALID_ARG;
    if (cfg->dtype != MPA_BF16 && cfg->dtype != MPA_FP16) return MPA_ERR_UNSUPPORTED;
    if (cfg->num_kv_heads <= 0) return MPA_ERR_INVALID_ARG;
    if (cfg->num_kv_heads > cfg->num_heads || cfg->num_heads % cfg->num_kv_heads != 0) return MPA_ERR_UNSUPPORTED;
    if (cfg->head_dim != 64 && cfg->head_dim != 128) return MPA_ERR_UNSUPPORTED;
    if (cfg->block_size != 16 && cfg->block_size != 32 && cfg->block_size != 64 && cfg->block_size != 128)
        return MPA_ERR_UNSUPPORTED;
    mpa_ctx *c = new (std::nothrow) mpa_ctx();
    if (!c) return MPA_ERR_NO_MEMORY;
    c->cfg = *cfg;
    c->opt.heads = cfg->num_heads;
    c->opt.kv_heads = cfg->num_kv_heads;
    c->opt.head_dim = cfg->head_dim;
    c->opt.block_size = cfg->block_size;
    *out = c;
    return MPA_OK;
}

int mpa_destroy(mpa_ctx *ctx)
{
    if (!ctx) return MPA_OK;
    for (auto &s : ctx->staging) {
        // a slot whose upload never reported back may still be read by the GPU: it is left allocated
        if (s.wait(ctx->staging_timeout_ms) || !s.pinned) s.release();
    }
    for (hipEvent_t e : ctx->prof_events) (void)hipEventDestroy(e);
    delete ctx;
    return MPA_OK;
}

int mpa_profile_enable(mpa_ctx *ctx, int32_t max_calls)
{
    if (!ctx || max_calls < 0 || max_calls > (1 << 24)) return MPA_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> g(ctx->mu);
    for (hipEvent_t e : ctx->prof_events) (void)hipEventDestroy(e);
    ctx->prof_events.clear();
    ctx->prof_used = 0;
    ctx->prof_calls = 0;
    return guarded([&]() -> int {
        ctx->prof_events.reserve(2 * (size_t)max_calls);
        for (int32_t i = 0; i < 2 * max_calls; ++i) {
            hipEvent_t e;
            hipError_t rc = hipEventCreate(&e);
            if (rc != hipSuccess) {
                ctx->last_hip = (int)rc;
                return MPA_ERR_HIP;
            }
            ctx->prof_events.push_back(e);
        }
        return MPA_OK;
    }, MPA_ERR_NO_MEMORY);
}

int mpa_profile_read(mpa_ctx *ctx, float *ms, int32_t cap, int32_t *n_out)
{
    if (!ctx || cap < 0 || (cap > 0 && !ms) || !n_out) return MPA_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> g(ctx->mu);
    int32_t n = ctx->prof_used < cap ? ctx->prof_used : cap;
    for (int32_t i = 0; i < n; ++i) {
        hipError_t rc = hipEventSynchronize(ctx->prof_events[2 * i + 1]);
        if (rc == hipSuccess) rc = hipEventElapsedTime(&ms[i], ctx->prof_events[2 * i], ctx->prof_events[2 * i + 1]);
        if (rc == hipSuccess) ms[i] /= (float)ctx->prof_repeat;
        if (rc != hipSuccess) {
            ctx->last_hip = (int)rc;
            return MPA_ERR_HIP;
        }
    }
    *n_out = n;
    ctx->prof_used = 0;
    return MPA_OK;
}

int mpa_set_option(mpa_ctx *ctx, int32_t option, int64_t value)
{
    if (!ctx || value < 0) return MPA_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> g(ctx->mu);
    ctx->plan_valid = false;   // the cached plan was made under the old options
    switch (option) {
    case MPA_OPT_TG_SPLIT_BLOCKS: ctx->opt.tg_split_blocks = value; return MPA_OK;
    case MPA_OPT_PP_SPLIT_TOKENS: ctx->opt.pp_split_tokens = value; return MPA_OK;
    case MPA_OPT_PP_ROWSTREAM: ctx->opt.pp_rowstream = value ? 1 : 0; return MPA_OK;
    case MPA_OPT_PP_RESIDENT_WGS:
        if (value < 0) return MPA_ERR_INVALID_ARG;
        ctx->opt.pp_resident_wgs = value;
        return MPA_OK;
    case MPA_OPT_PLAN_CACHE:
        if (value < 0 || value > 2) return MPA_ERR_INVALID_ARG;
        ctx->plan_cache = value != 0;
        ctx->keep_upload = value == 2;
        return MPA_OK;
    case MPA_OPT_PROFILE_EVERY:
        if (value < 1 || value > 1 << 20) return MPA_ERR_INVALID_ARG;
        ctx->prof_every = (int32_t)value;
        return MPA_OK;
    case MPA_OPT_PP_TEAM_MIN_STEPS:
        if (value < 0) return MPA_ERR_INVALID_ARG;
        ctx->opt.pp_team_min_steps = value;
        return MPA_OK;
    case MPA_OPT_PROFILE_REPEAT:
        if (value < 1 || value > 1024) return MPA_ERR_INVALID_ARG;
        ctx->prof_repeat = (int32_t)value;
        return MPA_OK;
    case MPA_OPT_FUSE_APPEND:
        if (value > 1) return MPA_ERR_INVALID_ARG;
        ctx->fuse_append = value == 1;
        return MPA_OK;
    case MPA_OPT_TILE_MODE:
        if (value > 2) return MPA_ERR_INVALID_ARG;
        ctx->opt.tile_mode = value;
        return MPA_OK;
    case MPA_OPT_STAGING_TIMEOUT_MS:
        if (value < 1 || value > 600000) return MPA_ERR_INVALID_ARG;
        ctx->staging_timeout_ms = value;
        return MPA_OK;
    case MPA_OPT_TEST_STUCK_UPLOAD: {
        // The slot the next upload would use is made to look like one whose upload kernel never
        // reported back (ordinary host memory, a ticket that no kernel will write): the error
        // path of the staging ring can then be driven from the host, without a GPU.
        if (value != 1) return MPA_ERR_INVALID_ARG;
        Staging &st = ctx->staging[ctx->next_slot];
        if (st.in_flight) return MPA_ERR_INVALID_ARG;
        st.release();
        st.host = std::calloc(1, kStagingHeader + 4096);
        if (!st.host) return MPA_ERR_INVALID_ARG;
        st.pinned = false;
        st.bytes = 4096;
        st.ticket = ctx->next_ticket++;
        st.in_flight = true;
        return MPA_OK;
    }
    default: return MPA_ERR_INVALID_ARG;
    }
}

int mpa_last_hip_error(const mpa_ctx *ctx) { return ctx ? ctx->last_hip : 0; }

size_t mpa_workspace_bytes_for_batch(const mpa_ctx *ctx, const int32_t *chunk_starts,
                                     const int32_t *context_lens, int32_t num_seqs)
{
    if (!ctx || num_seqs < 0 || (num_seqs > 0 && (!chunk_starts || !context_lens))) return 0;
    return guarded([&]() -> size_t {
        Plan p;
        if (build_plan(ctx->opt, chunk_starts, context_lens, num_seqs, &p) != MPA_OK) return 0;
        return p.total_bytes > 256 ? p.total_bytes : 256;
    }, (size_t)0);
}

size_t mpa_workspace_bytes(const mpa_ctx *ctx, int32_t max_seqs, int32_t max_tokens, int32_t max_ctx)
{
    if (!ctx) return 0;
    return plan_bytes_upper_bound(ctx->opt, max_seqs, max_tokens, max_ctx);
}

int64_t mpa_plan_describe(const mpa_ctx *ctx, const int32_t *chunk_starts,
                          const int32_t *context_lens, int32_t num_seqs, int32_t *items,
                          int64_t cap, int32_t *counts)
{
    if (!ctx || num_seqs < 0 || (num_seqs > 0 && (!chunk_starts || !context_lens)) || cap < 0 ||
        (cap > 0 && !items))
        return MPA_ERR_INVALID_ARG;
    return guarded([&]() -> int64_t {
        Plan p;
        int rc = build_plan(ctx->opt, chunk_starts, context_lens, num_seqs, &p);
        if (rc != MPA_OK) return rc;
        const int64_t n = (int64_t)p.items.size();
        if (cap > 0) std::memcpy(items, p.items.data(), (size_t)(n < cap ? n : cap) * sizeof(WorkItem));
        if (counts) {
            counts[0] = p.n_tile_items + p.n_group_items;
            counts[1] = p.n_row_items;
            counts[2] = (int32_t)p.merge.size();
            counts[3] = (int32_t)p.part_rows;
        }
        return n;
    }, (int64_t)MPA_ERR_NO_MEMORY);
}

int mpa_kv_append(mpa_ctx *ctx, const void *k_new, const void *v_new, const int64_t *slot_map,
                  int32_t num_tokens, void *k_cache, void *v_cache, void *stream)
{
    if (!ctx || num_tokens < 0) return MPA_ERR_INVALID_ARG;
    if (num_tokens == 0) return MPA_OK;
    if (!k_new || !v_new || !slot_map || !k_cache || !v_cache) return MPA_ERR_INVALID_ARG;
    if (!aligned(k_new, 16) || !aligned(v_new, 16) || !aligned(k_cache, 16) || !aligned(v_cache, 16) ||
        !aligned(slot_map, 8))
        return MPA_ERR_INVALID_ARG;
    int e = launch_kv_append(k_new, v_new, slot_map, num_tokens, ctx->cfg.num_kv_heads, ctx->cfg.head_dim,
                             ctx->cfg.block_size,
                             k_cache, v_cache, stream);
    if (e != 0) {
        ctx->last_hip = e;
        return MPA_ERR_HIP;
    }
    return MPA_OK;
}

int mpa_copy_blocks(mpa_ctx *ctx, const void *src_k, const void *src_v, void *dst_k, void *dst_v,
                    const int64_t *pairs, int32_t num_pairs, void *stream)
{
    if (!ctx || num_pairs < 0) return MPA_ERR_INVALID_ARG;
    if (num_pairs == 0) return MPA_OK;
    if (!src_k || !src_v || !dst_k || !dst_v || !pairs) return MPA_ERR_INVALID_ARG;
    if (!aligned(src_k, 16) || !aligned(src_v, 16) || !aligned(dst_k, 16) || !aligned(dst_v, 16) || !aligned(pairs, 8))
        return MPA_ERR_INVALID_ARG;
    const int64_t block_bytes = (int64_t)ctx->cfg.num_kv_heads * ctx->cfg.block_size * ctx->cfg.head_dim * 2;
    // at most 65,535 pairs per launch (the grid's second dimension)
    for (int32_t done = 0; done < num_pairs; done += 65535) {
        const int32_t n = std::min<int32_t>(65535, num_pairs - done);
        int e = launch_copy_blocks(src_k, src_v, dst_k, dst_v, pairs + 2 * (int64_t)done, n, block_bytes, stream);
        if (e != 0) {
            ctx->last_hip = e;
            return MPA_ERR_HIP;
        }
    }
    return MPA_OK;
}

}  // extern "C"

namespace {
// The new K/V of the iteration, when the append travels with the attention call.
struct AppendArgs {
    const void *k_new, *v_new;
    const int64_t *slot_map;
    void *k_cache, *v_cache;
};

int attend_may_throw(mpa_ctx *ctx, const AppendArgs *app, const void *q, const void *k_cache, const void *v_cache,
                     const int32_t *block_table, int32_t block_table_stride, const int32_t *chunk_starts,
                     const int32_t *context_lens, int32_t num_seqs, int32_t num_tokens, float scale, void *out,
                     void *workspace, size_t workspace_bytes, bool static_ws, void *stream);

int attend(mpa_ctx *ctx, const AppendArgs *app, const void *q, const void *k_cache, const void *v_cache,
           const int32_t *block_table, int32_t block_table_stride, const int32_t *chunk_starts,
           const int32_t *context_lens, int32_t num_seqs, int32_t num_tokens, float scale, void *out,
           void *workspace, size_t workspace_bytes, bool static_ws, void *stream)
{
    const int rc = guarded([&]() -> int {
        return attend_may_throw(ctx, app, q, k_cache, v_cache, block_table, block_table_stride, chunk_starts, context_lens,
                                num_seqs, num_tokens, scale, out, workspace, workspace_bytes, static_ws, stream);
    }, MPA_ERR_NO_MEMORY);
    if (rc == MPA_ERR_NO_MEMORY && ctx) {
        // whatever was being put together is not trusted: the next call plans and uploads afresh
        std::lock_guard<std::mutex> g(ctx->mu);
        ctx->plan_valid = false;
        ctx->uploaded_valid = false;
    }
    return rc;
}

int attend_may_throw(mpa_ctx *ctx, const AppendArgs *app, const void *q, const void *k_cache, const void *v_cache,
                     const int32_t *block_table, int32_t block_table_stride, const int32_t *chunk_starts,
                     const int32_t *context_lens, int32_t num_seqs, int32_t num_tokens, float scale, void *out,
                     void *workspace, size_t workspace_bytes, bool static_ws, void *stream)
{
    if (!ctx || num_seqs < 0 || num_tokens < 0) return MPA_ERR_INVALID_ARG;
    if (num_seqs == 0) return num_tokens == 0 ? MPA_OK : MPA_ERR_BAD_BATCH;
    if (app && (!app->k_new || !app->v_new || !app->slot_map || !aligned(app->k_new, 16) || !aligned(app->v_new, 16) ||
                !aligned(app->slot_map, 8)))
        return MPA_ERR_INVALID_ARG;
    if (!q || !k_cache || !v_cache || !block_table || !chunk_starts || !context_lens || !out)
        return MPA_ERR_INVALID_ARG;
    if (block_table_stride <= 0) return MPA_ERR_INVALID_ARG;
    if (!aligned(q, 16) || !aligned(out, 16) || !aligned(k_cache, 16) || !aligned(v_cache, 16) ||
        !aligned(block_table, 4))
        return MPA_ERR_INVALID_ARG;
    if (!(scale == scale)) return MPA_ERR_INVALID_ARG;  // NaN

    std::lock_guard<std::mutex> g(ctx->mu);
    Plan &plan = ctx->plan;
    const size_t n_key = 2 * (size_t)num_seqs + 1;
    const bool same = ctx->plan_cache && ctx->plan_valid && ctx->plan_key.size() == n_key &&
                      std::memcmp(ctx->plan_key.data(), chunk_starts, ((size_t)num_seqs + 1) * sizeof(int32_t)) == 0 &&
                      std::memcmp(ctx->plan_key.data() + num_seqs + 1, context_lens, (size_t)num_seqs * sizeof(int32_t)) == 0;
    if (!same) {
        ctx->plan_valid = false;
        ctx->uploaded_valid = false;
        int rc = build_plan(ctx->opt, chunk_starts, context_lens, num_seqs, &plan);
        if (rc != MPA_OK) return rc;
        ctx->plan_key.assign(chunk_starts, chunk_starts + num_seqs + 1);
        ctx->plan_key.insert(ctx->plan_key.end(), context_lens, context_lens + num_seqs);
        ctx->plan_valid = true;
    }
    if (chunk_starts[num_seqs] != num_tokens) return MPA_ERR_BAD_BATCH;
    for (int32_t i = 0; i < num_seqs; ++i)
        if (((int64_t)context_lens[i] + ctx->cfg.block_size - 1) / ctx->cfg.block_size > block_table_stride)
            return MPA_ERR_BAD_BATCH;
    static_assert(kStaticScratchBytes == MPA_STATIC_SCRATCH_BYTES, "the header states the limit");
    if (static_ws) {
        if (plan.total_bytes > kStaticScratchBytes) return MPA_ERR_WORKSPACE;   // before any HIP call
    } else if (!workspace || !aligned(workspace, 256) || workspace_bytes < plan.total_bytes) {
        return MPA_ERR_WORKSPACE;
    }

    auto fail = [&](hipError_t e) {
        ctx->last_hip = (int)e;
        ctx->uploaded_valid = false;
        return MPA_ERR_HIP;
    };
    if (static_ws) {
        // The library's own device array stands in for the workspace.  Every context and every
        // call on this GPU shares it, so nothing is assumed to be in it from an earlier call.
        const int se = static_scratch(&workspace);
        if (se != 0) return fail((hipError_t)se);
        ctx->uploaded_valid = false;
    }

    // The work list of this very plan may still sit in this workspace from the previous call on
    // this stream (the kernels only read it, and every progress word is back at its start value
    // when a launch has finished): then nothing is copied.
    const bool list_in_place = !static_ws && same && ctx->keep_upload && ctx->uploaded_valid &&
                               ctx->uploaded_ws == workspace && ctx->uploaded_stream == stream;
    hipStream_t s = (hipStream_t)stream;
    hipError_t e;
    // the append inside the attention launch: no append kernel of its own, in either branch below
    const bool fused = app && ctx->fuse_append && plan.fusable;
    if (list_in_place && app && !fused) {
        int ae = launch_kv_append(app->k_new, app->v_new, app->slot_map, num_tokens, ctx->cfg.num_kv_heads,
                                  ctx->cfg.head_dim, ctx->cfg.block_size, app->k_cache, app->v_cache, stream);
        if (ae != 0) return fail((hipError_t)ae);
    }
    auto write_list = [&](char *h) {
        std::memcpy(h + plan.off_items, plan.items.data(), plan.items.size() * sizeof(WorkItem));
        std::memcpy(h + plan.off_merge, plan.merge.data(), plan.merge.size() * sizeof(MergeRow));
        std::memcpy(h + plan.off_teams, plan.teams.data(), plan.teams.size() * sizeof(TeamRef));
        std::memset(h + plan.off_progress, 0xFF, (size_t)plan.progress_words * sizeof(uint32_t));  // kNotRunning
    };
    if (static_ws) {
        // No staging memory: the list is put together in ordinary host memory and handed to the
        // device as kernel arguments.
        const size_t list_bytes = plan.off_acc;
        if (list_bytes % 16 != 0) return MPA_ERR_WORKSPACE;
        ctx->list_host.assign(list_bytes, 0);
        write_list(ctx->list_host.data());
        const int le = launch_list_chunks(ctx->list_host.data(), workspace, list_bytes, stream);
        if (le != 0) return fail((hipError_t)le);
    } else if (!list_in_place) {
        // stage the work list in pinned memory; a small kernel carries it into the workspace on the stream
        const size_t list_bytes = plan.off_acc;  // items, merge rows, teams, progress words; padded
        Staging &st = ctx->staging[ctx->next_slot];
        if (!st.wait(ctx->staging_timeout_ms)) {
            // The upload that last used this slot never reported back.  Nothing is written to the
            // slot and nothing is launched; the work list this context believes to be on the
            // device is not trusted any more.  The ring does not advance: the next call finds the
            // same slot and succeeds once its ticket has arrived.
            ctx->plan_valid = false;
            return fail(hipErrorNotReady);
        }
        ctx->next_slot = (ctx->next_slot + 1) % kStagingSlots;
        if (st.bytes < list_bytes || !st.pinned) {
            st.release();
            st.pinned = true;
            size_t want = list_bytes * 2;
            if ((e = hipHostMalloc(&st.host, kStagingHeader + want, hipHostMallocCoherent)) != hipSuccess)
                return fail(e);
            st.bytes = want;
            *st.flag() = 0;
        }
        char *h = st.data();
        write_list(h);
        if (list_bytes % 16 != 0) return MPA_ERR_WORKSPACE;   // the plan pads its sections
        st.ticket = ctx->next_ticket++;
        const int ue = app && !fused ? launch_append_upload(app->k_new, app->v_new, app->slot_map, num_tokens, ctx->cfg.num_kv_heads,
                                                  ctx->cfg.head_dim, ctx->cfg.block_size, app->k_cache, app->v_cache, h,
                                                  workspace, list_bytes, const_cast<uint64_t *>(st.flag()), st.ticket, stream)
                           : launch_upload(h, workspace, list_bytes, const_cast<uint64_t *>(st.flag()), st.ticket, stream);
        if (ue != 0) return fail((hipError_t)ue);
        st.in_flight = true;
        ctx->uploaded_ws = workspace;
        ctx->uploaded_stream = stream;
        ctx->uploaded_valid = true;
    }

    char *ws = static_cast<char *>(workspace);
    AttnParams p;
    p.q = static_cast<const uint16_t *>(q);
    p.k_cache = static_cast<const uint16_t *>(k_cache);
    p.v_cache = static_cast<const uint16_t *>(v_cache);
    p.block_table = block_table;
    p.table_stride = block_table_stride;
    p.page_shift = ctx->cfg.block_size == 16 ? 0 : ctx->cfg.block_size == 32 ? 1 : ctx->cfg.block_size == 64 ? 2 : 3;
    p.heads = ctx->cfg.num_heads;
    p.kv_heads = ctx->cfg.num_kv_heads;
    p.group = ctx->cfg.num_heads / ctx->cfg.num_kv_heads;
    const float sc = scale > 0.f ? scale : 1.0f / std::sqrt((float)ctx->cfg.head_dim);
    p.scale_log2e = sc * 1.4426950408889634f;
    p.out = static_cast<uint16_t *>(out);
    p.items = reinterpret_cast<const WorkItem *>(ws + plan.off_items);
    p.n_tile_items = plan.n_tile_items;
    p.n_group_items = plan.n_group_items;
    p.n_row_items = plan.n_row_items;
    p.n_tile_wgs = plan.n_tile_wgs;
    p.part_acc = reinterpret_cast<float *>(ws + plan.off_acc);
    p.part_ml = reinterpret_cast<float *>(ws + plan.off_ml);
    p.merge = reinterpret_cast<const MergeRow *>(ws + plan.off_merge);
    p.n_merge = (int32_t)plan.merge.size();
    p.teams = reinterpret_cast<const TeamRef *>(ws + plan.off_teams);
    p.progress = reinterpret_cast<uint32_t *>(ws + plan.off_progress);
    p.wide = plan.wide ? 1 : 0;
    p.k_new = fused ? static_cast<const uint16_t *>(app->k_new) : nullptr;
    p.v_new = fused ? static_cast<const uint16_t *>(app->v_new) : nullptr;
    p.slot_map = fused ? app->slot_map : nullptr;
    p.n_new = fused ? num_tokens : 0;
    p.block_size = ctx->cfg.block_size;
    p.n_append_wgs = 0;   // the launcher counts them

    const bool prof = (size_t)(2 * ctx->prof_used + 1) < ctx->prof_events.size() &&
                      ctx->prof_calls++ % ctx->prof_every == 0;
    if (prof && (e = hipEventRecord(ctx->prof_events[2 * ctx->prof_used], s)) != hipSuccess) return fail(e);
    int he = launch_attention(p, ctx->cfg.head_dim, ctx->cfg.dtype == MPA_FP16, stream);
    if (he != 0) return fail((hipError_t)he);
    // A timed call may launch the kernel several times back to back between its two events (the
    // launch only reads its inputs and rewrites the same outputs and partial results), so that
    // the events' own cost in the queue is shared by all of them.
    for (int32_t r = 1; prof && r < ctx->prof_repeat; ++r) {
        he = launch_attention(p, ctx->cfg.head_dim, ctx->cfg.dtype == MPA_FP16, stream);
        if (he != 0) return fail((hipError_t)he);
    }
    if (prof) {
        if ((e = hipEventRecord(ctx->prof_events[2 * ctx->prof_used + 1], s)) != hipSuccess) return fail(e);
        ++ctx->prof_used;
    }
    he = launch_merge(p, ctx->cfg.head_dim, ctx->cfg.dtype == MPA_FP16, stream);
    if (he != 0) return fail((hipError_t)he);
    return MPA_OK;
}
}  // namespace

extern "C" {

int mpa_mixed_paged_attention(mpa_ctx *ctx, const void *q, const void *k_cache, const void *v_cache,
                              const int32_t *block_table, int32_t block_table_stride,
                              const int32_t *chunk_starts, const int32_t *context_lens,
                              int32_t num_seqs, int32_t num_tokens, float scale, void *out,
                              void *workspace, size_t workspace_bytes, void *stream)
{
    return attend(ctx, nullptr, q, k_cache, v_cache, block_table, block_table_stride, chunk_starts, context_lens,
                  num_seqs, num_tokens, scale, out, workspace, workspace_bytes, false, stream);
}

int mpa_mixed_paged_attention_static(mpa_ctx *ctx, const void *q, const void *k_cache, const void *v_cache,
                                     const int32_t *block_table, int32_t block_table_stride,
                                     const int32_t *chunk_starts, const int32_t *context_lens,
                                     int32_t num_seqs, int32_t num_tokens, float scale, void *out, void *stream)
{
    return attend(ctx, nullptr, q, k_cache, v_cache, block_table, block_table_stride, chunk_starts, context_lens,
                  num_seqs, num_tokens, scale, out, nullptr, 0, true, stream);
}

int mpa_append_and_attend(mpa_ctx *ctx, const void *k_new, const void *v_new, const int64_t *slot_map,
                          const void *q, void *k_cache, void *v_cache, const int32_t *block_table,
                          int32_t block_table_stride, const int32_t *chunk_starts, const int32_t *context_lens,
                          int32_t num_seqs, int32_t num_tokens, float scale, void *out, void *workspace,
                          size_t workspace_bytes, void *stream)
{
    const AppendArgs app = {k_new, v_new, slot_map, k_cache, v_cache};
    return attend(ctx, &app, q, k_cache, v_cache, block_table, block_table_stride, chunk_starts, context_lens,
                  num_seqs, num_tokens, scale, out, workspace, workspace_bytes, false, stream);
}

}  // extern "C"
