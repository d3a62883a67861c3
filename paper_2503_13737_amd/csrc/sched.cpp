// Batch scheduler of the attention path (host only): token budget (Sec. 4.2, Eq. 6), remaining-time
// order (Sec. 4.3), dynamic chunking with one long prompt at a time (Sec. 4.2), block-granular KVC
// demand (Sec. 4.4) and the two batching algorithms (Sec. 4.4, Algorithms 1 and 2), over a block
// pool of its own.  See include/mpa_sched.h for the contract.
//
// All decisions are integer, except the remaining times and the budget, which are IEEE doubles
// evaluated in a fixed order without contraction so that every implementation of the same
// formulas decides alike.
#pragma clang fp contract(off)

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <memory>
#include <new>
#include <unordered_map>
#include <vector>

#include "../../include/mpa.h"
#include "../../include/mpa_sched.h"

namespace {

// prompt; generation task back from the last iteration; set aside with its blocks; set aside with
// its blocks moved to the swap pool
enum State : uint8_t { kPrompt = 0, kReturned = 1, kSetAside = 2, kSwapped = 3 };

struct Req {
    int64_t id;
    int64_t prompt_len, max_new, processed = 0, generated = 0;
    double slo_first, slo_token, t_enter, t_r = 0.0;
    State state = kPrompt;
    bool started = false;     // a chunk of it has been scheduled
    bool in_batch = false;
    bool evicted_now = false; // preempted by the decision being formed
    bool taken = false;       // scratch of the selection loop
    bool offline = false;     // JCT SLO: `allowance` seconds of waiting per iteration, `carry` moved on
    double allowance = 0.0, carry = 0.0;
    std::vector<int32_t> blocks;
    std::vector<int32_t> swap;    // its blocks in the swap pool while it is swapped out

    bool is_prompt() const { return state == kPrompt; }
    // tokens whose K/V are cached; a generation task has not fed its newest token yet
    int64_t cached() const { return is_prompt() ? processed : prompt_len + generated - 1; }
    double waited(double now) const { return state == kReturned ? 0.0 : now - t_enter; }
};

struct Entry {
    Req *r;
    int64_t tokens;
    int64_t new_blocks;
};

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

}  // namespace

struct mpa_sched {
    mpa_sched_config cfg;
    std::vector<int32_t> free_blocks;                       // stack, next block at the back
    std::vector<int32_t> swap_free;                         // the same for the swap pool
    std::vector<int64_t> swap_out, swap_in;                 // {source, destination} pairs of the last decision
    std::unordered_map<int64_t, std::unique_ptr<Req>> live;
    std::vector<Entry> batch;
    int64_t chunk_tokens = 0, chunks = 0;                   // for L_c, the mean chunk length
    int32_t token_budget = 0, evicted = 0;

    int64_t b() const { return cfg.block_size; }
    // Sec. 4.4: blocks a request needs for `tokens` more tokens (what fits its last block is free)
    int64_t demand_blocks(const Req &r, int64_t tokens) const
    {
        return std::max<int64_t>(0, ceil_div(r.cached() + tokens, b()) - (int64_t)r.blocks.size());
    }
    // tokens it could take with `extra` more blocks
    int64_t room_tokens(const Req &r, int64_t extra) const
    {
        return ((int64_t)r.blocks.size() + extra) * b() - r.cached();
    }
    bool is_long(const Req &r) const { return r.prompt_len > cfg.pivot_forward_size; }
    bool long_in_progress(const Req &r) const
    {
        return is_long(r) && r.is_prompt() && r.started && r.processed < r.prompt_len;
    }
    double mean_chunk() const
    {
        return chunks == 0 ? (double)cfg.pivot_forward_size : (double)chunk_tokens / (double)chunks;
    }
    // the iteration-level SLO that enters Eq. 6
    double slo(const Req &r) const
    {
        if (r.offline) return r.allowance + cfg.max_batch_time;
        return r.is_prompt() ? r.slo_first : r.slo_token;
    }
    // Sec. 4.3: T_r = SLO - T_w - N_ck * T_max; for a JCT SLO what is left of the iteration's allowance
    double remaining_time(const Req &r, double now) const
    {
        if (r.offline) {
            const double allowed = r.allowance + r.carry;
            return allowed - r.waited(now);
        }
        double n_ck = 1.0, waited = 0.0;
        if (r.is_prompt()) {
            n_ck = std::ceil((double)(r.prompt_len - r.processed) / mean_chunk());
            waited = now - r.t_enter;
        } else if (r.state != kReturned) {   // set aside, with its blocks or swapped out
            waited = now - r.t_enter;
        }
        const double slack = (r.is_prompt() ? r.slo_first : r.slo_token) - waited;
        const double exec = n_ck * cfg.max_batch_time;
        return slack - exec;
    }
    void evict(Req &r, double now, bool give_back_blocks)
    {
        ++evicted;
        r.evicted_now = true;
        r.t_enter = now;
        if (r.state == kSwapped) return;   // it holds nothing here; it simply does not get in
        if (!give_back_blocks) {
            r.state = kSetAside;
            return;
        }
        if (cfg.num_swap_blocks > 0 && r.blocks.size() <= swap_free.size()) {
            for (int32_t blk : r.blocks) {   // its blocks move to the other pool and are free here
                const int32_t sb = swap_free.back();
                swap_free.pop_back();
                swap_out.push_back(blk);
                swap_out.push_back(sb);
                r.swap.push_back(sb);
                free_blocks.push_back(blk);
            }
            r.blocks.clear();
            r.state = kSwapped;
            return;
        }
        for (int32_t blk : r.blocks) free_blocks.push_back(blk);
        r.blocks.clear();
        r.prompt_len += r.generated;   // the prompt and every token produced so far
        r.max_new -= r.generated;      // the recomputed prompt yields the next one
        r.processed = r.generated = 0;
        r.state = kPrompt;
        r.started = false;
    }
    void select_requests(int64_t a_c, int64_t a_m, const std::vector<Req *> &order);
};

// Algorithm 2: among the requests within gamma of the first one that may run, keep taking the one
// whose demand is nearest to what is left of both resources.
void mpa_sched::select_requests(int64_t a_c, int64_t a_m, const std::vector<Req *> &order)
{
    bool long_busy = false;
    for (auto &kv : live) {
        const Req &r = *kv.second;
        if (long_in_progress(r) || (is_long(r) && r.is_prompt() && r.in_batch)) long_busy = true;
    }
    auto blocked = [&](const Req &r) { return r.is_prompt() && is_long(r) && !r.started && long_busy; };

    std::vector<Req *> cands;
    bool have_first = false;
    double t_first = 0.0;
    for (Req *r : order) {
        if (r->in_batch || r->evicted_now || blocked(*r)) continue;
        if (!have_first) {
            have_first = true;
            t_first = r->t_r;
        }
        if (r->t_r <= t_first + cfg.gamma || long_in_progress(*r)) {
            r->taken = false;
            cands.push_back(r);
        }
    }
    for (;;) {
        Req *best = nullptr;
        int64_t best_d2 = 0, best_c = 0, best_blocks = 0;
        for (Req *r : cands) {
            if (r->taken || blocked(*r)) continue;
            int64_t d_c = 1;
            if (r->is_prompt()) {
                d_c = std::min({r->prompt_len - r->processed, a_c, room_tokens(*r, a_m)});
                if (d_c < 1) continue;
            }
            const int64_t d_blocks = demand_blocks(*r, d_c);
            if (d_c > a_c || d_blocks > a_m) continue;
            const int64_t dc = a_c - d_c, dm = (a_m - d_blocks) * b();
            const int64_t d2 = dc * dc + dm * dm;
            if (!best || d2 < best_d2) {
                best = r;
                best_d2 = d2;
                best_c = d_c;
                best_blocks = d_blocks;
            }
        }
        if (!best) return;
        best->taken = best->in_batch = true;
        batch.push_back({best, best_c, best_blocks});
        if (best->is_prompt() && is_long(*best)) long_busy = true;
        a_c -= best_c;
        a_m -= best_blocks;
    }
}

extern "C" {

int mpa_sched_create(mpa_sched **out, const mpa_sched_config *cfg, const int32_t *block_order)
try {
    if (!out || !cfg) return MPA_ERR_INVALID_ARG;
    *out = nullptr;
    if (cfg->block_size < 1 || cfg->num_blocks < 1 || cfg->pivot_forward_size < 1 || cfg->max_batch_tokens < 1 ||
        !(cfg->pivot_time > 0.0) || !(cfg->max_batch_time > 0.0) || !(cfg->gamma >= 0.0) ||
        !(cfg->preempt_max_time >= 0.0) || !(cfg->preempt_probability >= 0.0) || cfg->num_swap_blocks < 0)
        return MPA_ERR_INVALID_ARG;
    std::unique_ptr<mpa_sched> s(new (std::nothrow) mpa_sched());
    if (!s) return MPA_ERR_NO_MEMORY;
    s->cfg = *cfg;
    const int32_t n = cfg->num_blocks;
    s->free_blocks.resize(n);
    std::vector<char> seen(n, 0);
    for (int32_t i = 0; i < n; ++i) {
        const int32_t blk = block_order ? block_order[i] : i;
        if (blk < 0 || blk >= n || seen[blk]) return MPA_ERR_INVALID_ARG;
        seen[blk] = 1;
        s->free_blocks[n - 1 - i] = blk;   // handed out from the back
    }
    s->swap_free.resize((size_t)cfg->num_swap_blocks);
    for (int32_t i = 0; i < cfg->num_swap_blocks; ++i) s->swap_free[(size_t)(cfg->num_swap_blocks - 1 - i)] = i;
    *out = s.release();
    return MPA_OK;
} catch (...) {
    return MPA_ERR_NO_MEMORY;   // host containers could not grow
}

int mpa_sched_destroy(mpa_sched *s)
{
    delete s;
    return MPA_OK;
}

int mpa_sched_add_request(mpa_sched *s, int64_t id, int32_t prompt_len, int32_t max_new_tokens,
                          double slo_first, double slo_token, double now)
try {
    if (!s || prompt_len < 1 || max_new_tokens < 1) return MPA_ERR_INVALID_ARG;
    if ((int64_t)prompt_len + max_new_tokens - 1 > (int64_t)s->cfg.num_blocks * s->cfg.block_size) return MPA_ERR_INVALID_ARG;
    if (s->live.count(id)) return MPA_ERR_INVALID_ARG;
    std::unique_ptr<Req> r(new (std::nothrow) Req());
    if (!r) return MPA_ERR_NO_MEMORY;
    r->id = id;
    r->prompt_len = prompt_len;
    r->max_new = max_new_tokens;
    r->slo_first = slo_first;
    r->slo_token = slo_token;
    r->t_enter = now;
    s->live.emplace(id, std::move(r));
    return MPA_OK;
} catch (...) {
    return MPA_ERR_NO_MEMORY;   // host containers could not grow
}

int mpa_sched_add_offline_request(mpa_sched *s, int64_t id, int32_t prompt_len, int32_t max_new_tokens,
                                  int32_t predicted_new_tokens, double slo_jct, double now)
try {
    if (!s || predicted_new_tokens < 1) return MPA_ERR_INVALID_ARG;
    const int rc = mpa_sched_add_request(s, id, prompt_len, max_new_tokens, 0.0, 0.0, now);
    if (rc != MPA_OK) return rc;
    Req &r = *s->live[id];
    const double n_ck = std::ceil((double)r.prompt_len / s->mean_chunk());
    const double preempt = s->cfg.preempt_max_time * s->cfg.preempt_probability;
    const double per_token = s->cfg.max_batch_time + preempt;
    const double prompt_time = n_ck * s->cfg.max_batch_time;
    const double gen_time = (double)predicted_new_tokens * per_token;
    const double t_e = prompt_time + gen_time;
    r.offline = true;
    r.allowance = (slo_jct - t_e) / (n_ck + (double)predicted_new_tokens);
    return MPA_OK;
} catch (...) {
    return MPA_ERR_NO_MEMORY;   // host containers could not grow
}

// Algorithm 1.
int mpa_sched_next_batch(mpa_sched *s, double now, mpa_sched_batch *info)
try {
    if (!s || !info) return MPA_ERR_INVALID_ARG;
    s->batch.clear();
    s->swap_out.clear();
    s->swap_in.clear();
    s->evicted = 0;
    s->token_budget = 0;
    *info = mpa_sched_batch{};
    if (s->live.empty()) {
        info->free_blocks = (int32_t)s->free_blocks.size();
        return MPA_OK;
    }
    // the queue: ascending remaining time
    std::vector<Req *> order;
    order.reserve(s->live.size());
    for (auto &kv : s->live) {
        Req *r = kv.second.get();
        r->t_r = s->remaining_time(*r, now);
        r->in_batch = r->evicted_now = false;
        order.push_back(r);
    }
    std::sort(order.begin(), order.end(), [](const Req *x, const Req *y) {
        return x->t_r != y->t_r ? x->t_r < y->t_r : x->id < y->id;
    });
    // Eq. 6.  SLO_min is the smallest iteration-level SLO among the requests that are certain to be
    // in the batch before anything is selected -- the generation tasks back from the last iteration
    // and the urgent requests -- and the queue head, which the selection considers first.  (The
    // queue is ordered by remaining time, not by SLO: a prompt with a loose SLO that has waited
    // long can be its head while generation tasks with much tighter SLOs are in the batch.)
    {
        double slo_min = s->slo(*order[0]);
        for (const Req *r : order)
            if (r->state == kReturned || r->t_r <= s->cfg.max_batch_time) slo_min = std::min(slo_min, s->slo(*r));
        const double scaled = (double)s->cfg.pivot_forward_size * slo_min;
        const double budget = std::floor(scaled / s->cfg.pivot_time);
        int64_t sb = budget >= (double)s->cfg.max_batch_tokens ? s->cfg.max_batch_tokens : (int64_t)budget;
        s->token_budget = (int32_t)std::max<int64_t>(1, std::min<int64_t>(sb, s->cfg.max_batch_tokens));
    }
    const int64_t s_b = s->token_budget;
    int64_t s_f = 0, need = 0;
    auto put = [&](Req *r, int64_t tokens) {
        const int64_t nb = s->demand_blocks(*r, tokens);
        s->batch.push_back({r, tokens, nb});
        r->in_batch = true;
        s_f += tokens;
        need += nb;
    };
    for (Req *r : order)   // generation tasks of the last iteration stay
        if (r->state == kReturned) put(r, 1);
    for (Req *r : order)   // urgent requests
        if (r->state != kReturned && r->t_r <= s->cfg.max_batch_time)
            put(r, r->is_prompt() ? std::min<int64_t>(r->prompt_len - r->processed, s_b) : 1);
    // while a resource is over-committed the request with the largest remaining time gives way:
    // a prompt chunk is cut to what fits before it is dropped, a generation task is preempted
    while (s_f > s_b || need > (int64_t)s->free_blocks.size()) {
        size_t v = 0;
        for (size_t i = 1; i < s->batch.size(); ++i) {
            const Req *x = s->batch[i].r, *y = s->batch[v].r;
            if (x->t_r != y->t_r ? x->t_r > y->t_r : x->id > y->id) v = i;
        }
        Entry e = s->batch[v];
        const int64_t others_tokens = s_f - e.tokens, others_blocks = need - e.new_blocks;
        const bool blocks_short = need > (int64_t)s->free_blocks.size();
        if (e.r->is_prompt()) {
            const int64_t fit = std::min({e.tokens, s_b - others_tokens,
                                          s->room_tokens(*e.r, (int64_t)s->free_blocks.size() - others_blocks)});
            if (fit >= 1 && fit < e.tokens) {
                s->batch[v].tokens = fit;
                s->batch[v].new_blocks = s->demand_blocks(*e.r, fit);
                s_f = others_tokens + fit;
                need = others_blocks + s->batch[v].new_blocks;
                continue;
            }
        }
        s->batch.erase(s->batch.begin() + (ptrdiff_t)v);
        e.r->in_batch = false;
        s_f = others_tokens;
        need = others_blocks;
        if (!e.r->is_prompt()) s->evict(*e.r, now, blocks_short);
    }
    if (s_b - s_f > 0) s->select_requests(s_b - s_f, (int64_t)s->free_blocks.size() - need, order);

    // allocation, in batch order
    for (Entry &e : s->batch) {
        if (e.r->offline) {   // the iteration starts: unused or overdrawn waiting time moves on
            const double allowed = e.r->allowance + e.r->carry;
            e.r->carry = allowed - e.r->waited(now);
        }
        for (int64_t k = 0; k < e.new_blocks; ++k) {
            e.r->blocks.push_back(s->free_blocks.back());
            s->free_blocks.pop_back();
        }
        if (e.r->state == kSwapped) {   // back in: its content returns into the first of its fresh blocks
            for (size_t k = 0; k < e.r->swap.size(); ++k) {
                s->swap_in.push_back(e.r->swap[k]);
                s->swap_in.push_back(e.r->blocks[k]);
                s->swap_free.push_back(e.r->swap[k]);
            }
            e.r->swap.clear();
            e.r->state = kSetAside;
        }
        info->num_tokens += (int32_t)e.tokens;
        if (e.r->is_prompt()) {
            e.r->started = true;
            s->chunk_tokens += e.tokens;
            ++s->chunks;
            ++info->num_prompt_chunks;
        } else {
            ++info->num_generation;
        }
        info->max_blocks_per_seq = std::max<int32_t>(info->max_blocks_per_seq, (int32_t)e.r->blocks.size());
    }
    info->num_seqs = (int32_t)s->batch.size();
    info->token_budget = s->token_budget;
    info->num_preempted = s->evicted;
    info->free_blocks = (int32_t)s->free_blocks.size();
    info->num_swap_out = (int32_t)(s->swap_out.size() / 2);
    info->num_swap_in = (int32_t)(s->swap_in.size() / 2);
    return MPA_OK;
} catch (...) {
    return MPA_ERR_NO_MEMORY;   // host containers could not grow
}

int mpa_sched_batch_swaps(const mpa_sched *s, int64_t *out_pairs, int64_t *in_pairs)
try {
    if (!s) return MPA_ERR_INVALID_ARG;
    if (out_pairs) std::copy(s->swap_out.begin(), s->swap_out.end(), out_pairs);
    if (in_pairs) std::copy(s->swap_in.begin(), s->swap_in.end(), in_pairs);
    return MPA_OK;
} catch (...) {
    return MPA_ERR_NO_MEMORY;   // host containers could not grow
}

int mpa_sched_batch_arrays(const mpa_sched *s, int64_t *request_ids, int32_t *chunk_starts,
                           int32_t *context_lens, int64_t *slot_map, int32_t *block_table,
                           int32_t block_table_stride)
try {
    if (!s) return MPA_ERR_INVALID_ARG;
    int32_t row0 = 0;
    const int64_t b = s->cfg.block_size;
    for (size_t i = 0; i < s->batch.size(); ++i) {
        const Entry &e = s->batch[i];
        const int64_t prior = e.r->cached(), end = prior + e.tokens;
        const int64_t nblk = ceil_div(end, b);
        if (nblk > (int64_t)e.r->blocks.size()) return MPA_ERR_BAD_BATCH;
        if (request_ids) request_ids[i] = e.r->id;
        if (chunk_starts) chunk_starts[i] = row0;
        if (context_lens) context_lens[i] = (int32_t)end;
        if (slot_map)
            for (int64_t pos = prior; pos < end; ++pos)
                slot_map[row0 + (pos - prior)] = (int64_t)e.r->blocks[(size_t)(pos / b)] * b + pos % b;
        if (block_table) {
            if (nblk > block_table_stride) return MPA_ERR_INVALID_ARG;
            int32_t *row = block_table + i * (size_t)block_table_stride;
            for (int32_t j = 0; j < block_table_stride; ++j) row[j] = j < nblk ? e.r->blocks[(size_t)j] : -1;
        }
        row0 += (int32_t)e.tokens;
    }
    if (chunk_starts) chunk_starts[s->batch.size()] = row0;
    return MPA_OK;
} catch (...) {
    return MPA_ERR_NO_MEMORY;   // host containers could not grow
}

int mpa_sched_complete(mpa_sched *s, double now, int64_t *finished_ids, int32_t cap, int32_t *num_finished)
try {
    if (!s) return MPA_ERR_INVALID_ARG;
    int32_t n = 0;
    for (const Entry &e : s->batch) {
        Req &r = *e.r;
        if (r.is_prompt()) {
            r.processed += e.tokens;
            if (r.processed == r.prompt_len) {   // the last chunk yields the prompt's token
                r.generated = 1;
                r.state = kReturned;
            } else if (r.offline) {
                r.t_enter = now;                 // the next chunk's iteration waits from here
            }
        } else {
            r.generated += 1;
            r.state = kReturned;
        }
        if (r.state == kReturned && r.generated >= r.max_new) {
            if (finished_ids && n < cap) finished_ids[n] = r.id;
            ++n;
            for (int32_t blk : r.blocks) s->free_blocks.push_back(blk);
            s->live.erase(r.id);
        }
    }
    s->batch.clear();
    if (num_finished) *num_finished = n;
    return MPA_OK;
} catch (...) {
    return MPA_ERR_NO_MEMORY;   // host containers could not grow
}

int32_t mpa_sched_live_requests(const mpa_sched *s) { return s ? (int32_t)s->live.size() : 0; }

}  // extern "C"
