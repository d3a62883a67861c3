"""Plain Python oracle of the batch scheduler that feeds the attention path (paper Sec. 4).

TEST INFRASTRUCTURE ONLY: imported by tests/ and by the benchmark's baseline leg, never by the
product package, and it imports nothing from it.  Slow and literal on purpose: every iteration
recomputes everything from the request list, in the order the paper gives.

What it follows
  * token budget            S_b = S_pf * SLO_min / T_pf                         (Sec. 4.2, Eq. 6)
  * remaining time          T_r = SLO - T_w - T_e,  T_e = N_ck * T_max,
                            N_ck = ceil(S_r / L_c) for a prompt, 1 for a generation task (Sec. 4.3)
  * queue order             ascending T_r; urgent = T_r <= T_max                (Sec. 4.3)
  * offline requests        a JCT SLO is spread over the request's iterations:
                            T_e = N_ck * T_max + S_g * (T_max + P_max * P),
                            allowance per iteration = (SLO_JCT - T_e) / (N_ck + S_g); waiting longer
                            or shorter than the allowance is carried into the next one (Sec. 4.3)
  * dynamic chunking        tokens are taken from a prompt until the budget or the KVC is used up;
                            the prompt is cut wherever that happens               (Sec. 4.2)
  * one long prompt at a time: a new long prompt does not start while another is being
                            processed                                            (Sec. 4.2)
  * KVC demand D_m          first chunk / whole prompt: ceil(S_l / b) * b; later chunk: only the
                            tokens that do not fit the last block's free slots; generation task:
                            0 if its last block has room, else b                  (Sec. 4.4)
  * batching                Alg. 1 (urgent requests first, preempt the largest T_r while a resource
                            is over-committed, then SelectRequests) and Alg. 2 (candidates within
                            gamma of the first non-urgent T_r; repeatedly take the candidate whose
                            (D_c, D_m) is nearest to the available (A_c, A_m))     (Sec. 4.4)

Readings where the paper is silent are listed in the design notes of the repository; the ones that
shape this file: SLO_min is the smallest SLO among the queue head, the generation tasks returning
from the last iteration and the urgent requests; generation tasks returning from the last
iteration stay in the batch; a victim that is a prompt chunk is shortened before it is dropped; a
generation task preempted for KVC gives its blocks back and re-enters as a prompt over all its
tokens (recompute) -- or, when a swap pool is configured and has room, moves them there and
copies them back into fresh blocks when it is scheduled again --, one preempted for the token
budget keeps them; L_c is the mean length of the
chunks formed so far (S_pf before the first); a prompt is long if it exceeds S_pf; a long prompt
that may not begin yet is skipped when the candidates are drawn, and one in progress is always a
candidate; distances are compared as exact integers (squared), ties go to the earlier queue
position.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

# prompt (new / partly processed / recompute), TG back from the last iteration, TG set aside with its
# blocks, TG set aside with its blocks moved to the swap pool
WAITING, RETURNED, PREEMPTED, SWAPPED = 0, 1, 2, 3


@dataclass
class Request:
    id: int
    prompt_len: int        # tokens to run as prompt (grows when a generation task is recomputed)
    max_new: int           # tokens still to be produced once the prompt is done, including the prompt's own
    slo_first: float       # seconds allowed until the prompt's token
    slo_token: float       # seconds allowed per generated token
    t_enter: float
    processed: int = 0     # prompt tokens whose K/V are in the cache
    generated: int = 0     # tokens produced so far (the prompt's counts)
    state: int = WAITING
    started: bool = False
    blocks: list = field(default_factory=list)
    t_r: float = 0.0
    offline: bool = False  # has a JCT SLO instead of per-token SLOs
    allowance: float = 0.0 # waiting time allowed per iteration, fixed when the request arrives
    carry: float = 0.0     # unused (+) or overdrawn (-) waiting time of the iterations so far
    swap: list = field(default_factory=list)   # its blocks in the swap pool while it is swapped out

    @property
    def is_prompt(self):
        return self.state == WAITING

    @property
    def context(self):     # tokens whose K/V are in the cache: a generation task has not fed its newest token yet
        return self.processed if self.state == WAITING else self.prompt_len + self.generated - 1


@dataclass
class Entry:
    req: Request
    tokens: int
    new_blocks: int


class Scheduler:
    def __init__(self, block_size, num_blocks, pivot_forward_size, pivot_time, max_batch_time, gamma,
                 max_batch_tokens, block_order=None, preempt_max_time=0.0, preempt_probability=0.0, swap_blocks=0):
        self.swap_free = list(range(int(swap_blocks)))[::-1]   # a stack like the main pool's
        self.swap_out, self.swap_in = [], []                   # (from, to) block pairs of the last decision
        self._has_swap = int(swap_blocks) > 0
        self.p_max, self.p_prob = float(preempt_max_time), float(preempt_probability)
        self.b, self.nb = int(block_size), int(num_blocks)
        self.s_pf, self.t_pf, self.t_max, self.gamma = int(pivot_forward_size), float(pivot_time), float(max_batch_time), float(gamma)
        self.max_tokens = int(max_batch_tokens)
        order = list(range(self.nb)) if block_order is None else [int(x) for x in block_order]
        assert sorted(order) == list(range(self.nb))
        self.free = order[::-1]            # a stack: the next block handed out is the last element
        self.reqs = {}                     # live requests by id, in order of arrival
        self.chunk_tokens, self.chunks = 0, 0
        self.batch = []
        self.token_budget = 0
        self.preempted_now = []

    # ---- Sec. 4.4, KVC demand (in blocks) of `tokens` more tokens of a request
    def new_blocks(self, r: Request, tokens: int) -> int:
        return max(0, -(-(r.context + tokens) // self.b) - len(r.blocks))

    def fit_tokens(self, r: Request, free_blocks: int) -> int:
        return (len(r.blocks) + free_blocks) * self.b - r.context

    def add_request(self, rid, prompt_len, max_new, slo_first, slo_token, now):
        if rid in self.reqs or prompt_len < 1 or max_new < 1 or prompt_len + max_new - 1 > self.nb * self.b:
            raise ValueError("bad request")
        self.reqs[rid] = Request(rid, int(prompt_len), int(max_new), float(slo_first), float(slo_token), float(now))

    def add_offline_request(self, rid, prompt_len, max_new, predicted_new, slo_jct, now):
        """Sec. 4.3, SLOs of offline applications: predicted_new is S_g, the estimated number of
        tokens the request will generate."""
        self.add_request(rid, prompt_len, max_new, 0.0, 0.0, now)
        r = self.reqs[rid]
        n_ck = math.ceil(r.prompt_len / self.mean_chunk())
        per_token = self.t_max + self.p_max * self.p_prob
        t_e = n_ck * self.t_max + predicted_new * per_token
        r.offline, r.allowance = True, (slo_jct - t_e) / (n_ck + predicted_new)

    def mean_chunk(self) -> float:
        return float(self.s_pf) if self.chunks == 0 else self.chunk_tokens / self.chunks

    def remaining_time(self, r: Request, now: float) -> float:
        if r.offline:
            # what is left of this iteration's allowance (a returned task has not waited yet)
            waited = 0.0 if r.state == RETURNED else now - r.t_enter
            return (r.allowance + r.carry) - waited
        if r.state == WAITING:
            n_ck = math.ceil((r.prompt_len - r.processed) / self.mean_chunk())
            return (r.slo_first - (now - r.t_enter)) - n_ck * self.t_max
        if r.state == RETURNED:
            return (r.slo_token - 0.0) - 1 * self.t_max
        return (r.slo_token - (now - r.t_enter)) - 1 * self.t_max

    def slo_of(self, r: Request) -> float:
        """The iteration-level SLO that enters Eq. 6: an offline request's is its allowance plus
        the execution of one batch."""
        if r.offline:
            return r.allowance + self.t_max
        return r.slo_first if r.is_prompt else r.slo_token

    def is_long(self, r: Request) -> bool:
        return r.prompt_len > self.s_pf

    # ---- one scheduling decision (Alg. 1)
    def next_batch(self, now: float):
        live = list(self.reqs.values())
        self.batch, self.preempted_now = [], []
        self.swap_out, self.swap_in = [], []
        if not live:
            self.token_budget = 0
            return self.batch
        for r in live:
            r.t_r = self.remaining_time(r, now)
        order = sorted(live, key=lambda r: (r.t_r, r.id))
        # SLO_min of Eq. 6: over the requests that are in the batch whatever is selected later (tasks
        # back from the last iteration, urgent requests) and the head of the queue
        certain = [r for r in order if r.state == RETURNED or r.t_r <= self.t_max]
        slo_min = min(self.slo_of(r) for r in [order[0]] + certain)
        s_b = int(math.floor(self.s_pf * slo_min / self.t_pf))
        s_b = max(1, min(s_b, self.max_tokens))
        self.token_budget = s_b
        batch = self.batch

        def s_f():
            return sum(e.tokens for e in batch)

        def need():
            return sum(e.new_blocks for e in batch)

        # generation tasks of the last iteration stay
        for r in order:
            if r.state == RETURNED:
                batch.append(Entry(r, 1, self.new_blocks(r, 1)))
        # urgent requests enter first (Alg. 1, its opening step)
        for r in order:
            if r.state != RETURNED and r.t_r <= self.t_max:
                t = min(r.prompt_len - r.processed, s_b) if r.is_prompt else 1
                batch.append(Entry(r, t, self.new_blocks(r, t)))
        # over-committed: the request with the largest T_r gives way, until the batch fits (Alg. 1, the preemption loop)
        while s_f() > s_b or need() > len(self.free):
            victim = max(batch, key=lambda e: (e.req.t_r, e.req.id))
            r = victim.req
            others_tokens, others_blocks = s_f() - victim.tokens, need() - victim.new_blocks
            if r.is_prompt:
                fit = min(victim.tokens, s_b - others_tokens, self.fit_tokens(r, len(self.free) - others_blocks))
                if fit >= 1 and fit < victim.tokens:
                    victim.tokens, victim.new_blocks = fit, self.new_blocks(r, fit)
                    continue
                batch.remove(victim)
            else:
                kvc_short = need() > len(self.free)
                batch.remove(victim)
                self.preempt(r, now, release=kvc_short)
        # fill what is left by multi-resource selection (Alg. 1, its last step: Alg. 2)
        a_c = s_b - s_f()
        a_m = len(self.free) - need()          # in blocks
        if a_c > 0:
            self.select_requests(a_c, a_m, order)
        # blocks are handed out in batch order; chunk statistics feed L_c
        for e in batch:
            r = e.req
            if r.offline:
                # the iteration starts now: what it under- or over-used of its allowance moves on
                waited = 0.0 if r.state == RETURNED else now - r.t_enter
                r.carry = (r.allowance + r.carry) - waited
            for _ in range(e.new_blocks):
                e.req.blocks.append(self.free.pop())
            if r.state == SWAPPED:
                # back in: its content returns into the first of its fresh blocks, in order
                for i, sb in enumerate(r.swap):
                    self.swap_in.append((sb, r.blocks[i]))
                    self.swap_free.append(sb)
                r.swap, r.state = [], PREEMPTED
            if e.req.is_prompt:
                e.req.started = True
                self.chunk_tokens += e.tokens
                self.chunks += 1
        return batch

    def preempt(self, r: Request, now: float, release: bool):
        self.preempted_now.append(r.id)
        r.t_enter = now
        if r.state == SWAPPED:
            return                       # it holds nothing here; it simply does not get in
        if release and self._has_swap and len(r.blocks) <= len(self.swap_free):
            # swap: its blocks move to the other pool and are free here
            for blk in r.blocks:
                sb = self.swap_free.pop()
                self.swap_out.append((blk, sb))
                r.swap.append(sb)
                self.free.append(blk)
            r.blocks, r.state = [], SWAPPED
            return
        if release:
            # recompute: everything it holds goes back, all its tokens become a prompt again
            for blk in r.blocks:
                self.free.append(blk)
            r.blocks = []
            r.prompt_len = r.prompt_len + r.generated   # its prompt and every token produced so far
            r.max_new = r.max_new - r.generated         # the recomputed prompt yields the next one
            r.processed, r.generated, r.state, r.started = 0, 0, WAITING, False
        else:
            r.state = PREEMPTED

    # ---- Alg. 2
    def select_requests(self, a_c: int, a_m: int, order):
        in_batch = {e.req.id for e in self.batch}

        def long_in_progress(r):
            return self.is_long(r) and r.is_prompt and r.started and r.processed < r.prompt_len

        long_busy = any(long_in_progress(r) or (self.is_long(r) and r.is_prompt and r.id in in_batch)
                        for r in self.reqs.values())

        def blocked(r):       # a long prompt that has not begun, while another is being processed
            return r.is_prompt and self.is_long(r) and not r.started and long_busy

        rest = [r for r in order if r.id not in in_batch and r.id not in self.preempted_now]
        eligible = [r for r in rest if not blocked(r)]
        if not eligible:
            return
        t_r1 = eligible[0].t_r
        # within gamma of the first; a long prompt in progress is always considered, so that it ends
        cands = [r for r in eligible if r.t_r <= t_r1 + self.gamma or long_in_progress(r)]
        while True:
            best = None
            for pos, r in enumerate(cands):
                if blocked(r):
                    continue
                if r.is_prompt:
                    d_c = min(r.prompt_len - r.processed, a_c, self.fit_tokens(r, a_m))
                    if d_c < 1:
                        continue
                else:
                    d_c = 1
                d_blocks = self.new_blocks(r, d_c)
                if d_c > a_c or d_blocks > a_m:
                    continue
                dist2 = (a_c - d_c) ** 2 + ((a_m - d_blocks) * self.b) ** 2
                if best is None or dist2 < best[0]:
                    best = (dist2, pos, r, d_c, d_blocks)
            if best is None:
                return
            _, pos, r, d_c, d_blocks = best
            self.batch.append(Entry(r, d_c, d_blocks))
            cands.pop(pos)
            if r.is_prompt and self.is_long(r):
                long_busy = True
            a_c -= d_c
            a_m -= d_blocks

    # ---- the arrays the attention path takes for this batch
    def batch_arrays(self):
        ids, chunk_starts, context_lens, slot_map, tables = [], [0], [], [], []
        for e in self.batch:
            r = e.req
            prior = r.context
            ids.append(r.id)
            chunk_starts.append(chunk_starts[-1] + e.tokens)
            context_lens.append(prior + e.tokens)
            for pos in range(prior, prior + e.tokens):
                slot_map.append(r.blocks[pos // self.b] * self.b + pos % self.b)
            tables.append(list(r.blocks[: -(-(prior + e.tokens) // self.b)]))
        return ids, chunk_starts, context_lens, slot_map, tables

    def batch_swaps(self):
        """Block copies this decision asks for, as (source, destination) pairs: first those out of
        the cache pool into the swap pool, then those back in.  All of them come before the
        iteration's append; the ones out before the ones in (a block given up may be handed to a
        returning request in the same decision)."""
        return list(self.swap_out), list(self.swap_in)

    # ---- the iteration has run
    def complete(self, now: float):
        finished = []
        for e in self.batch:
            r = e.req
            if r.is_prompt:
                r.processed += e.tokens
                if r.processed == r.prompt_len:
                    r.generated, r.state = 1, RETURNED
                elif r.offline:
                    r.t_enter = now      # the next chunk's iteration waits from here
            else:
                r.generated += 1
                r.state = RETURNED
            if r.state == RETURNED and r.generated >= r.max_new:
                finished.append(r.id)
        for rid in finished:
            r = self.reqs.pop(rid)
            for blk in r.blocks:
                self.free.append(blk)
        self.batch = []
        return finished


def sequential_chunks(lengths, budgets, kvc_tokens):
    """Sec. 4.2, dynamic chunking on its own: prompts of the given lengths wait in order; iteration j
    may take budgets[j] tokens and has room for kvc_tokens[j] tokens in the cache.  Returns, per
    iteration, the list of (prompt index, tokens taken)."""
    left = list(lengths)
    out = []
    for budget, room in zip(budgets, kvc_tokens):
        take_total = min(budget, room)
        picks = []
        for i, n in enumerate(left):
            if take_total == 0:
                break
            if n == 0:
                continue
            t = min(n, take_total)
            picks.append((i, t))
            left[i] -= t
            take_total -= t
        out.append(picks)
    return out
