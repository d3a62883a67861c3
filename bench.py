#!/usr/bin/env python3
"""Benchmark of the mixed-batch paged-attention hot path on one MI355X.

A step = one pass of the whole hot path over one synthetic batch: kv_append of the iteration's
new K/V followed by mixed_paged_attention (work-list planning and upload included), with all
tensors already resident in HBM.  Default workload: the OPT-13B-shaped mixed batch (one
512-token prompt chunk + 48 generation rows, 40 heads x 128, block size 16).

Prints ONE JSON line: metric / value / unit (tokens/s of the whole step), ms_per_step, the
workload in `config`, and the objects below.  `roofline` describes the attention
kernel of the mixed step (HBM bound: the generation rows dominate); `roofline_tg` and
`roofline_pp` are the same kernel timed on the generation-only and prompt-only parts of the
batch, against the HBM and bf16 matrix-core peaks respectively; `cpu_baseline` is the fp64
oracle timed on the host cores on a sample of the same batch.  Other workloads (--workload): cfg1,
cfg2, cfg3:p<prior>, cfg4, cfg5[:iteration], gqa, gqa-decode, <cfg>@bs32|64|128, <cfg>@fp16, held:<name> (scheduler-shaped
batches no planner constant was fitted on), sched13b (batches formed by the scheduler from a Poisson trace), swap13b
(block copies).  Modes: --clocks (the clock sustained under each part), --ceilings (the library's micro-kernels: what this machine reaches), --planner-sweep (the planner's
choices against a grid of forced ones), --only-part tg|pp, --fuse-append (the step's append inside the attention launch).
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16 matrix, published
PART_REPEAT = 8   # launches between one pair of timing events when a part of the batch is timed alone


def csrc_digest() -> str:
    """Content hash of the kernel and planner sources: stored with every HBM-traffic figure taken
    from a profiler run, so that a figure measured on other sources is recognised as stale."""
    import hashlib
    h = hashlib.sha256()
    for name in ("kernels.hip", "planner.cpp", "mpa_internal.h"):
        with open(os.path.join(ROOT, "paper_2503_13737_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def measure_ceilings(mpa, full: bool = False) -> dict:
    """What plain micro-kernels of the library reach on this machine, measured now: a streaming
    non-temporal read, matrix instructions back to back from registers and, with `full`, reads of
    randomly placed 4 KiB and 16 KiB chunks (the access pattern of a paged cache)."""
    import torch
    nbytes = 4 << 30
    buf = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    kinds = [("stream_read_GBs", mpa.MPA_CEIL_STREAM_READ, 0, 1e9), ("mfma_bf16_TFLOPs", mpa.MPA_CEIL_MFMA_BF16, 2000, 1e12),
             ("mfma_bf16_noisy_operands_TFLOPs", mpa.MPA_CEIL_MFMA_BF16_NOISY, 20000, 1e12)]   # long enough for the clock to settle
    if full:
        kinds += [("random_4KiB_GBs", mpa.MPA_CEIL_RANDOM_4K, 32, 1e9), ("random_16KiB_GBs", mpa.MPA_CEIL_RANDOM_16K, 8, 1e9)]
    out = {}
    for name, kind, iters, unit in kinds:
        mpa.ceiling_launch(kind, buf, nbytes, iters, sink)
        torch.cuda.synchronize()
        best = 0.0
        for _ in range(3):
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]   # the launches go to torch's current stream
            ev[0].record()
            work = sum(mpa.ceiling_launch(kind, buf, nbytes, iters, sink) for _ in range(5))
            ev[1].record()
            torch.cuda.synchronize()
            best = max(best, work / (ev[0].elapsed_time(ev[1]) * 1e-3) / unit)
        out[name] = best
    del buf
    torch.cuda.empty_cache()
    return out


class ClockSampler:
    """Shader clock of GPU 0 as rocm-smi reports it, sampled from a thread while a load runs."""

    def __init__(self, period_s: float = 0.2):
        import threading
        self.period, self.mhz, self._stop = period_s, [], threading.Event()
        self._thread = threading.Thread(target=self._run, daemon=True)

    def _run(self):
        import re, subprocess
        while not self._stop.is_set():
            try:
                r = subprocess.run(["rocm-smi", "--showclocks", "--json"], capture_output=True, text=True, timeout=20)
                card = json.loads(r.stdout)
                card = card[sorted(card)[0]]
                for k, v in card.items():
                    if "sclk" in k.lower() and "speed" in k.lower():
                        self.mhz.append(float(re.findall(r"[0-9.]+", str(v))[0]))
            except Exception:   # no tool, no permission, other output: the mode then reports no clock
                pass
            self._stop.wait(self.period)

    def __enter__(self):
        self._thread.start()
        return self

    def __exit__(self, *exc):
        self._stop.set()
        self._thread.join()

    def summary(self) -> dict:
        v = self.mhz[1:] or self.mhz    # the first sample may predate the load
        return {"samples": len(v), "mean_mhz": float(np.mean(v)) if v else None, "min_mhz": float(np.min(v)) if v else None,
                "max_mhz": float(np.max(v)) if v else None}


def run_clocks(args, mpa, b):
    """--clocks: the clock the chip sustains under each part of the workload.  Each load runs for a few
    seconds (the power management needs milliseconds to settle, the sampling tool a fraction of a second per
    reading).  The prompt part also runs on all-zero q / K / V: the same launch, the same instructions, operands
    that toggle nothing -- the difference to the seeded data is what the chip's power management takes."""
    import torch
    dw = DeviceWorkload(b, mpa)
    seconds = 4.0
    rows = []

    def load(label, fn, work=None, unit=None):
        fn()
        torch.cuda.synchronize()
        n, t0 = 0, time.perf_counter()
        with ClockSampler() as cs:
            while time.perf_counter() - t0 < seconds:
                for _ in range(20):
                    fn()
                torch.cuda.synchronize()
                n += 20
            el = time.perf_counter() - t0
        row = {"load": label, "ms_per_call": el / n * 1e3, "calls": n, "sclk": cs.summary()}
        if work:
            row["rate"] = work / (el / n) / unit[1]
            row["unit"] = unit[0]
        rows.append(row)

    tg = [i for i in range(b.S) if b.q_lens[i] == 1]
    pp = [i for i in range(b.S) if b.q_lens[i] > 1]
    def parts(suffix):
        if pp:
            sub, q, out, ws = sub_batch(dw, pp)
            load("prompt chunks only" + suffix, lambda: dw.attention_only(sub, q, out, ws), algorithmic_flops_pp(b, pp), ("TFLOP/s", 1e12))
        if tg:
            sub2, q2, out2, ws2 = sub_batch(dw, tg)
            load("generation rows only" + suffix, lambda: dw.attention_only(sub2, q2, out2, ws2), algorithmic_bytes(b, tg), ("GB/s", 1e9))
        if tg and pp:
            load("mixed" + suffix, lambda: dw.ctx.mixed_paged_attention(dw.q, dw.k_cache, dw.v_cache, dw.block_table, b.chunk_starts,
                                                                          b.context_lens, dw.out, dw.ws, scale=b.scale))

    parts("")
    if pp:
        dw.k_cache.zero_(); dw.v_cache.zero_(); dw.q.zero_()     # (the workload is not used again)
        parts(", all-zero q/K/V")
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    for label, kind in (("matrix instructions from registers", mpa.MPA_CEIL_MFMA_BF16),
                        ("matrix instructions from registers, noisy operands", mpa.MPA_CEIL_MFMA_BF16_NOISY)):
        w = mpa.ceiling_launch(kind, None, 0, 4000, sink)
        load(label, lambda: mpa.ceiling_launch(kind, None, 0, 4000, sink), w, ("TFLOP/s", 1e12))
    print(json.dumps({"clocks_under_load": rows, "workload": b.name, "nominal_mhz": 2400,
                      "note": "wall time per call over back-to-back calls (launch gaps included); sclk from rocm-smi --showclocks"}), flush=True)


def stored_mfma_busy(workload: str) -> dict:
    """Matrix-pipe utilisation of the prompt part from the profiler's counters (a stored figure, like `traffic`:
    counters need a profiler run of their own): busy cycles of the matrix pipe over the cycles the compute
    units were busy.  Counts only if it was taken on the kernel sources this library is built from."""
    path = os.path.join(ROOT, "profiles", "mfma_busy.json")
    if not os.path.exists(path):
        return {"mfma_pipe_busy": None, "mfma_pipe_busy_note": "no counter run stored"}
    rec = json.load(open(path))
    v = rec.get("mfma_busy_over_cu_busy", {}).get(workload)
    if v is None:
        return {"mfma_pipe_busy": None, "mfma_pipe_busy_note": "no counter run stored for this workload"}
    if rec.get("csrc_digest") != csrc_digest():
        return {"mfma_pipe_busy": None, "mfma_pipe_busy_note": f"stale: the stored figure ({v:.3f}) was taken on other kernel sources"}
    return {"mfma_pipe_busy": v, "mfma_pipe_busy_note": "SQ_VALU_MFMA_BUSY_CYCLES / (4 x SQ_BUSY_CU_CYCLES), rocprofv3 counters on these "
                                                        f"sources ({rec['source']}); in cycles, whatever clock the chip held"}


def spread(ms) -> dict:
    """Median and 10th / 90th percentile of the sampled kernel durations."""
    p10, p50, p90 = (float(x) for x in np.percentile(ms, [10, 50, 90]))
    return {"kernel_ms_p10": p10, "kernel_ms_p50": p50, "kernel_ms_p90": p90}


def make_workload(name: str):
    import workloads as W
    if name.endswith("@fp16"):   # the same batch with IEEE-half storage (the paper's precision)
        base = name[: -len("@fp16")]
        makers = {"cfg1": W.config1, "cfg2": W.config2, "cfg3": W.config3, "cfg4": W.config4}
        if base in makers:
            return makers[base](dtype="fp16")
        if base.startswith("cfg5"):
            return W.config5(int(base.split(":")[1]) if ":" in base else 47, dtype="fp16")
        raise SystemExit(f"unknown workload {name}")
    if name.startswith(("cfg2@bs", "cfg3@bs")):   # the same batch on KV blocks of 32, 64, 128 tokens
        bs = int(name.split("@bs")[1])
        return W.config2(bs) if name.startswith("cfg2") else W.config3(bs=bs)
    if name.startswith("held:"):     # scheduler-shaped batches kept out of every fit (see workloads.held_out)
        return W.held_out(name[len("held:"):])
    if name == "cfg3":
        return W.config3()
    if name.startswith("cfg3:p"):    # the same batch with the prompt chunk at a chosen prior context
        return W.config3(prior=int(name[len("cfg3:p"):]))
    if name == "cfg2":
        return W.config2()
    if name == "cfg4":
        return W.config4()
    if name == "cfg1":
        return W.config1()
    if name == "gqa":
        return W.config_gqa()
    if name == "gqa-decode":
        return W.config_gqa_decode()
    if name.startswith("cfg5"):
        it = int(name.split(":")[1]) if ":" in name else 47
        return W.config5(it)
    raise SystemExit(f"unknown workload {name}")


class DeviceWorkload:
    """Device-resident tensors of a batch; only referenced blocks of the pool are generated."""

    def __init__(self, b, mpa, chunk_blocks: int = 512):
        import torch
        self.b = b
        self.mpa = mpa
        dev = "cuda"
        shape = (b.NB, b.HK, b.bs, b.D)
        self.k_cache = torch.full(shape, 0x7FFF, dtype=torch.int16, device=dev)
        self.v_cache = torch.full(shape, 0x7FFF, dtype=torch.int16, device=dev)
        ids = b.referenced_blocks()
        for s in range(0, len(ids), chunk_blocks):
            part = ids[s : s + chunk_blocks]
            idx = torch.from_numpy(part).to(dev)
            for which, dst in (("k", self.k_cache), ("v", self.v_cache)):
                blk = b.blocks_state(which, part, "prior")
                dst.index_copy_(0, idx, torch.from_numpy(blk.view(np.int16)).to(dev))
        kn, vn = b.new_kv()
        self.k_new = torch.from_numpy(kn.view(np.int16)).to(dev)
        self.v_new = torch.from_numpy(vn.view(np.int16)).to(dev)
        self.slot_map = torch.from_numpy(b.slot_map).to(dev)
        self.q = torch.from_numpy(b.q.view(np.int16)).to(dev)
        self.block_table = torch.from_numpy(np.ascontiguousarray(b.block_table)).to(dev)
        self.out = torch.zeros((b.T, b.H, b.D), dtype=torch.int16, device=dev)
        self.ctx = mpa.Context(b.H, b.D, block_size=b.bs, num_kv_heads=b.HK,
                               dtype=mpa.MPA_FP16 if b.dtype == "fp16" else mpa.MPA_BF16)
        # every timed step plans its batch anew, as the first layer of a model iteration does
        # (the library would otherwise reuse the work list of the identical previous call)
        self.ctx.set_option(mpa.MPA_OPT_PLAN_CACHE, 0)
        self.ws = torch.empty(self.ctx.workspace_bytes_for_batch(b.chunk_starts, b.context_lens),
                              dtype=torch.uint8, device=dev)

    def step(self):
        b = self.b
        # kv_append + mixed_paged_attention through the library's one-call form
        self.ctx.append_and_attend(self.k_new, self.v_new, self.slot_map, self.q, self.k_cache, self.v_cache,
                                   self.block_table, b.chunk_starts, b.context_lens, self.out, self.ws, scale=b.scale)

    def attention_only(self, sub, q_rows, out, ws):
        """Attention over a sub-batch (sequence subset) sharing this workload's cache."""
        self.ctx.mixed_paged_attention(q_rows, self.k_cache, self.v_cache, sub["table"], sub["cs"],
                                       sub["ctx"], out, ws, scale=self.b.scale)


def algorithmic_bytes(b, seqs=None) -> int:
    """HBM bytes the attention step must move: every K and V element of every sequence's context
    once (4*D bytes per token per K/V head, K and V in bf16), plus q in and out out."""
    sel = np.arange(b.S) if seqs is None else np.asarray(seqs)
    kv_tokens = int(b.context_lens[sel].sum())
    rows = int(b.q_lens[sel].sum())
    return kv_tokens * 4 * b.D * b.HK + rows * b.H * b.D * 2 * 2


def algorithmic_flops_pp(b, seqs) -> int:
    """4*D flop per (query, key, head) pair under the causal mask (QK^T and PV)."""
    ql, pr = b.q_lens[seqs], b.priors[seqs]
    pairs = int((ql * pr + ql * (ql + 1) // 2).sum())
    return 4 * b.D * b.H * pairs


def time_kernel(dw, fn, steps, warmup, every: int = 1, repeat: int = 1):
    """Wall time of `steps` calls of fn, and the attention kernel's duration (HIP events recorded by
    the library around the launch) in every `every`-th of them.  With repeat > 1 a timed call
    launches the kernel that many times between its two events and the duration is per launch: a
    pair of events holds the queue for about ten microseconds, which would be counted into a lone
    launch (15 % of a 45 us kernel)."""
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    dw.ctx.set_option(dw.mpa.MPA_OPT_PROFILE_EVERY, every)
    dw.ctx.set_option(dw.mpa.MPA_OPT_PROFILE_REPEAT, repeat)
    dw.ctx.profile_enable(steps)
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms = dw.ctx.profile_read(steps)
    dw.ctx.profile_enable(0)
    dw.ctx.set_option(dw.mpa.MPA_OPT_PROFILE_REPEAT, 1)
    return wall, ms


def sub_batch(dw, seqs):
    import torch
    b = dw.b
    seqs = np.asarray(seqs)
    ql = b.q_lens[seqs]
    cs = np.concatenate([[0], np.cumsum(ql)]).astype(np.int32)
    rows = np.concatenate([np.arange(b.chunk_starts[i], b.chunk_starts[i + 1]) for i in seqs])
    q = dw.q[torch.from_numpy(rows).cuda()].contiguous()
    table = dw.block_table[torch.from_numpy(seqs).cuda()].contiguous()
    ctx = b.context_lens[seqs].copy()
    out = torch.zeros_like(q)
    ws = torch.empty(dw.ctx.workspace_bytes_for_batch(cs, ctx), dtype=torch.uint8, device="cuda")
    return {"cs": cs, "ctx": ctx, "table": table}, q, out, ws


def cpu_baseline(b, budget_pair_heads: float = 1.0e9):
    """The fp64 oracle, as it stands, on a bounded sample of the same batch: all generation rows
    and every k-th prompt row (all heads), k chosen so the sample is ~budget (query,key,head)
    triples.  Throughput is scaled to tokens/s of the full batch by triples visited."""
    import oracle
    ql, pr = b.q_lens, b.priors
    rows, triples_full, triples_sample = [], 0, 0
    tg = [i for i in range(b.S) if ql[i] == 1]
    pp = [i for i in range(b.S) if ql[i] > 1]
    tg_triples = int(b.context_lens[tg].sum()) * b.H if tg else 0
    pp_triples = b.pp_pairs() * b.H
    triples_full = tg_triples + pp_triples
    stride = max(1, int(np.ceil(pp_triples / max(budget_pair_heads - tg_triples, budget_pair_heads * 0.25))))
    for i in tg:
        rows.append(int(b.chunk_starts[i]))
    triples_sample += tg_triples
    for i in pp:
        js = np.arange(0, int(ql[i]), stride)
        rows.extend((int(b.chunk_starts[i]) + js).tolist())
        triples_sample += int((pr[i] + js + 1).sum()) * b.H
    rows = np.asarray(rows, dtype=np.int32)
    # compact pool holding the blocks of the whole batch after the append
    sub = b.compact(range(b.S))
    kc, vc = sub.compact_cache(b, "ctx")
    rr = np.repeat(rows, b.H)
    hh = np.tile(np.arange(b.H, dtype=np.int32), rows.size)
    t0 = time.perf_counter()
    oracle.attention_rows(sub.q, kc, vc, sub.block_table, sub.chunk_starts, sub.context_lens, b.scale, rr, hh,
                          dtype=b.dtype)
    dt = time.perf_counter() - t0
    est_full = dt * triples_full / triples_sample
    return {
        "value": b.T / est_full, "unit": "tokens/s", "cores": oracle.threads(), "kind": "oracle",
        "sample": (f"all {len(tg)} generation rows + every {stride}th prompt row, all heads: "
                   f"{triples_sample:.3g} of {triples_full:.3g} (query,key,head) triples in {dt:.1f} s; "
                   f"scaled by triples"),
    }


def run_scheduled(args, mpa):
    """Workload "sched13b": the batches come from the scheduler (include/mpa_sched.h) driven by a
    Poisson trace with the paper's length mix, on an OPT-13B-shaped layer with the paper's block
    size (32) and pivot forward size (768).  A step is one iteration: arrivals, scheduling decision,
    upload of its arrays, kv_append + mixed_paged_attention, completion.  The scheduler's clock is a
    model of the whole network's iteration time (20 ms + 30 ms per 768 tokens: T_pf = 50 ms at the
    pivot); the arrival rate puts the modelled system at 70 % load, where it reaches a steady state
    of about a hundred generation tasks next to the prompt chunks.  The cache pool holds seeded random
    values everywhere (this workload measures speed; parity on scheduled batches is a test)."""
    import torch
    import workloads as W
    H, HK, D, bs, NB = 40, 40, 128, 32, 16384
    s_pf, t_pf, gamma, max_tokens = 768, 0.05, 0.75, 4096
    n_req = 6000
    trace = W.poisson_trace(n_req, 31, rate=1.0, max_prompt=16384, max_new=2048)
    mean_tokens = float((trace["prompt_len"] + trace["max_new"]).mean())
    rate = 0.7 * (s_pf / t_pf) / mean_tokens
    trace["arrival"] = trace["arrival"] / rate
    iter_time = lambda sf: 0.02 + 0.03 * sf / s_pf
    t_max = iter_time(s_pf * 0.1875 / t_pf)   # the budget of the tightest SLO class
    order = W.permutation(NB, 31)
    dev = "cuda"
    g = torch.Generator(device=dev)
    g.manual_seed(31)
    caches = []
    for _ in range(2):
        c = torch.empty((NB, HK, bs, D), dtype=torch.bfloat16, device=dev)
        for s0 in range(0, NB, 2048):
            c[s0:s0 + 2048].normal_(generator=g)
        caches.append(c.view(torch.int16))
    k_cache, v_cache = caches
    pool = torch.empty((3, max_tokens, H, D), dtype=torch.bfloat16, device=dev).normal_(generator=g).view(torch.int16)
    q_all, k_all, v_all = pool[0], pool[1], pool[2]
    out = torch.empty((max_tokens, H, D), dtype=torch.int16, device=dev)
    ctx = mpa.Context(H, D, block_size=bs, num_kv_heads=HK)
    if args.fuse_append:
        ctx.set_option(mpa.MPA_OPT_FUSE_APPEND, 1)
    ws = {"buf": torch.empty(1 << 30, dtype=torch.uint8, device=dev)}
    sched = mpa.Scheduler(bs, NB, s_pf, t_pf, t_max, gamma, max_tokens, block_order=order)
    state = {"now": 0.0, "next": 0}

    def arrivals(sc):
        while state["next"] < n_req and trace["arrival"][state["next"]] <= state["now"]:
            i = state["next"]
            sc.add_request(i, int(trace["prompt_len"][i]), int(trace["max_new"][i]), float(trace["slo_first"][i]),
                           float(trace["slo_token"][i]), float(trace["arrival"][i]))
            state["next"] += 1

    # reach a steady state without the GPU (the pool's content is valid everywhere)
    pre = 6000
    for _ in range(pre):
        arrivals(sched)
        info = sched.next_batch(state["now"])
        state["now"] += iter_time(info.num_tokens)
        sched.complete(state["now"])
    snapshot = dict(state)

    def iteration(timed):
        t0 = time.perf_counter()
        arrivals(sched)
        info = sched.next_batch(state["now"])
        ids, cs, ctxl, slots, table = sched.batch_arrays()
        t1 = time.perf_counter()
        T = info.num_tokens
        if T:
            d_slots = torch.from_numpy(slots).to(dev, non_blocking=True)
            d_table = torch.from_numpy(table).to(dev, non_blocking=True)
            need = ctx.workspace_bytes_for_batch(cs, ctxl)
            if need > ws["buf"].numel():
                torch.cuda.synchronize()
                ws["buf"] = torch.empty(need * 2, dtype=torch.uint8, device=dev)
            ctx.append_and_attend(k_all[:T, :HK], v_all[:T, :HK], d_slots, q_all[:T], k_cache, v_cache, d_table, cs, ctxl,
                                  out[:T], ws["buf"], scale=1.0 / math.sqrt(D))
        t2 = time.perf_counter()
        state["now"] += iter_time(T)
        sched.complete(state["now"])
        t3 = time.perf_counter()
        if timed is not None:
            timed["sched_s"] += (t1 - t0) + (t3 - t2)
            timed["tokens"] += T
            timed["seqs"] += info.num_seqs
            timed["chunks"] += info.num_prompt_chunks
            timed["chunk_tokens"] += T - info.num_generation
            timed["bytes"] += int(ctxl.sum()) * 4 * D * HK + T * H * D * 4
            timed["kv_tokens"] += int(ctxl.sum())
            timed["launches"] += 1 if T else 0
            timed["live"] += sched.live_requests

    for _ in range(args.warmup):
        iteration(None)
    torch.cuda.synchronize()
    ctx.profile_enable(args.steps)
    timed = dict.fromkeys(["sched_s", "tokens", "seqs", "chunks", "chunk_tokens", "bytes", "kv_tokens", "launches", "live"], 0)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        iteration(timed)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms = ctx.profile_read(args.steps)
    ctx.profile_enable(0)
    kernel_s = float(ms.sum()) * 1e-3
    achieved = timed["bytes"] / kernel_s / 1e9
    k = args.steps
    result = {
        "metric": "scheduler-driven mixed-batch paged-attn tokens/s", "value": timed["tokens"] / wall, "unit": "tokens/s",
        "n_gpus": 1, "steps": k, "warmup": args.warmup, "ms_per_step": wall * 1e3 / k, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"sched13b: H={H} D={D} bs={bs}, pool {NB} blocks, S_pf={s_pf}, gamma={gamma}, Poisson trace at "
                               f"{rate:.2f} req/s (70 % of the modelled capacity), {pre} iterations of run-in; per iteration: "
                               f"{timed['seqs'] / k:.1f} sequences, {timed['tokens'] / k:.1f} tokens "
                               f"({timed['chunks'] / k:.2f} prompt chunks of {timed['chunk_tokens'] / max(timed['chunks'], 1):.0f} tokens), "
                               f"{timed['kv_tokens'] / k:.0f} KV tokens read, {timed['live'] / k:.0f} live requests",
                   "step": "arrivals + scheduling decision + array upload + kv_append + mixed_paged_attention + completion"},
        "scheduler": {"us_per_iteration": timed["sched_s"] * 1e6 / k, "fraction_of_step": timed["sched_s"] / wall},
        "roofline": {"kernel": "attention_kernel (scheduled batches)", "bound": "hbm", "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": None,
                     "algorithmic_bytes": timed["bytes"] / max(timed["launches"], 1), "kernel_ms": kernel_s * 1e3 / max(timed["launches"], 1)},
    }
    if not args.no_cpu_baseline:
        # the scheduler oracle over the same run-in and timed iterations (decisions only)
        from oracle import sched_oracle as SO
        o = SO.Scheduler(bs, NB, s_pf, t_pf, t_max, gamma, max_tokens, order)
        state.update(now=0.0, next=0)
        n_it, t_or = pre + args.warmup + k, 0.0
        for it in range(n_it):
            arrivals(o)
            t0 = time.perf_counter()
            batch = o.next_batch(state["now"])
            o.batch_arrays()
            state["now"] += iter_time(sum(e.tokens for e in batch))
            o.complete(state["now"])
            if it >= pre + args.warmup:
                t_or += time.perf_counter() - t0
        result["cpu_baseline"] = {"value": k / t_or, "unit": "scheduling iterations/s", "cores": 1, "kind": "oracle",
                                  "sample": f"the scheduler oracle (Python) on the same {k} timed iterations of the same trace; "
                                            f"the library takes {timed['sched_s'] * 1e6 / k:.0f} us per iteration"}
    print(json.dumps(result), flush=True)


def run_copy_blocks(args, mpa):
    """Workload "swap13b": mpa_copy_blocks moving the 2,048 scattered blocks of preempted requests
    (64 K tokens of an OPT-13B-shaped layer, block size 32) from the cache pool to a second pool.
    A step is one call; bytes = blocks x block bytes x (K and V) x (read + write)."""
    import torch
    import workloads as W
    HK, D, bs, NB, n = 40, 128, 32, 8192, 2048
    ctx = mpa.Context(HK, D, block_size=bs)
    g = torch.Generator(device="cuda")
    g.manual_seed(7)
    pool = [torch.empty((NB, HK, bs, D), dtype=torch.bfloat16, device="cuda").normal_(generator=g).view(torch.int16) for _ in range(2)]
    other = [torch.zeros((n, HK, bs, D), dtype=torch.int16, device="cuda") for _ in range(2)]
    pairs = np.stack([W.permutation(NB, 7)[:n], W.permutation(n, 8)], axis=1).astype(np.int64)
    d_pairs = torch.from_numpy(pairs).cuda()
    call = lambda: ctx.copy_blocks(pool[0], pool[1], other[0], other[1], d_pairs)
    for _ in range(args.warmup):
        call()
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]   # the calls go to torch's current stream
    t0 = time.perf_counter()
    ev[0].record()
    for _ in range(args.steps):
        call()
    ev[1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms = ev[0].elapsed_time(ev[1]) / args.steps
    by = n * HK * bs * D * 2 * 2 * 2
    ok = bool(torch.equal(other[0][d_pairs[:, 1]], pool[0][d_pairs[:, 0]]) and torch.equal(other[1][d_pairs[:, 1]], pool[1][d_pairs[:, 0]]))
    a = by / (ms * 1e-3) / 1e9
    print(json.dumps({
        "metric": "block-copy tokens/s", "value": n * bs * args.steps / wall, "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": wall * 1e3 / args.steps, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": {"workload": f"swap13b: {n} scattered blocks of {HK} heads x {bs} tokens x {D} (K and V) from a pool of {NB} "
                               f"to a second pool", "copied_correctly": ok},
        "roofline": {"kernel": "copy_blocks_kernel", "bound": "hbm", "achieved": a, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": a / HBM_PEAK_GBS, "traffic": None, "algorithmic_bytes": by, "kernel_ms": ms}}), flush=True)


def run_planner_sweep(args, mpa, b):
    """The planner's own choice of key-range length and of work-groups for the prompt tiles against
    a grid of forced values, on one batch: the attention kernel's duration per setting (median of
    the library's event timings).  Prints one JSON object with the whole table."""
    import torch
    dw = DeviceWorkload(b, mpa)
    dw.ctx.kv_append(dw.k_new, dw.v_new, dw.slot_map, dw.k_cache, dw.v_cache)
    torch.cuda.synchronize()
    has_rows = bool((b.q_lens == 1).any())
    residents = [0, 64, 128, 192, 256, 320, 384, 448] if has_rows else [0]
    splits = [0, 512, 1024, 2048, 4096, 8192, 16384]

    def measure(resident, split):
        dw.ctx.set_option(mpa.MPA_OPT_PP_RESIDENT_WGS, resident)
        dw.ctx.set_option(mpa.MPA_OPT_PP_SPLIT_TOKENS, split)
        ws = torch.empty(dw.ctx.workspace_bytes_for_batch(b.chunk_starts, b.context_lens), dtype=torch.uint8, device="cuda")
        fn = lambda: dw.ctx.mixed_paged_attention(dw.q, dw.k_cache, dw.v_cache, dw.block_table, b.chunk_starts,
                                                  b.context_lens, dw.out, ws, scale=b.scale)
        best = 1e9
        for _ in range(3):
            _, ms = time_kernel(dw, fn, 12, 3)
            best = min(best, float(np.median(ms)))
        return best

    table = {}
    for r in residents:
        for sp in splits:
            table[f"{r}/{sp}"] = measure(r, sp)
    auto = min(measure(0, 0), table["0/0"])
    table["0/0"] = auto
    best_key = min(table, key=table.get)
    print(json.dumps({"planner_sweep": b.name, "heads": b.H, "prompt_chunks": b.q_lens[b.q_lens > 1].tolist(),
                      "priors": b.priors[b.q_lens > 1].tolist(), "generation_rows": int((b.q_lens == 1).sum()),
                      "automatic_ms": auto, "best_ms": table[best_key], "best_setting_resident/split": best_key,
                      "automatic_over_best": auto / table[best_key], "table_ms": table}), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg3")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-parts", action="store_true", help="skip the generation-only / prompt-only timings")
    ap.add_argument("--only-part", choices=["tg", "pp"], default=None,
                    help="profiling aid: time ONLY the generation rows (tg) or ONLY the prompt chunks (pp) of the "
                         "workload, so that a profiler run sees one launch shape; prints that part's roofline")
    ap.add_argument("--part-repeat", type=int, default=PART_REPEAT,
                    help="launches between one pair of timing events when a part of the batch is timed alone")
    ap.add_argument("--planner-sweep", action="store_true",
                    help="time the attention kernel of the workload under the planner's own choices and under a grid of "
                         "forced key-range lengths / tile work-group counts; prints the table")
    ap.add_argument("--ceilings", action="store_true",
                    help="only measure what the library's micro-kernels reach on this machine (streaming read, random "
                         "4 KiB / 16 KiB chunk reads, matrix instructions from registers) and print them")
    ap.add_argument("--fuse-append", action="store_true",
                    help="the step's append runs inside the attention launch (MPA_OPT_FUSE_APPEND) instead of before it")
    ap.add_argument("--clocks", action="store_true",
                    help="run each part of the workload (and the matrix-instruction micro-kernels) for a few seconds and "
                         "report the shader clock the chip sustains under it (rocm-smi), plus the prompt part on all-zero data")
    ap.add_argument("--calibrate-append-tokens", type=int, default=0,
                    help="also run kv_append on this many synthetic tokens (a plain copy kernel of known size, "
                         "used to scale the HBM byte counters of a profiler run)")
    args = ap.parse_args()
    if args.gpus != 1:
        raise SystemExit("this build runs on ONE GPU: the path has no cross-GPU part; run with --gpus 1")

    import torch
    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU")
    import paper_2503_13737_amd as mpa
    mpa.load()  # fails loudly when the HIP library is missing

    if args.ceilings:
        print(json.dumps({"ceilings": measure_ceilings(mpa, full=True), "published_peaks": {"hbm_GBs": HBM_PEAK_GBS, "mfma_bf16_TFLOPs": MFMA_BF16_PEAK_TFLOPS}}), flush=True)
        return
    if args.workload == "sched13b":
        run_scheduled(args, mpa)
        return
    if args.workload == "swap13b":
        run_copy_blocks(args, mpa)
        return
    b = make_workload(args.workload)
    if args.planner_sweep:
        run_planner_sweep(args, mpa, b)
        return
    if args.clocks:
        run_clocks(args, mpa, b)
        return
    dw = DeviceWorkload(b, mpa)
    if args.fuse_append:
        dw.ctx.set_option(mpa.MPA_OPT_FUSE_APPEND, 1)
    torch.cuda.synchronize()

    if args.only_part:
        sel = [i for i in range(b.S) if (b.q_lens[i] == 1) == (args.only_part == "tg")]
        if not sel:
            raise SystemExit(f"workload has no {args.only_part} sequences")
        sub, q, out, ws = sub_batch(dw, sel)
        _, ms = time_kernel(dw, lambda: dw.attention_only(sub, q, out, ws), args.steps, args.warmup, repeat=args.part_repeat)
        t = float(ms.mean()) * 1e-3
        if args.only_part == "tg":
            by = algorithmic_bytes(b, sel)
            part = {"kernel": "attention_kernel (generation rows only)", "bound": "hbm", "achieved": by / t / 1e9,
                    "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": by / t / 1e9 / HBM_PEAK_GBS,
                    "algorithmic_bytes": by, "kernel_ms": t * 1e3}
        else:
            fl = algorithmic_flops_pp(b, sel)
            part = {"kernel": "attention_kernel (prompt chunks only)", "bound": "mfma", "achieved": fl / t / 1e12,
                    "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": fl / t / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                    "algorithmic_flops": fl, "kernel_ms": t * 1e3, **stored_mfma_busy(args.workload)}
        part["launches_per_event_pair"] = args.part_repeat
        print(json.dumps({"only_part": args.only_part, "workload": b.name, "steps": args.steps, "roofline": part}), flush=True)
        return

    # a pair of timing events costs the queue about ten microseconds, so the kernel is timed in every
    # fourth step of the timed region: 1/4 of the steps carry them
    every = 4 if args.steps >= 16 else 1
    wall, attn_ms = time_kernel(dw, dw.step, args.steps, args.warmup, every)
    ms_per_step = wall * 1e3 / args.steps
    tokens_per_s = b.T * args.steps / wall
    attn_avg_ms = float(attn_ms.mean())
    bytes_alg = algorithmic_bytes(b)
    achieved = bytes_alg / (attn_avg_ms * 1e-3) / 1e9
    # HBM bytes per launch from the profiler's counters (a stored figure: counters need a profiler
    # run of their own); it counts only if it was taken on the kernel sources this library is built from
    traffic, traffic_note = None, "no counter run stored for this workload"
    tpath = os.path.join(ROOT, "profiles", f"traffic_{args.workload.replace(':', '_')}.json")
    if os.path.exists(tpath):
        rec = json.load(open(tpath))
        if rec.get("csrc_digest") == csrc_digest():
            traffic, traffic_note = rec.get("hbm_bytes_per_launch"), f"rocprofv3 counters on these sources ({rec.get('csrc_digest')})"
        else:
            traffic_note = (f"stale: the stored figure ({rec.get('hbm_bytes_per_launch')}) was taken on other kernel sources "
                            f"({rec.get('csrc_digest')} vs {csrc_digest()})")
    ceil = measure_ceilings(mpa)

    result = {
        "metric": "mixed-batch paged-attn tokens/s", "value": tokens_per_s, "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": b.dtype,
        "data": "synthetic",
        "config": {"workload": f"{b.name}: H={b.H} D={b.D} bs={b.bs}, {int((b.q_lens > 1).sum())} prompt chunk(s) "
                               f"{b.q_lens[b.q_lens > 1].tolist()} at prior {b.priors[b.q_lens > 1].tolist()}, "
                               f"{int((b.q_lens == 1).sum())} generation rows, {b.tg_kv_tokens()} generation KV tokens",
                   "rows": b.T, "seqs": b.S, "step": "kv_append + mixed_paged_attention in the one-call form mpa_append_and_attend (plan + upload included)"
                           + ("; append inside the attention launch" if args.fuse_append else "")},
        "roofline": {"kernel": "attention_kernel (mixed)", "bound": "hbm", "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "algorithmic_bytes": bytes_alg, "kernel_ms": attn_avg_ms,
                     "traffic_note": traffic_note,
                     "kernel_ms_samples": int(attn_ms.size), **spread(attn_ms),
                     "achievable_peak": ceil["stream_read_GBs"], "frac_of_achievable": achieved / ceil["stream_read_GBs"]},
        "ceilings": {**ceil, "note": "measured in this run with the library's micro-kernels (mpa_ceiling_launch)"},
    }

    if not args.no_parts:
        tg = [i for i in range(b.S) if b.q_lens[i] == 1]
        pp = [i for i in range(b.S) if b.q_lens[i] > 1]
        if tg:
            sub, q, out, ws = sub_batch(dw, tg)
            _, ms = time_kernel(dw, lambda: dw.attention_only(sub, q, out, ws), args.steps, args.warmup, repeat=args.part_repeat)
            by = algorithmic_bytes(b, tg)
            a = by / (float(ms.mean()) * 1e-3) / 1e9
            result["roofline_tg"] = {"kernel": "attention_kernel (generation rows only)", "bound": "hbm",
                                     "achieved": a, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": a / HBM_PEAK_GBS,
                                     "algorithmic_bytes": by, "kernel_ms": float(ms.mean()), **spread(ms),
                                     "launches_per_event_pair": args.part_repeat,
                                     "achievable_peak": ceil["stream_read_GBs"], "frac_of_achievable": a / ceil["stream_read_GBs"]}
        if pp:
            sub, q, out, ws = sub_batch(dw, pp)
            _, ms = time_kernel(dw, lambda: dw.attention_only(sub, q, out, ws), args.steps, args.warmup, repeat=args.part_repeat)
            fl = algorithmic_flops_pp(b, pp)
            a = fl / (float(ms.mean()) * 1e-3) / 1e12
            result["roofline_pp"] = {"kernel": "attention_kernel (prompt chunks only)", "bound": "mfma",
                                     "achieved": a, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                                     "frac": a / MFMA_BF16_PEAK_TFLOPS, "algorithmic_flops": fl,
                                     "kernel_ms": float(ms.mean()), **spread(ms),
                                     "launches_per_event_pair": args.part_repeat,
                                     # matrix instructions back to back from registers on operands as noisy as the
                                     # batch's (the chip lowers its clock under them): what any kernel could reach here
                                     "achievable_peak": ceil["mfma_bf16_noisy_operands_TFLOPs"],
                                     "frac_of_achievable": a / ceil["mfma_bf16_noisy_operands_TFLOPs"],
                                     **stored_mfma_busy(args.workload)}
        if tg and pp:
            # how much of the two parts' time the one launch hides: 1.0 = no overlap, lower is better
            result["mixed_over_parts"] = attn_avg_ms / (result["roofline_tg"]["kernel_ms"] + result["roofline_pp"]["kernel_ms"])

    if args.calibrate_append_tokens > 0:
        n = args.calibrate_append_tokens
        assert n <= b.NB * b.bs
        kn = torch.zeros((n, b.H, b.D), dtype=torch.int16, device="cuda")
        vn = torch.ones((n, b.H, b.D), dtype=torch.int16, device="cuda")
        slots = torch.arange(n, dtype=torch.int64, device="cuda")
        kc = torch.empty((b.NB, b.H, b.bs, b.D), dtype=torch.int16, device="cuda")
        vc = torch.empty_like(kc)
        torch.cuda.synchronize()
        for _ in range(3):
            dw.ctx.kv_append(kn, vn, slots, kc, vc)
        torch.cuda.synchronize()
        result["calibration"] = {"kernel": "kv_append_kernel", "tokens": n,
                                 "bytes_read": 2 * n * b.H * b.D * 2 + n * 8,
                                 "bytes_written": 2 * n * b.H * b.D * 2}
        del kn, vn, kc, vc

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(b)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
