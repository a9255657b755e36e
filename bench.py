#!/usr/bin/env python3
"""Benchmark of the prefix-reuse prefill hot path on one MI355X.

A step = one pass of the hot path over one synthetic batch, inputs resident in HBM:
prefix-reuse prefill attention on the main stream, the paged KV append of the same
suffix on a side stream (the two touch disjoint memory and overlap; the streams are
joined before the clock stops) and, for the mixed hit/miss workload, the host->pool
page swap-in that must land first.
Prints ONE JSON line on stdout.
"""
import argparse
import ctypes
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0


def _profile_traffic(workload):
    """HBM bytes per attention launch measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE).  This
    run does not measure them: the figure is read from the committed profile summary of the same
    command for this workload (None if there is none), and the line says so."""
    rel = "profiles/attn_bf16_%s_pmc.txt" % workload
    try:
        m = re.search(r"^traffic_bytes_per_launch:\s*([0-9.eE+]+)", open(os.path.join(ROOT, rel)).read(), re.M)
        return (float(m.group(1)), "read from %s (rocprofv3 --pmc run of this command), not measured by this run" % rel) \
            if m else (None, None)
    except OSError:
        return None, None


_SIDE = None


def side_stream(torch):
    """The ONE side stream of this process.  Streams map onto a few hardware queues (4 per process
    on this machine) in creation order, so a stream made late can land on the main stream's queue and
    then runs behind it instead of beside it; this one is created first and used for every overlap."""
    global _SIDE
    if _SIDE is None:
        _SIDE = torch.cuda.Stream()
    return _SIDE


class Step:
    """Pre-marshalled C calls for one batch (marshalling only; the work is in the kernels)."""

    def __init__(self, db, torch, binding):
        b = db.b
        self.db, self.torch = db, torch
        self.lib = binding.load()
        self.shape = ctypes.byref(db.shape)
        vp = ctypes.c_void_p
        self.pl = np.ascontiguousarray(b.prefix_lens, np.int32)
        self.nl = np.ascontiguousarray(b.new_lens, np.int32)
        self.args_prefill = [vp(t.data_ptr()) for t in (db.q, db.k_new, db.v_new, db.kv_pool, db.block_table)]
        self.plp, self.nlp = vp(self.pl.ctypes.data), vp(self.nl.ctypes.data)
        self.outp = vp(db.out.data_ptr())
        self.main = torch.cuda.current_stream()
        self.side = side_stream(torch)
        self.mainp, self.sidep = vp(self.main.cuda_stream), vp(self.side.cuda_stream)
        self.join_ev = torch.cuda.Event()
        self.side.wait_stream(self.main)          # inputs were produced on the main stream

    def attention(self):
        rc = self.lib.pbkv_prefix_prefill(self.shape, *self.args_prefill, self.plp, self.nlp, self.outp, self.mainp)
        assert rc == 0, self.lib.pbkv_last_error()

    def append(self):
        a = self.args_prefill
        rc = self.lib.pbkv_append_kv(self.shape, a[1], a[2], a[3], a[4], self.plp, self.nlp, self.sidep)
        assert rc == 0, self.lib.pbkv_last_error()

    def run(self, ev0=None, ev1=None):
        """One step: the append of this batch's suffix is enqueued on the side stream and the
        attention on the main stream.  The two touch disjoint memory (attention reads the
        suffix from k_new / v_new, the append writes pool slots no attention reads), so
        neither stream waits for the other inside a step; the caller joins them before it
        stops the clock."""
        self.append()
        if ev0 is not None:
            ev0.record(self.main)
        self.attention()
        if ev1 is not None:
            ev1.record(self.main)

    def join(self):
        self.join_ev.record(self.side)
        self.main.wait_event(self.join_ev)


CLOCK_WARM_STEPS = {}


def time_config(name, steps, warmup, torch, binding, W, DeviceBatch, events=True, seed=None):
    b = W.CONFIGS[name]() if seed is None else W.CONFIGS[name](seed=seed)
    db = DeviceBatch(b)
    if b.host_pages is not None:            # make every prefix page resident before timing attention
        db.swap_in()
    st = Step(db, torch, binding)
    # the chip raises its clocks only after tens of milliseconds of load: run the step untimed until
    # about 60 ms of it have passed (CLOCK_WARM_STEPS says how many that were), then the W warm-up steps
    st.run()
    st.join()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    pre = 0
    while time.perf_counter() - t0 < 0.06:
        for _ in range(8):
            st.run()
        st.join()
        torch.cuda.synchronize()
        pre += 8
    CLOCK_WARM_STEPS[name] = pre + 1
    for _ in range(warmup):
        st.run()
    st.join()
    torch.cuda.synchronize()
    # every attention launch of the timed region is bracketed by HIP events (events=False: none is; the
    # two event packets per step cost ~6 % of a cfg1 step, reported apart as a second measurement)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) if events else (None, None)
           for k in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        st.run(*evs[k])
    st.join()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    kern_ms = float(np.mean([a.elapsed_time(c) for a, c in evs])) if events else None
    return b, db, wall, kern_ms


def swap_in_rate(db, torch, binding, reps=3):
    """Host->pool swap-in of every host-tier page of the batch, GB/s (best of reps)."""
    b = db.b
    best = None
    for _ in range(reps):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        db.swap_in()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        best = dt if best is None else min(best, dt)
    return b.host_pages.nbytes / best / 1e9, best


def append_rate(db, torch, reps=20):
    """The paged append alone (HBM roofline: algorithmic bytes = suffix K/V read once + written once)."""
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for _ in range(5):
        db.append()
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        db.append()
    e1.record()
    torch.cuda.synchronize()
    t = e0.elapsed_time(e1) * 1e-3 / reps
    nbytes = db.b.append_bytes()
    return {"workload": db.b.name, "ms": t * 1e3, "bytes": nbytes,
            "roofline": {"bound": "hbm", "kernel": "append_kernel", "achieved": nbytes / t / 1e9, "peak": PEAK_HBM_GBS,
                         "unit": "GB/s", "frac": nbytes / t / 1e9 / PEAK_HBM_GBS}}


def swap_rates(db, torch, binding):
    """Swap-in and swap-out of the batch's host-tier pages against the box's own pinned copy rates."""
    b = db.b
    gbs, secs = swap_in_rate(db, torch, binding)
    stage = torch.empty_like(db.host_pages, device="cuda")
    best = None
    for _ in range(3):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        stage.copy_(db.host_pages, non_blocking=True)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        best = dt if best is None else min(best, dt)
    del stage
    out = {"workload": b.name, "swap_in_GBps": gbs, "swap_in_bytes": int(b.host_pages.nbytes), "swap_in_ms": secs * 1e3,
           "pinned_h2d_memcpy_GBps": b.host_pages.nbytes / best / 1e9,
           "swap_in_frac_of_pinned_memcpy": gbs / (b.host_pages.nbytes / best / 1e9)}
    out.update(swap_out_rate(db, torch, binding))
    return out


def tiny_config(torch, binding, W, DeviceBatch, oracle, reps=200):
    """cfg0 (the fp32 correctness configuration): time of the fp32 kernel, and the oracle on one thread."""
    b = W.CONFIGS["cfg0"]()
    db = DeviceBatch(b)
    for _ in range(5):
        db.prefill()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        db.prefill()
    e1.record()
    torch.cuda.synchronize()
    gpu_ms = e0.elapsed_time(e1) / reps
    want = None
    n_threads = oracle.threads()
    try:
        oracle.set_threads(1)
        t0 = time.perf_counter()
        for _ in range(5):
            want = oracle.prefill(b.q, b.k_new, b.v_new, b.kv_pool, b.block_table, b.prefix_lens, b.new_lens)
        one = (time.perf_counter() - t0) / 5
    finally:
        oracle.set_threads(n_threads)
    from tests.gpu_util import to_numpy
    err = float(np.abs(W.to_f64(to_numpy(db.out)) - want).max())
    return {"workload": b.name, "gpu_ms_per_call": gpu_ms, "oracle_single_thread_ms": one * 1e3,
            "new_tokens": b.N, "max_abs_err": err}


def overlap_schedule(db, torch, binding, groups=8, reps=3):
    """Mixed hit/miss batch end to end (Sec. 4.3: transfers hidden behind compute).  The scheduler
    orders the batch by missing pages and cuts it into groups; the side stream swaps group g+1 in (one
    call per group) while the main stream attends to group g, whose pages have landed (one call per
    group over the group's slice of the packed batch); then the suffix KV is appended.  Clock: enqueue
    of the first swap-in to completion of the last attention and append.  The back-to-back order
    runs one swap-in, one attention and one append call for the whole batch."""
    b = db.b
    main, side = torch.cuda.current_stream(), side_stream(torch)
    order = np.argsort(np.diff(b.swap_offsets), kind="stable")
    off = np.concatenate([[0], np.cumsum(b.new_lens)]).astype(np.int64)
    # the batch in scheduler order: packed rows, block-table rows and lengths permuted once, outside the clock
    rows = torch.from_numpy(np.concatenate([np.arange(off[r], off[r + 1]) for r in order])).to("cuda")
    q, k_new, v_new = db.q[rows].contiguous(), db.k_new[rows].contiguous(), db.v_new[rows].contiguous()
    table = db.block_table[torch.from_numpy(order).to("cuda")].contiguous()
    pl, nl = np.ascontiguousarray(b.prefix_lens[order]), np.ascontiguousarray(b.new_lens[order])
    out = torch.empty_like(q)
    noff = np.concatenate([[0], np.cumsum(nl)]).astype(np.int64)
    cuts = [0] + [int(c[-1]) + 1 for c in np.array_split(np.arange(b.B), groups) if len(c)]
    # host pages and destination ids of every group, in scheduler order (pinned staging is the caller's)
    ids = [np.concatenate([b.swap_page_ids[b.swap_offsets[r]:b.swap_offsets[r + 1]] for r in order[lo:hi]] or [np.zeros(0, np.int32)])
           for lo, hi in zip(cuts[:-1], cuts[1:])]
    src = torch.cat([db.host_pages[int(b.swap_offsets[r]):int(b.swap_offsets[r + 1])] for r in order]).pin_memory()
    poff = np.concatenate([[0], np.cumsum([len(i) for i in ids])]).astype(np.int64)

    def attend(g):
        lo, hi = cuts[g], cuts[g + 1]
        sl = slice(int(noff[lo]), int(noff[hi]))
        binding.prefix_prefill(db.sub_shape(hi - lo), q[sl], k_new[sl], v_new[sl], db.kv_pool, table[lo:hi],
                               pl[lo:hi], nl[lo:hi], out[sl], main)

    def swap(g, stream):
        if len(ids[g]):
            binding.swap_in_pages(db.shape, src[int(poff[g]):int(poff[g + 1])], ids[g], db.kv_pool, stream)

    def run(overlapped):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        if overlapped:
            side.wait_stream(main)
            for g in range(len(cuts) - 1):
                swap(g, side)
                ev = torch.cuda.Event()
                ev.record(side)
                main.wait_event(ev)
                attend(g)
            done = torch.cuda.Event()
            done.record(main)
            side.wait_event(done)
            db.append(stream=side)
        else:
            db.swap_in(stream=main)
            db.prefill(stream=main)
            db.append(stream=main)
        torch.cuda.synchronize()
        return time.perf_counter() - t0
    run(True)
    # the grouped calls must give what the whole-batch call gives
    db.prefill()
    torch.cuda.synchronize()
    same = bool(torch.equal(out, db.out[rows]))
    seq = min(run(False) for _ in range(reps))
    ovl = min(run(True) for _ in range(reps))
    return {"end_to_end_ms_overlapped": ovl * 1e3, "end_to_end_ms_back_to_back": seq * 1e3,
            "groups": len(cuts) - 1, "grouped_output_equals_whole_batch_output": same,
            "note": "swap-in of %d pages; overlapped: one swap-in and one attention call per group; "
                    "back to back: one call each for the whole batch" % int(b.host_pages.shape[0])}


def swap_out_rate(db, torch, binding, reps=3):
    """Pool->host swap-out of the pages the batch swapped in, GB/s (best of reps), and the box's
    pinned device->host copy rate for a buffer of the same size."""
    b = db.b
    host = torch.empty_like(db.host_pages).pin_memory()
    best = None
    for _ in range(reps):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        binding.swap_out_pages(db.shape, db.kv_pool, b.swap_page_ids, host)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        best = dt if best is None else min(best, dt)
    stage = torch.empty_like(db.host_pages, device="cuda")
    ceil = None
    for _ in range(reps):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        host.copy_(stage, non_blocking=True)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        ceil = dt if ceil is None else min(ceil, dt)
    return {"swap_out_GBps": host.numel() * host.element_size() / best / 1e9, "swap_out_ms": best * 1e3,
            "pinned_d2h_memcpy_GBps": host.numel() * host.element_size() / ceil / 1e9}


def decode_rate(torch, binding, W, DeviceBatch, reps=20):
    """Paged decode attention on a pure-decode batch: the HBM-bound step behind which prefetch
    transfers are hidden.  Algorithmic bytes = every K and V row of every context once
    (+ q and out, negligible)."""
    b = W.decode_batch()
    db = DeviceBatch(b)
    out = torch.zeros_like(db.q)
    lens = np.ascontiguousarray(b.prefix_lens, np.int32)
    kv_bytes = int(lens.sum()) * 2 * b.Hkv * b.d * b.elt
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for _ in range(3):
        binding.paged_decode(db.shape, db.q, db.kv_pool, db.block_table, lens, out)
    torch.cuda.synchronize()
    times = []
    for _ in range(reps):
        e0.record()
        binding.paged_decode(db.shape, db.q, db.kv_pool, db.block_table, lens, out)
        e1.record()
        torch.cuda.synchronize()
        times.append(e0.elapsed_time(e1) * 1e-3)
    t = float(np.median(times))
    hidden = prefetch_behind_decode(db, out, lens, t, torch, binding)
    return {"prefetch_behind_decode": hidden, "workload": "decode_batch: 64 requests, contexts U{1024..16384} (%d tokens), 32/8 heads, d=128" % int(lens.sum()),
            "step_ms": t * 1e3, "min_ms": min(times) * 1e3, "kv_bytes": kv_bytes,
            "roofline": {"bound": "hbm", "achieved": kv_bytes / t / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                         "frac": kv_bytes / t / 1e9 / PEAK_HBM_GBS},
            "tokens_per_s": b.B / t}


def prefetch_behind_decode(db, out, lens, step_alone, torch, binding, steps=10):
    """Sec. 4.3: a prefetch of S_bw = Bandwidth * StepDuration bytes is meant to hide behind one
    pure-decode step.  Swap-in of that many pages runs on a side stream while the decode steps
    run on the main stream; reported: the decode step time with the transfer beside it, and the
    link rate the transfer reaches."""
    b = db.b
    page_bytes = b.page_bytes
    link = 55e9                                         # the swap-in rate measured on this machine
    n_pages = max(int(link * step_alone / page_bytes), 1)
    used = set(int(x) for r in range(b.B) for x in b.block_table[r, :-(-int(lens[r]) // b.P)])
    free = np.array([i for i in range(b.num_pages) if i not in used][:n_pages * steps], np.int32)
    n_pages = min(n_pages, len(free) // steps)
    if n_pages == 0:
        return {"error": "no free pages in the pool"}
    host = torch.empty((n_pages * steps,) + tuple(db.kv_pool.shape[1:]), dtype=db.kv_pool.dtype).pin_memory()
    side = side_stream(torch)
    main = torch.cuda.current_stream()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    s0, s1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    # the transfers alone, for comparison
    s0.record(side)
    for k in range(steps):
        binding.swap_in_pages(db.shape, host[k * n_pages:(k + 1) * n_pages], free[k * n_pages:(k + 1) * n_pages],
                              db.kv_pool, side)
    s1.record(side)
    torch.cuda.synchronize()
    t_swap_alone = s0.elapsed_time(s1) * 1e-3 / steps
    side.wait_stream(main)
    e0.record(main)
    s0.record(side)
    for k in range(steps):
        binding.swap_in_pages(db.shape, host[k * n_pages:(k + 1) * n_pages], free[k * n_pages:(k + 1) * n_pages],
                              db.kv_pool, side)
        binding.paged_decode(db.shape, db.q, db.kv_pool, db.block_table, lens, out, main)
    e1.record(main)
    s1.record(side)
    torch.cuda.synchronize()
    t_dec = e0.elapsed_time(e1) * 1e-3 / steps
    t_swap = s0.elapsed_time(s1) * 1e-3 / steps
    t_both = max(t_dec, t_swap)
    return {"pages_per_step": n_pages, "bytes_per_step": n_pages * page_bytes,
            "decode_step_ms_alone": step_alone * 1e3, "swap_in_ms_per_step_alone": t_swap_alone * 1e3,
            "decode_step_ms_with_prefetch": t_dec * 1e3,
            "swap_in_ms_per_step": t_swap * 1e3, "swap_in_GBps": n_pages * page_bytes / t_swap / 1e9,
            "back_to_back_ms": (step_alone + t_swap_alone) * 1e3,
            "hidden_fraction_of_transfer": max(0.0, min(1.0, (step_alone + t_swap_alone - t_both) / t_swap_alone)),
            "overlapped": bool(t_both < 0.9 * (step_alone + t_swap_alone))}


def policy_latency(steps=6000, warm=3000, concurrency=72):
    """Per-call latency of the policy core (host C++) on the synthetic workflow driver at the
    paper's operating point of 72 concurrent workflows (App. F, Table of scheduler overhead),
    with the reference model timed beside it on a shorter run of the same trace."""
    from paper_2605_06472_amd import policy as PC, policy_sim as SIM
    from oracle import policy_oracle as PO

    class Timed:
        def __init__(self, inner):
            self.inner, self.t = inner, {"forecast": [], "evict": [], "prefetch": []}

        def __getattr__(self, name):
            f = getattr(self.inner, name)
            if name not in self.t:
                return f
            acc = self.t[name]

            def call(*a, **k):
                t0 = time.perf_counter_ns()
                r = f(*a, **k)
                acc.append(time.perf_counter_ns() - t0)
                return r
            return call

    def run(pol, n_warm, n_steps):
        tp = Timed(pol)
        w = SIM.World(tp, capacity_pages=900, concurrency=concurrency, seed=5, horizon=3, prefetch=True)
        w.run(n_warm)
        for v in tp.t.values():
            v.clear()
        w.run(n_steps)
        nodes_per_wf = np.mean([2 + sum(len(c) for (wf, a), c in w.chains.items() if wf == x) for x in w.cur])
        return {k: float(np.mean(v)) / 1e3 for k, v in tp.t.items() if v}, float(nodes_per_wf), len(w.tier)

    core, npw, n_nodes = run(PC.Policy(6, 3, 0.7, PC.MODE_HE), warm, steps)
    p0 = PC.Policy(6, 3, 0.7, PC.MODE_HE)
    t0 = time.perf_counter_ns()
    for _ in range(20000):
        p0.retired_pages()
    call_us = (time.perf_counter_ns() - t0) / 20000 / 1e3          # cost of one call through ctypes
    model, _, _ = run(PO.PolicyOracle(6, 3, 0.7, PO.MODE_HE), 300, 300)
    return {"workload": "synthetic looped call graph, 6 agents, K=3, gamma=0.7, %d concurrent workflows, "
                        "900-page GPU tier, %d nodes tracked" % (concurrency, n_nodes),
            "forecast_refresh_us": core["forecast"], "nodes_rescored_per_refresh": npw,
            "score_update_us_per_node": max(core["forecast"] - call_us, 0.0) / npw,
            "evict_decision_us": core["evict"], "prefetch_decision_us": core["prefetch"],
            "ctypes_call_overhead_us": call_us,
            "reference_model_us": {"forecast_refresh": model["forecast"], "evict_decision": model["evict"],
                                   "prefetch_decision": model["prefetch"]},
            "paper_context_us": {"ScoreUpdate": 1.53, "EvictDecision": 440.0, "PrefetchDecision": 640.0,
                                 "note": "App. F table: Python scheduler hooks inside SGLang on the paper's host, "
                                         "HoVer+LangChain at concurrency 72; not the same trace"}}


def gather_rate(db, torch, binding, reps=5):
    """The page gather alone (pbkv_gather_probe: the attention kernel's work units, block-table
    walk and loads into LDS, no arithmetic).  Staged bytes = what the units pull into LDS
    (shared pages counted once per unit); distinct bytes = what must come from HBM at least
    once.  Warm = best of reps back to back; cold = after a 512 MiB fill that evicts L2 / MALL."""
    b = db.b
    n_units, T = binding.gather_probe(db.shape, db.k_new, db.v_new, db.kv_pool, db.block_table,
                                      b.prefix_lens, b.new_lens, None)
    buf = torch.zeros(n_units, dtype=torch.int32, device="cuda")
    row_bytes = 2 * b.d * b.elt                                   # K and V of one token, one head
    G = b.Hq // b.Hkv
    nsplit = G // min(G, 4)
    staged = 0
    for r in range(b.B):
        p, n = int(b.prefix_lens[r]), int(b.new_lens[r])
        for t0 in range(0, n, T):
            staged += (p + min(t0 + T, n)) * row_bytes * b.Hkv * nsplit
    pages = set()
    for r in range(b.B):
        pages.update(int(x) for x in b.block_table[r, :-(-int(b.prefix_lens[r]) // b.P)])
    distinct = len(pages) * b.page_bytes + b.N * row_bytes * b.Hkv
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def once():
        e0.record()
        binding.gather_probe(db.shape, db.k_new, db.v_new, db.kv_pool, db.block_table,
                             b.prefix_lens, b.new_lens, buf)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3
    once()
    warm = min(once() for _ in range(reps))
    flush = torch.empty(512 << 20, dtype=torch.uint8, device="cuda")
    cold = None
    for _ in range(3):
        flush.fill_(1)
        torch.cuda.synchronize()
        dt = once()
        cold = dt if cold is None else min(cold, dt)
    del flush
    return {"gather_units": n_units, "gather_staged_bytes": staged, "gather_distinct_bytes": distinct,
            "gather_warm_ms": warm * 1e3, "gather_cold_ms": cold * 1e3,
            "gather_staged_GBps_warm": staged / warm / 1e9, "gather_staged_GBps_cold": staged / cold / 1e9,
            "gather_distinct_GBps_cold": distinct / cold / 1e9,
            "gather_distinct_frac_of_hbm_peak_cold": distinct / cold / 1e9 / PEAK_HBM_GBS}


def predictor_rate(torch, W, reps=2000, n_x=32):
    """Forward pass of the workflow predictor (App. B) on a batch of 1024 workflow states, the
    batch the paper quotes its latency on (Sec. 4.1).  The hidden states rotate over n_x buffers
    (336 MB, more than the 256 MB of Infinity Cache) so that x comes from HBM as it would after a
    prefill.  Algorithmic bytes per batch = x + indices + probabilities + the prepared weights once."""
    from paper_2605_06472_amd import predictor as PR
    from tests.gpu_util import to_torch
    m = W.predictor_model()
    L, B = 16, 1024
    b = W.predictor_batch(m, B=B, L=L)
    shape = PR.make_shape(m.V, m.d, m.d_x, m.hidden, m.K, L)
    nbytes = PR.predictor_workspace_bytes(shape, B)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    weights = {n: to_torch(np.ascontiguousarray(getattr(m, n))) for n in PR.WEIGHT_NAMES}
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    PR.predictor_prepare(shape, weights, ws, nbytes, B)
    e1.record()
    torch.cuda.synchronize()
    prepare_ms = e0.elapsed_time(e1)
    xs = [to_torch(b.x) for _ in range(n_x)]
    cur, pre, plen = to_torch(b.cur_agent), to_torch(b.prefix), to_torch(b.prefix_len)
    probs = torch.empty((B, m.K, m.V + 1), dtype=torch.float32, device="cuda")
    for i in range(300):                             # long enough for the clocks to come up
        PR.predictor_forward(shape, ws, nbytes, B, xs[i % n_x], cur, pre, plen, B, probs)
    torch.cuda.synchronize()
    e0.record()
    for i in range(reps):
        PR.predictor_forward(shape, ws, nbytes, B, xs[i % n_x], cur, pre, plen, B, probs)
    e1.record()
    torch.cuda.synchronize()
    t = e0.elapsed_time(e1) * 1e-3 / reps
    # same buffer every time: x served by the caches
    e0.record()
    for i in range(reps):
        PR.predictor_forward(shape, ws, nbytes, B, xs[0], cur, pre, plen, B, probs)
    e1.record()
    torch.cuda.synchronize()
    t_warm = e0.elapsed_time(e1) * 1e-3 / reps
    from oracle import predictor_oracle
    t0 = time.perf_counter()
    want = predictor_oracle.forward(m, b.x, b.cur_agent, b.prefix, b.prefix_len)
    ref_ms = (time.perf_counter() - t0) * 1e3
    err = float(np.abs(probs.cpu().numpy().astype(np.float64) - want).max())
    alg = B * m.d_x * 2 + B * (L + 2) * 4 + B * m.K * (m.V + 1) * 4 + 2 * m.d * m.d_x * 2 + (m.V * m.d + m.V * m.V + 3 * m.d * m.hidden + m.hidden * (m.K * (m.V + 1) + 1) + m.K * (m.V + 1)) * 4
    flops = 2 * 2 * B * m.d * m.d_x + 2 * B * (3 * m.d * m.hidden + m.hidden * m.K * (m.V + 1))
    return {"workload": "predictor forward: %d requests, |V|=%d, d=%d, d_x=%d, hidden=%d, K=%d, %d parameters"
                        % (B, m.V, m.d, m.d_x, m.hidden, m.K, m.num_params()),
            "batch_ms": t * 1e3, "batch_ms_x_cached": t_warm * 1e3, "requests_per_s": B / t, "prepare_ms": prepare_ms,
            "max_abs_err_vs_reference": err, "reference_model_ms": ref_ms,
            "roofline": {"bound": "hbm", "achieved": alg / t / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                         "frac": alg / t / 1e9 / PEAK_HBM_GBS, "algorithmic_bytes": alg},
            "mfma_tflops": flops / t / 1e12,
            "paper_context_ms": {"PredictInfer_batch_1024": 1.56,
                                 "note": "Sec. 4.1: the paper's predictor (PyTorch, its GPUs), same batch size; widths are not published"}}


def attention_roofline(b, name, kern_ms):
    """Roofline object of the attention launch of one workload: exact FLOPs of the launch
    (4 d H_q sum_r(n_r p_r + n_r(n_r+1)/2), masked upper triangle not counted) over the average of the
    HIP-event brackets around the launches on their own stream inside the timed region."""
    flops = b.attention_flops()
    tf = flops / (kern_ms * 1e-3) / 1e12
    traffic, source = _profile_traffic(name)
    return {"bound": "mfma", "kernel": "attn_bf16_kernel", "achieved": tf, "peak": PEAK_BF16_TFLOPS,
            "unit": "TFLOP/s", "frac": tf / PEAK_BF16_TFLOPS, "flops_per_launch": flops,
            "avg_launch_ms": kern_ms, "traffic": traffic, "traffic_source": source,
            "algorithmic_bytes_per_launch": b.attention_bytes()}


def oracle_baseline(b, oracle, budget_s=12.0):
    """The oracle as it stands on this host's cores, on a bounded, evenly spaced sample of the
    suffix rows of the same batch (all query heads of each row); rows per second of that sample
    stand for new tokens per second of the batch."""
    pool = b.kv_pool if b.host_pages is None else oracle.swap_in(b.host_pages, b.swap_page_ids, b.kv_pool)
    probe = np.unique(np.linspace(0, b.N - 1, 64).astype(np.int64))
    t0 = time.perf_counter()
    oracle.prefill(b.q, b.k_new, b.v_new, pool, b.block_table, b.prefix_lens, b.new_lens, rows=probe)
    per_row = (time.perf_counter() - t0) / len(probe)
    n_rows = int(min(b.N, max(64, budget_s / per_row)))
    rows = np.unique(np.linspace(0, b.N - 1, n_rows).astype(np.int64))
    t0 = time.perf_counter()
    oracle.prefill(b.q, b.k_new, b.v_new, pool, b.block_table, b.prefix_lens, b.new_lens, rows=rows)
    dt = time.perf_counter() - t0
    p = b.prefix_lens.astype(np.int64)
    off = np.concatenate([[0], np.cumsum(b.new_lens)]).astype(np.int64)
    req = np.searchsorted(off, rows, side="right") - 1
    sample_flops = int(4 * b.d * b.Hq * np.sum(p[req] + (rows - off[req]) + 1))
    return {"value": len(rows) / dt, "unit": "new tokens/s", "cores": oracle.threads(), "kind": "oracle",
            "sample": "%d of %d suffix rows of %s, evenly spaced over the packed batch, all %d query heads, one "
                      "pass, %.1f s; the sample holds %.4f of the batch's FLOPs against %.4f of its rows, so "
                      "rows/s of the sample stand for the batch"
                      % (len(rows), b.N, b.name, b.Hq, dt, sample_flops / b.attention_flops(), len(rows) / b.N),
            "gflops_fp64": sample_flops / dt / 1e9}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--config", default="cfg4", choices=["cfg1", "cfg2", "cfg3", "cfg4"],
                    help="workload of the headline line (default: the largest one, the mixed hit/miss batch with "
                         "its pages resident)")
    ap.add_argument("--no-extra", action="store_true", help="skip the other workloads and the CPU baseline")
    ap.add_argument("--part", default=None, choices=["decode", "policy", "predictor", "swap", "gather", "append"],
                    help="run only this secondary measurement and print its JSON object (for profiling runs)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run three 256 MiB device-to-device copies (known HBM traffic) so that a "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE run of this command can be scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2605_06472_amd import binding
    from paper_2605_06472_amd import workloads as W
    from tests.gpu_util import DeviceBatch

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    side_stream(torch)                        # before any other stream exists
    import __graft_entry__
    __graft_entry__.ensure_built()            # compiles only if nothing is built yet
    binding.load()

    if args.calibrate_copy:
        src = torch.empty(64 << 20, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if args.part == "decode":
        print(json.dumps(decode_rate(torch, binding, W, DeviceBatch)))
        return
    if args.part == "policy":
        print(json.dumps(policy_latency()))
        return
    if args.part == "predictor":
        print(json.dumps(predictor_rate(torch, W)))
        return
    if args.part == "swap":
        db = DeviceBatch(W.CONFIGS["cfg4"]())
        gbs, secs = swap_in_rate(db, torch, binding)
        out = {"swap_in_GBps": gbs, "swap_in_ms": secs * 1e3, "swap_in_bytes": int(db.b.host_pages.nbytes)}
        out.update(swap_out_rate(db, torch, binding))
        print(json.dumps(out))
        return
    if args.part == "gather":
        db = DeviceBatch(W.CONFIGS["cfg3"]())
        print(json.dumps(gather_rate(db, torch, binding)))
        return
    if args.part == "append":
        db = DeviceBatch(W.CONFIGS["cfg3"]())
        print(json.dumps(append_rate(db, torch)))
        return

    b, db, wall, kern_ms = time_config(args.config, args.steps, args.warmup, torch, binding, W, DeviceBatch)
    ms_per_step = wall / args.steps * 1e3
    flops = b.attention_flops()
    line = {
        "metric": "prefix-reuse prefill new tokens/s + TFLOP/s (MFMA util %), 8B-class GQA",
        "value": b.N / (ms_per_step * 1e-3),
        "unit": "new tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": b.name, "batch": b.B, "new_tokens": b.N,
                   "prefix_lens": [int(b.prefix_lens.min()), int(b.prefix_lens.max())],
                   "new_lens": [int(b.new_lens.min()), int(b.new_lens.max())],
                   "heads_q_kv": [b.Hq, b.Hkv], "head_dim": b.d, "page_size": b.P,
                   "untimed_steps_before_the_warmup": CLOCK_WARM_STEPS.get(args.config),
                   "step": "attention (main stream) + paged append (side stream, overlapped), one layer, every "
                           "prefix page resident in the pool; the host->pool swap-in of this workload and the "
                           "overlapped schedule are timed under extra"},
        "tflops_step": flops / (ms_per_step * 1e-3) / 1e12,
        "mfma_util_step": flops / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        "roofline": attention_roofline(b, args.config, kern_ms),
        "paper_context": "PBKV end-to-end workflow latency 1.85x vs LRU and 1.26x vs KVFlow on 8x A6000 "
                         "(SGLang + HiCache, Qwen3-14B/32B); cache-policy numbers, not a kernel baseline",
    }

    if not args.no_extra:
        import oracle
        line["cpu_baseline"] = oracle_baseline(b, oracle)
        extra = {}
        rooflines = {args.config: dict(line["roofline"], ms_per_step=ms_per_step, new_tokens=b.N,
                                       new_tokens_per_s=line["value"], steps=args.steps, warmup=args.warmup)}
        try:
            extra["append"] = append_rate(db, torch)
            if b.host_pages is not None:
                extra["swap"] = swap_rates(db, torch, binding)
                extra["overlap_schedule"] = overlap_schedule(db, torch, binding)
        except Exception as e:                          # the headline line must still print
            extra["append"] = {"error": repr(e)}
        del db
        torch.cuda.empty_cache()
        for name, steps in (("cfg1", 1000), ("cfg2", 150), ("cfg3", 30), ("cfg4", 30)):
            if name == args.config:
                continue
            try:
                b2, db2, wall2, k2 = time_config(name, steps, 8, torch, binding, W, DeviceBatch)
                rooflines[name] = dict(attention_roofline(b2, name, k2), ms_per_step=wall2 / steps * 1e3,
                                       new_tokens=b2.N, new_tokens_per_s=b2.N / (wall2 / steps), steps=steps, warmup=8)
                if name == "cfg1":
                    _, dbn, walln, _ = time_config(name, steps, 8, torch, binding, W, DeviceBatch, events=False)
                    rooflines[name]["ms_per_step_without_event_packets"] = walln / steps * 1e3
                    del dbn
                if name == "cfg3":
                    extra["gather"] = gather_rate(db2, torch, binding)
                if b2.host_pages is not None and "swap" not in extra:
                    extra["swap"] = swap_rates(db2, torch, binding)
                    extra["overlap_schedule"] = overlap_schedule(db2, torch, binding)
                del db2, b2
                torch.cuda.empty_cache()
            except Exception as e:
                rooflines[name] = {"error": repr(e)}
        line["rooflines"] = rooflines
        # spread over seeds: the headline workload drawn again with seed + 100 and + 200
        try:
            seeds = {}
            base_seed = {"cfg1": 1001, "cfg2": 1002, "cfg3": 1003, "cfg4": 1004}[args.config]
            for ds in (100, 200):
                bs, dbs, walls, ks = time_config(args.config, 10, 5, torch, binding, W, DeviceBatch, seed=base_seed + ds)
                seeds[str(base_seed + ds)] = {"new_tokens": bs.N, "new_tokens_per_s": bs.N / (walls / 10),
                                              "attn_frac_of_bf16_peak": bs.attention_flops() / (ks * 1e-3) / 1e12 / PEAK_BF16_TFLOPS}
                del dbs, bs
                torch.cuda.empty_cache()
            extra["seeds"] = seeds
        except Exception as e:
            extra["seeds"] = {"error": repr(e)}
        try:
            extra["cfg0"] = tiny_config(torch, binding, W, DeviceBatch, oracle)
        except Exception as e:
            extra["cfg0"] = {"error": repr(e)}
        try:
            extra["decode"] = decode_rate(torch, binding, W, DeviceBatch)
        except Exception as e:
            extra["decode"] = {"error": repr(e)}
        try:
            extra["policy"] = policy_latency()
        except Exception as e:
            extra["policy"] = {"error": repr(e)}
        try:
            extra["predictor"] = predictor_rate(torch, W)
        except Exception as e:
            extra["predictor"] = {"error": repr(e)}
        line["extra"] = extra

    print(json.dumps(line))


if __name__ == "__main__":
    main()
