#!/usr/bin/env python3
"""Benchmark of the placement search on one MI355X.

A step is one scheduling round through the whole hot path, inputs resident in
HBM: standalone node cost -> critical path -> fused score + argmin + projected
ratio -> commit.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload large|mid|stream]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np

# The roofline of the search.  A SIMD of a compute unit issues one wave-wide fp32 vector instruction per 4 cycles
# on its main pipe (16 lanes per clock): 256 CU x 4 SIMD x 16 lanes x 2.4 GHz = 39.32 T lane-ops/s.  Additions,
# multiplications and fused multiply-adds can issue on a second fp32 pipe at the same time as an instruction of
# another wavefront on the main one (measured in calibration_leg: a stream of v_add_f32, or of v_add_f32
# alternating with v_max_f32, runs at twice the rate of a stream of v_max_f32 or v_min3_f32); the advertised
# 157.3 TFLOP/s is both pipes busy with fused multiply-adds.  Comparisons, maxima and minima have the main pipe
# only.  Per candidate the search needs one maximum, one addition and half a three-input minimum: 2.5 instructions,
# of which 1.5 are bound to the main pipe -- the resource that limits it.  achieved = candidates/s x 1.5 against
# 39.32 T main-pipe lane-ops/s; the same loop on registers alone is measured beside it.
ALU_PEAK_TOPS = 256 * 64 * 2.4e9 / 1e12
FP32_VECTOR_PEAK_TFLOPS = 157.3
MAIN_PIPE_OPS_PER_CANDIDATE = 1.5      # v_max_f32 + half a v_min3_f32
OPS_PER_CANDIDATE = 2.5                # with the v_add_f32
# Vector ops of the decode-stage search for one (call, instance) pair.  A free call goes through the instance's
# first-room table: 6 per step of the bisection for its threshold's rank, 8 per stretch of the timeline, 24 for
# the call's decode time, threshold and the comparison with its best so far.  A locked call scans its one
# instance's timeline entry by entry, 7 per entry.
DECODE_OPS_BISECT_STEP, DECODE_OPS_STRETCH, DECODE_OPS_PAIR, DECODE_OPS_ENTRY = 6.0, 8.0, 24.0, 7.0
HBM_PEAK_GBS = 8000.0


def source_sha(files):
    """sha256 over the named kernel sources: a counter summary under profiles/ names the sources it was taken on."""
    import hashlib
    h = hashlib.sha256()
    for f in files:
        h.update(open(os.path.join(ROOT, "paper_2605_16637_amd", "csrc", f), "rb").read())
    return h.hexdigest()


FUSED_SOURCES = ("hx_score.hip", "hx_search.hpp", "hx_terms.hpp", "hx_common.hpp", "hx_cp.hpp", "hx_append.hpp")
CP_SOURCES = ("hx_dag.hip", "hx_cp.hpp", "hx_append.hpp", "hx_terms.hpp", "hx_common.hpp")


def profiled_traffic(summary, sources, key="traffic_bytes_per_launch"):
    """HBM bytes per launch as the rocprofv3 counter runs summarised in profiles/<summary> found them, or None when
    there is no such line or the kernel's sources have changed since (the summary records their sha256)."""
    path = os.path.join(ROOT, "profiles", summary)
    if not os.path.exists(path):
        return None
    vals = {}
    for line in open(path):
        if ":" in line:
            k, v = line.split(":", 1)
            vals[k.strip()] = v.strip()
    if vals.get("source_sha256") != source_sha(sources) or key not in vals:
        return None
    return float(vals[key].split()[0])


def dev(x):
    import torch
    return torch.from_numpy(np.ascontiguousarray(x)).to("cuda:0")


class RoundOnDevice:
    """One synthetic round with every input and output buffer resident in HBM."""

    def __init__(self, ctx, rnd):
        import torch
        from paper_2605_16637_amd import binding
        self.ctx, self.rnd = ctx, rnd
        d = rnd.dag
        self.calls = binding.to_device(rnd.calls)
        self.pre = binding.to_device(rnd.pre)
        self.dec = binding.to_device(rnd.dec)
        self.links = binding.to_device(rnd.links)
        self.tF, self.tB = dev(rnd.types["flops"]), dev(rnd.types["hbm_bw"])
        self.L_in, self.L_out = dev(d.L_in), dev(d.L_out)
        self.row_ptr, self.col, self.wf_ptr = dev(d.succ_row_ptr), dev(d.succ_col), dev(d.wf_ptr)
        f32 = dict(dtype=torch.float32, device="cuda:0")
        i32 = dict(dtype=torch.int32, device="cuda:0")
        self.cost = torch.empty(d.n_nodes, **f32)
        self.rem = torch.empty(d.n_nodes, **f32); self.tail = torch.empty(d.n_nodes, **f32)
        self.level = torch.empty(d.n_nodes, **i32); self.hor = torch.empty(d.n_wf, **f32)
        n = rnd.calls["n"]
        self.bp = torch.empty(n, **i32); self.bd = torch.empty(n, **i32)
        self.bc = torch.empty(n, **f32); self.ratio = torch.empty(n, **f32)
        # per-round drains sized to what a round adds, so the pool stays in its regime
        P, D = rnd.pre["n"], rnd.dec["n"]
        Ls, Os = float(rnd.calls["L_in"].sum()), float(rnd.calls["L_out"].sum())
        self.drain_p = dev(np.full(P, int(Ls / max(P, 1)), np.int32))
        self.drain_q = dev(np.full(D, int(Os / max(D, 1)), np.int32))
        self.release = dev(np.full(D, int((Ls + Os) / max(D, 1)), np.int32))
        self.side = None

    def horizons(self, stream=None):
        r = self.rnd
        # node cost and critical path in one launch
        self.ctx.hx_horizons(r.model, self.row_ptr, self.col, self.L_in, self.L_out, self.tF, self.tB, self.links,
                             self.wf_ptr, self.cost, self.rem, self.tail, self.level, self.hor, stream=stream)

    def score(self):
        self.ctx.hx_score_placements(self.rnd.model, self.calls, self.pre, self.dec, self.links,
                                     tail=self.tail, horizon=self.hor,
                                     best_p=self.bp, best_d=self.bd, best_cost=self.bc, ratio=self.ratio)

    def commit(self):
        self.ctx.hx_commit(self.calls, self.bp, self.bd, self.pre["backlog_tok"], self.dec["used_tok"],
                           self.dec["batch"], self.dec["qd_tok"], self.drain_p, self.drain_q, self.release)

    def search(self):
        """The search alone: best pair and cost of every call; needs no horizon."""
        self.ctx.hx_score_placements(self.rnd.model, self.calls, self.pre, self.dec, self.links,
                                     best_p=self.bp, best_d=self.bd, best_cost=self.bc)

    def urgency(self):
        self.ctx.hx_urgency(self.calls, self.bc, self.tail, self.hor, self.ratio)

    def step(self):
        """One round, every stage on one stream."""
        self.horizons()
        self.score()
        self.commit()

    def round_call(self):
        """One round as one library call (hx_round with the round's whole graph): two launches where the round
        fits -- the horizon refresh in the search's launch, the ratio in the commit's."""
        g = dict(succ_row_ptr=self.row_ptr, succ_col_idx=self.col, wf_ptr=self.wf_ptr, L_in=self.L_in, L_out=self.L_out,
                 node_cost=self.cost, rem=self.rem, tail=self.tail, level=self.level, horizon=self.hor)
        self.ctx.hx_round(self.rnd.model, self.calls, self.pre, self.dec, self.links, self.bp, self.bd, self.bc,
                          ratio=self.ratio, type_flops=self.tF, type_hbm_bw=self.tB, drain_prefill=self.drain_p,
                          drain_decode_q=self.drain_q, release_tok=self.release, graph=g)

    def step_overlapped(self):
        """One round with the horizon refresh (node cost -> critical path) on a second stream beside the
        search, which does not need it; the urgency fold joins the two, the commit follows."""
        import torch
        main = torch.cuda.current_stream()
        if self.side is None:
            self.side = torch.cuda.Stream()          # default priority
        self.side.wait_stream(main)
        self.horizons(stream=self.side)
        self.search()
        main.wait_stream(self.side)
        self.urgency()
        self.commit()


def capture(torch, fn):
    """Records one call of fn (kernel launches only) into a HIP graph."""
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        fn()
    return g


def time_steps(torch, fn, steps, warmup):
    """Wall-clock of exactly `steps` calls of fn, synchronised on both sides."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return time.perf_counter() - t0


def time_launches(torch, fn, reps, warmup=5):
    """Average GPU time of one call of fn from HIP events on the launch stream,
    over `reps` back-to-back calls."""
    for _ in range(warmup):
        fn()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps * 1e-3


def streaming_leg(torch, ctx, synth, binding, seed, rounds, n_live=20000, C=32768, P=512, D=512):
    """Rounds of a live system, the streaming configuration at its stated length: reveal (node cost + append to the
    graph the context keeps), score the ready calls with their projected ratio, commit; pool and graph state carried
    from round to round.  Every batch is resident in HBM before its clock starts.  Four ways of enqueueing a round are
    timed on alternating rounds of the same run (they give the same results, so the state evolves as one sequence):
    its four library calls on one stream; the reveal on a second stream beside the search (which needs no horizon),
    the urgency fold joining the two before the commit; the whole round as one library call (hx_round); and that
    call with its argument block built before the clock starts, as a caller written in C has it (through the
    binding the block costs tens of microseconds of Python during which the GPU waits).
    The batches are generated a chunk of rounds ahead, so that the rounds of a chunk follow each other without a
    pause; the first two rounds after each pause for generation are run (the state is one sequence) but not timed.
    A GPU left idle for milliseconds lowers its clocks, and the round after such a pause takes longer: that figure is
    measured apart, on further rounds each preceded by 10 ms of sleep."""
    rng = np.random.default_rng(seed)
    gen = synth.StreamGen(seed, n_live)
    L0, O0 = synth.gen_lengths(rng, 50000)
    types, links, pre, dec = synth.gen_pool(rng, P, D, 8, L0, O0, near_capacity=True)
    d_links, d_pre, d_dec = binding.to_device(links), binding.to_device(pre), binding.to_device(dec)
    tF, tB = dev(types["flops"]), dev(types["hbm_bw"])
    chunk, skip, n_idle = 50, 2, 24
    n_chunks = (rounds + chunk - skip - 1) // (chunk - skip)
    total = rounds + skip * n_chunks + skip + n_idle
    # the run's whole graph stays in the context's store: at most 4 new calls per live workflow and round on average
    cap_n = int(total * n_live * 4.1) + 64 * n_live
    ctx.hx_dag_reserve(cap_n, int(cap_n * 1.35), n_live + cap_n // 10 + 1024, 32)
    i32 = dict(dtype=torch.int32, device="cuda:0")
    bp, bd = torch.empty(C, **i32), torch.empty(C, **i32)
    bc, ratio = torch.empty(C, device="cuda:0"), torch.empty(C, device="cuda:0")
    side = torch.cuda.Stream()            # default priority

    def next_batch():
        b = gen.next_batch()
        n = b["n_new"]
        pick = np.sort(rng.choice(n, min(C, n), replace=False)).astype(np.int32)
        Ls, Os = int(b["L_in"][pick].sum()), int(b["L_out"][pick].sum())
        return dict(
            n_new=n, n_wf=b["n_wf_total"], prow=dev(b["parent_row_ptr"]), pcol=dev(b["parent_col"]), wf=dev(b["wf"]),
            L_in=dev(b["L_in"]), L_out=dev(b["L_out"]), cost=torch.empty(n, device="cuda:0"),
            calls=dict(n=int(pick.size), L_in=dev(b["L_in"][pick]), L_out=dev(b["L_out"][pick]), node=dev(b["ids"][pick]),
                       wf=dev(b["wf"][pick]), elapsed=dev(rng.uniform(0, 30, pick.size).astype(np.float32))),
            drain_p=dev(np.full(P, Ls // P, np.int32)), drain_q=dev(np.full(D, Os // D, np.int32)),
            release=dev(np.full(D, (Ls + Os) // D, np.int32)))

    def one_stream(b):
        ctx.hx_node_cost(synth.MODEL, b["L_in"], b["L_out"], tF, tB, d_links, b["cost"])
        ctx.hx_dag_append(b["prow"], b["pcol"], b["cost"], b["wf"])
        _, tail, _, hor, _ = ctx.hx_dag_view(b["n_wf"])
        ctx.hx_score_placements(synth.MODEL, b["calls"], d_pre, d_dec, d_links, tail=tail, horizon=hor,
                                best_p=bp, best_d=bd, best_cost=bc, ratio=ratio)
        ctx.hx_commit(b["calls"], bp, bd, d_pre["backlog_tok"], d_dec["used_tok"], d_dec["batch"], d_dec["qd_tok"],
                      b["drain_p"], b["drain_q"], b["release"])

    def two_streams(b):
        main = torch.cuda.current_stream()
        side.wait_stream(main)
        ctx.hx_node_cost(synth.MODEL, b["L_in"], b["L_out"], tF, tB, d_links, b["cost"], stream=side)
        ctx.hx_dag_append(b["prow"], b["pcol"], b["cost"], b["wf"], stream=side)
        ctx.hx_score_placements(synth.MODEL, b["calls"], d_pre, d_dec, d_links, best_p=bp, best_d=bd, best_cost=bc)
        main.wait_stream(side)
        _, tail, _, hor, _ = ctx.hx_dag_view(b["n_wf"])
        ctx.hx_urgency(b["calls"], bc, tail, hor, ratio)
        ctx.hx_commit(b["calls"], bp, bd, d_pre["backlog_tok"], d_dec["used_tok"], d_dec["batch"], d_dec["qd_tok"],
                      b["drain_p"], b["drain_q"], b["release"])

    def one_call(b):
        ctx.hx_round(synth.MODEL, b["calls"], d_pre, d_dec, d_links, bp, bd, bc, ratio=ratio, n_wf=b["n_wf"],
                     parent_row_ptr=b["prow"], parent_col_idx=b["pcol"], new_L_in=b["L_in"], new_L_out=b["L_out"],
                     new_wf=b["wf"], new_cost=b["cost"], type_flops=tF, type_hbm_bw=tB,
                     drain_prefill=b["drain_p"], drain_decode_q=b["drain_q"], release_tok=b["release"])

    # (name, order, arguments marshalled before the clock starts: what a caller written in C sees)
    modes = (("one stream", one_stream, False), ("reveal beside the search", two_streams, False),
             ("one library call per round (hx_round)", one_call, False),
             ("hx_round, arguments marshalled ahead", one_call, True))
    lat = {name: [] for name, _, _ in modes}
    cand = {name: 0 for name, _, _ in modes}
    state = {"nodes": 0, "placed": 0, "calls": 0, "rounds": 0}

    def timed(b, fn, ahead, pause_s=0.0):
        go = ctx.prepare(lambda: fn(b)) if ahead else (lambda: fn(b))
        torch.cuda.synchronize()
        if pause_s:
            time.sleep(pause_s)
        t0 = time.perf_counter()
        go()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        state["nodes"] += b["n_new"]; state["rounds"] += 1; state["calls"] += b["calls"]["n"]
        state["placed"] += int((bp[:b["calls"]["n"]] >= 0).sum().item())
        return dt * 1e6

    done = 0
    while done < rounds:
        n = min(chunk, rounds - done + skip)
        batches = [next_batch() for _ in range(n)]
        for k, b in enumerate(batches):
            name, fn, ahead = modes[done % len(modes)]
            us = timed(b, fn, ahead)
            if k >= skip:
                lat[name].append(us)
                cand[name] += b["calls"]["n"] * P * D
                done += 1
    # after a pause: the same round on a GPU that has been idle for 10 ms
    idle = []
    batches = [next_batch() for _ in range(skip + n_idle)]
    for k, b in enumerate(batches):
        us = timed(b, one_call, True, pause_s=0.010 if k >= skip else 0.0)
        if k >= skip:
            idle.append(us)
    ctx.hx_stream_status()
    res = {}
    for name, _, _ in modes:
        x = np.array(lat[name])
        res[name] = {"rounds": int(x.size), "p50_us": float(np.percentile(x, 50)), "p99_us": float(np.percentile(x, 99)),
                     "candidates_per_s": cand[name] / (x.sum() * 1e-6)}
    best = min(res, key=lambda k: res[k]["p50_us"])
    return {"workload": "streaming rounds: %d live workflows, +0..8 calls per workflow per round, %d ready calls x %d x %d, 8 classes"
                        % (n_live, C, P, D),
            "rounds": rounds, "candidates_per_round": C * P * D, "new_nodes_per_round": state["nodes"] / state["rounds"],
            "graph_nodes_at_the_end": state["nodes"],
            "p50_us": res[best]["p50_us"], "p99_us": res[best]["p99_us"], "candidates_per_s": res[best]["candidates_per_s"],
            "order": best, "by_order": res,
            "after_10ms_idle": {"order": "hx_round, arguments marshalled ahead", "rounds": len(idle),
                                "p50_us": float(np.percentile(idle, 50)), "p99_us": float(np.percentile(idle, 99))},
            "placed_fraction": state["placed"] / max(1, state["calls"]),
            "launch": "eager, synchronised every round, rounds back to back in chunks of %d generated ahead (the first %d "
                      "of a chunk untimed); the four orders on alternating rounds of one run" % (chunk, skip)}


def planner_leg(torch, ctx, synth, binding, seed):
    """The planner around the scoring loop: the recomputing greedy plan of a small queue on pools of the
    size the paper serves (8 + 8 instances of 3 classes), and of a larger queue; one-pass ordering."""
    from oracle import hx_oracle as o
    out = {}
    rng = np.random.default_rng(seed)
    for name, C, P, D, T in (("queue 64 x pool 8+8, 3 classes", 64, 8, 8, 3), ("queue 256 x pool 64+64, 4 classes", 256, 64, 64, 4)):
        L0, O0 = synth.gen_lengths(rng, C)
        types, links, pre, dec = synth.gen_pool(rng, P, D, T if T in (2, 4) else 4, L0, O0, near_capacity=False)
        if T == 3:      # three of the four listed classes
            pre["type"] %= 3; dec["type"] %= 3
            pre["flops"], pre["hbm_bw"] = types["flops"][pre["type"]].copy(), types["hbm_bw"][pre["type"]].copy()
            dec["flops"], dec["hbm_bw"] = types["flops"][dec["type"]].copy(), types["hbm_bw"][dec["type"]].copy()
        node = np.arange(C, dtype=np.int32); wf = (np.arange(C) % 8).astype(np.int32)
        tail = rng.uniform(0, 5, C).astype(np.float32); hor = rng.uniform(10, 60, 8).astype(np.float32)
        elapsed = rng.uniform(0, 30, C).astype(np.float32)
        calls = binding.to_device(dict(n=C, L_in=L0, L_out=O0, node=node, wf=wf, elapsed=elapsed))
        dp, dd, dl = binding.to_device(pre), binding.to_device(dec), binding.to_device(links)
        i32 = dict(dtype=torch.int32, device="cuda:0")
        bufs = [torch.empty(C, **i32), torch.empty(C, **i32), torch.empty(C, device="cuda:0"), torch.empty(C, device="cuda:0"),
                torch.empty(C, **i32)]
        d_tail, d_hor = dev(tail), dev(hor)
        fn = lambda: ctx.hx_plan_greedy(synth.MODEL, calls, dp, dd, dl, d_tail, d_hor, *bufs)
        gpu_s = time_launches(torch, fn, 30)
        t0 = time.perf_counter()
        o.plan_greedy(synth.MODEL, L0, O0, elapsed, node, wf, tail, hor, pre, dec, links)
        cpu_s = time.perf_counter() - t0
        out[name] = {"gpu_us": gpu_s * 1e6, "oracle_1_thread_us": cpu_s * 1e6,
                     "candidates_if_fully_rescored": C * (C + 1) // 2 * P * D}
    ctx.hx_stream_status()
    C = 32768
    ratio = dev(rng.uniform(0.1, 9.0, C).astype(np.float32)); rank = torch.empty(C, dtype=torch.int32, device="cuda:0")
    out["one-pass ordering of 32768 calls"] = {"gpu_us": time_launches(torch, lambda: ctx.hx_rank(ratio, rank), 30) * 1e6}
    return out


def decode_leg(torch, ctx, synth, binding, seed):
    """The decode stage: one scoring pass of a large queue (16384 calls x 256 instances, ~118 intervals
    each, half the calls locked) followed by the one-pass ordering, and the recomputing greedy on pools
    of the size the paper serves."""
    from oracle import hx_oracle as o
    out = {}
    r, lock, iv = synth.make_decode_round("decode_large", seed)
    Q, D = r.calls["n"], r.dec["n"]
    q = binding.to_device(r.calls)
    dd = binding.to_device(r.dec)
    div = dict(stride=iv["stride"], count=dev(iv["count"]), start=dev(iv["start"]), end=dev(iv["end"]), tok=dev(iv["tok"]))
    d_lock = dev(lock)
    tail = torch.zeros(r.dag.n_nodes, device="cuda:0")
    hor = torch.full((r.dag.n_wf,), 30.0, device="cuda:0")
    i32 = dict(dtype=torch.int32, device="cuda:0")
    bd, rk = torch.empty(Q, **i32), torch.empty(Q, **i32)
    bs, bc, rt = (torch.empty(Q, device="cuda:0") for _ in range(3))

    def one_pass():
        ctx.hx_decode_score(synth.MODEL, q, d_lock, dd, div, bd, bs, bc, tail=tail, horizon=hor, ratio=rt)
        ctx.hx_rank(rt, rk)

    score_s = time_launches(torch, lambda: ctx.hx_decode_score(synth.MODEL, q, d_lock, dd, div, bd, bs, bc, tail=tail, horizon=hor, ratio=rt), 30)
    both_s = time_launches(torch, one_pass, 30)
    ctx.hx_stream_status()
    n_free, locked_on = int((lock < 0).sum()), np.bincount(lock[lock >= 0], minlength=D)
    legal = n_free * D + int((lock >= 0).sum())
    # per instance: timeline entries = distinct event times from now on (the past folds onto now), and
    # stretches = 1 + the entries where occupancy rises
    K = iv["stride"]
    n_tl, m_tl = np.zeros(D, np.int64), np.zeros(D, np.int64)
    for d in range(D):
        k = int(iv["count"][d])
        st = np.maximum(iv["start"][d * K:d * K + k].astype(np.float64), 0.0)
        en = np.maximum(iv["end"][d * K:d * K + k].astype(np.float64), 0.0)
        tk = iv["tok"][d * K:d * K + k].astype(np.int64)
        t = np.unique(np.concatenate([[0.0], st, en]))
        occ = np.array([tk[(st <= x) & (x < en)].sum() for x in t])
        n_tl[d], m_tl[d] = t.size, 1 + int((occ[1:] > occ[:-1]).sum())
    table = (n_tl <= 512) & (m_tl * (n_tl + 1) <= 4096)
    per_free = np.where(table, DECODE_OPS_BISECT_STEP * np.ceil(np.log2(n_tl + 1)) + DECODE_OPS_STRETCH * m_tl, DECODE_OPS_ENTRY * n_tl) \
        + DECODE_OPS_PAIR
    ops = float(n_free * per_free.sum() + (locked_on * (DECODE_OPS_ENTRY * n_tl + DECODE_OPS_PAIR)).sum())
    out["one pass"] = {"workload": "%d calls x %d instances, %d..%d intervals each, %d%% of the calls locked"
                                   % (Q, D, int(iv["count"].min()), int(iv["count"].max()), round(100 * float((lock >= 0).mean()))),
                       "score_us": score_s * 1e6, "score_and_rank_us": both_s * 1e6,
                       "legal_pairs": legal, "legal_pairs_per_s": legal / score_s,
                       "timeline_entries_mean": float(n_tl.mean()), "stretches_mean": float(m_tl.mean()),
                       "instances_searched_by_table": int(table.sum()),
                       "roofline": {"kernel": "hx_decode_timeline_kernel + hx_decode_score_kernel + hx_decode_finish_kernel", "bound": "alu",
                                    "ops_per_free_pair_mean": float(per_free.mean()), "achieved": ops / score_s / 1e12,
                                    "peak": ALU_PEAK_TOPS, "unit": "T lane-ops/s", "frac": ops / score_s / 1e12 / ALU_PEAK_TOPS},
                       "waiting_fraction_of_placed": float(((bs > 0) & (bd >= 0)).float().sum().item() / max(1, int((bd >= 0).sum().item())))}
    rng = np.random.default_rng(seed)
    for name, Qg, Dg, T, res, plan in (("queue 64 x 8 instances, 3 classes", 64, 8, 4, 24, 4), ("queue 256 x 32 instances, 4 classes", 256, 32, 4, 24, 4)):
        r, lock, iv = synth.make_decode_round("decode_tiny", seed + 1, n_wf=64, Q=Qg, D=Dg, T=T, stride=res + plan, n_resident=res, n_planned=plan)
        K0, K = iv["stride"], min(iv["stride"] + Qg, 140)
        big = dict(stride=K, count=iv["count"].copy())
        for key, dt in (("start", np.float32), ("end", np.float32), ("tok", np.int32)):
            a = np.zeros((Dg, K), dt); a[:, :K0] = iv[key].reshape(Dg, K0); big[key] = a.reshape(-1)
        node = np.arange(Qg, dtype=np.int32); wf = (np.arange(Qg) % 8).astype(np.int32)
        tl = rng.uniform(0, 5, Qg).astype(np.float32); hz = rng.uniform(10, 60, 8).astype(np.float32)
        el = rng.uniform(0, 30, Qg).astype(np.float32)
        qg = binding.to_device(dict(n=Qg, L_in=r.calls["L_in"], L_out=r.calls["L_out"], node=node, wf=wf, elapsed=el))
        ddg, d_lk, d_tl, d_hz = binding.to_device(r.dec), dev(lock), dev(tl), dev(hz)
        cnt0 = dev(big["count"])
        dbig = dict(stride=K, count=cnt0.clone(), start=dev(big["start"]), end=dev(big["end"]), tok=dev(big["tok"]))
        outs = [torch.empty(Qg, **i32), torch.empty(Qg, device="cuda:0"), torch.empty(Qg, device="cuda:0"), torch.empty(Qg, device="cuda:0"),
                torch.empty(Qg, **i32)]

        def plan_once():
            dbig["count"].copy_(cnt0)         # every plan starts from the same snapshot
            ctx.hx_decode_plan_greedy(synth.MODEL, qg, d_lk, ddg, dbig, d_tl, d_hz, *outs)

        gpu_s = time_launches(torch, plan_once, 20)
        ctx.hx_stream_status()
        t0 = time.perf_counter()
        o.decode_plan_greedy(synth.MODEL, r.calls["L_in"], r.calls["L_out"], lock, el, node, wf, tl, hz, r.dec, big)
        cpu_s = time.perf_counter() - t0
        out[name] = {"gpu_us": gpu_s * 1e6, "oracle_1_thread_us": cpu_s * 1e6, "entries_per_instance": K}
    return out


def robustness_leg(torch, ctx, synth, binding, seed):
    """Sensitivity of the chosen pairs to estimate error (Sec. 7.6 injects deterministic multiplicative
    error into the scheduler-visible prefill and decode estimates): every instance's estimates are scaled by
    1 + e or 1 - e, alternating by instance index (its rates divided by that factor); reported are the
    fraction of calls whose pair changes and the true cost of the changed choice relative to the true best."""
    rnd = synth.make_round("large", seed)
    C, P, D = 2048, rnd.pre["n"], rnd.dec["n"]          # the cost tensor of 2048 calls is 512 MB
    sub = {k: (v[:C] if isinstance(v, np.ndarray) else v) for k, v in rnd.calls.items()}
    sub["n"] = C
    calls, links = binding.to_device(sub), binding.to_device(rnd.links)
    pre, dec = binding.to_device(rnd.pre), binding.to_device(rnd.dec)
    i32 = dict(dtype=torch.int32, device="cuda:0")
    cost = torch.empty(C * P * D, device="cuda:0")
    bp, bd, bc = torch.empty(C, **i32), torch.empty(C, **i32), torch.empty(C, device="cuda:0")
    ctx.hx_score_placements(synth.MODEL, calls, pre, dec, links, cost=cost, best_p=bp, best_d=bd, best_cost=bc)
    cost = cost.view(C, P * D)
    ok = bp >= 0
    out = {"workload": "large sweep, first %d calls x %d x %d" % (C, P, D)}
    for err in (0.1, 0.2, 0.3):
        fp = torch.where(torch.arange(P, device="cuda:0") % 2 == 0, 1.0 + err, 1.0 - err)
        fd = torch.where(torch.arange(D, device="cuda:0") % 2 == 0, 1.0 + err, 1.0 - err)
        npre = dict(pre, flops=pre["flops"] / fp, hbm_bw=pre["hbm_bw"] / fp)
        ndec = dict(dec, flops=dec["flops"] / fd, hbm_bw=dec["hbm_bw"] / fd)
        np_, nd_, nc_ = torch.empty(C, **i32), torch.empty(C, **i32), torch.empty(C, device="cuda:0")
        ctx.hx_score_placements(synth.MODEL, calls, npre, ndec, links, best_p=np_, best_d=nd_, best_cost=nc_)
        changed = ok & ((np_ != bp) | (nd_ != bd))
        flat = (np_.long() * D + nd_.long()).clamp(min=0)
        true_of_choice = cost.gather(1, flat.view(-1, 1)).view(-1)
        regret = (true_of_choice[ok] / bc[ok] - 1.0)
        out["%d%%" % round(err * 100)] = {"pairs_changed": float(changed.float().sum().item() / max(1, int(ok.sum().item()))),
                                         "decode_instance_changed": float((ok & (nd_ != bd)).float().sum().item() / max(1, int(ok.sum().item()))),
                                         "mean_cost_increase": float(regret.mean().item()),
                                         "p99_cost_increase": float(regret.quantile(0.99).item())}
    ctx.hx_stream_status()
    return out


def cpu_baseline(rnd, target_s=9.0):
    """The oracle, as it stands, on bounded samples of the same round: on all the host threads this process may use,
    and on one."""
    from oracle import hx_oracle as o
    host_cpus = os.cpu_count() or 1
    try:
        share = len(os.sched_getaffinity(0))
    except AttributeError:
        share = host_cpus
    threads = int(os.environ.get("OMP_NUM_THREADS") or min(share, 16))
    L, O = rnd.calls["L_in"], rnd.calls["L_out"]
    per = rnd.pre["n"] * rnd.dec["n"]

    def timed(nthreads, budget):
        n0 = max(1, min(len(L), 2_000_000 // per * nthreads))
        t0 = time.perf_counter()
        o.score(rnd.model, L[:n0], O[:n0], rnd.pre, rnd.dec, rnd.links, nthreads=nthreads)
        dt = time.perf_counter() - t0
        n1 = int(max(n0, min(len(L), n0 * budget / max(dt, 1e-6))))
        # when the whole round takes less than the budget, it is scored several times over
        passes = int(max(1, min(20, round(budget * n0 / max(dt, 1e-6) / n1)))) if n1 == len(L) else 1
        t0 = time.perf_counter()
        for _ in range(passes):
            o.score(rnd.model, L[:n1], O[:n1], rnd.pre, rnd.dec, rnd.links, nthreads=nthreads)
        dt = time.perf_counter() - t0
        return passes * n1 * per / dt, "%d pass(es) over the first %d of %d calls x %d x %d candidates, fp64, %.1f s" % (
            passes, n1, len(L), rnd.pre["n"], rnd.dec["n"], dt)

    v_all, s_all = timed(threads, target_s)
    v_one, s_one = timed(1, target_s * 0.6)
    return dict(value=v_all, unit="candidates/s", cores=threads, kind="oracle", sample=s_all,
                single_thread=dict(value=v_one, unit="candidates/s", cores=1, sample=s_one),
                host_cpus=host_cpus, cpus_this_process_may_use=share)


def calibration_leg(torch):
    """What the chip does on known work, in this run: the rate at which it issues plain fp32 vector instructions of
    each kind (v_max_f32 alone, v_add_f32 alone, the two alternating; 16 independent registers per lane, eight
    wavefronts per SIMD, no memory), the arithmetic of the search's inner loop on registers alone, and a plain
    256 MiB device copy."""
    import ctypes
    from paper_2605_16637_amd import build as hx_build
    if not os.path.exists(hx_build.CALIB_LIB):
        hx_build.build()
    lib = ctypes.CDLL(hx_build.CALIB_LIB)
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    blocks, iters = cus * 8, 1000
    sink = torch.empty(blocks * 256, device="cuda:0")
    ptr = ctypes.c_void_p(sink.data_ptr())
    stream = lambda: ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    out = {"compute_units": cus}
    for mix, name in ((0, "v_max_f32"), (1, "v_add_f32"), (2, "v_max_f32 and v_add_f32 alternating")):
        def fn():
            assert lib.hx_calib_valu(blocks, iters, mix, ptr, stream()) == 0
        sec = time_launches(torch, fn, 10, warmup=3)
        out[name] = {"lane_ops_per_s": blocks * 256 * iters * 32 / sec, "launch_ms": sec * 1e3}

    def search():
        assert lib.hx_calib_search(blocks, iters, ptr, stream()) == 0
    sec = time_launches(torch, search, 10, warmup=3)
    cand = blocks * 256 * iters * 32 / sec
    out["search loop on registers"] = {"candidates_per_s": cand, "main_pipe_lane_ops_per_s": cand * MAIN_PIPE_OPS_PER_CANDIDATE,
                                       "all_lane_ops_per_s": cand * OPS_PER_CANDIDATE, "launch_ms": sec * 1e3}
    n16 = 256 * 1024 * 1024 // 16
    src = torch.empty(n16 * 4, dtype=torch.float32, device="cuda:0").fill_(1.0)
    dst = torch.empty_like(src)

    def copy():
        assert lib.hx_calib_copy(ctypes.c_void_p(src.data_ptr()), ctypes.c_void_p(dst.data_ptr()), ctypes.c_size_t(n16),
                                 cus * 16, stream()) == 0
    sec = time_launches(torch, copy, 10, warmup=3)
    out["plain copy of 256 MiB"] = {"bytes_read": n16 * 16, "bytes_written": n16 * 16, "launch_ms": sec * 1e3,
                                    "GB_per_s": 2 * n16 * 16 / sec / 1e9, "frac_of_hbm_peak": 2 * n16 * 16 / sec / 1e9 / HBM_PEAK_GBS}
    out["published"] = {"main_pipe_lane_ops_per_s": ALU_PEAK_TOPS * 1e12, "clock_ghz": 2.4, "fp32_vector_tflops": FP32_VECTOR_PEAK_TFLOPS}
    return out


def round_latency(torch, ctx, synth, name, seed, eager, rounds=500):
    """p50 / p99 of one scheduling round, host clock from "round handed over" to "indices ready" (stream
    synchronised), and the share of calls whose projected ratio exceeds 1.5 when elapsed = U(0,1) x horizon (the
    deadline alpha x H_w of Eq. (1) with alpha = 1.5)."""
    rnd = synth.make_round(name, seed)
    rd = RoundOnDevice(ctx, rnd)
    rd.horizons()
    u = torch.rand(rnd.calls["n"], device="cuda:0", generator=torch.Generator(device="cuda:0").manual_seed(seed))
    rd.calls["elapsed"].copy_(u * rd.hor[rd.calls["wf"].long()])
    rd.score()
    torch.cuda.synchronize()
    late = float((rd.ratio > 1.5).float().mean().item())
    # The round is enqueued in several ways, timed on alternating rounds of one run (all give the same results, so
    # the pool state evolves as one sequence): replayed from a HIP graph; launched eagerly with the arguments of
    # its library calls marshalled beforehand (binding.Context.prepare: a replayed graph costs the host more than
    # three plain launches do); and as a graph with the horizon refresh on a second stream beside the search,
    # the urgency fold joining them.  With --eager the calls are marshalled at every round.
    rd.step()
    rd.step_overlapped()
    rd.round_call()
    torch.cuda.synchronize()
    if eager:
        runs = {"eager, one stream": rd.step, "eager, horizons beside the search": rd.step_overlapped,
                "eager, hx_round": rd.round_call}
    else:
        runs = {"hip graph replay, one stream": capture(torch, rd.step).replay,
                "hip graph replay, horizons beside the search": capture(torch, rd.step_overlapped).replay,
                "prepared launches, one stream": ctx.prepare(rd.step),
                "hx_round (two launches), arguments marshalled ahead": ctx.prepare(rd.round_call)}
    lat = {k: [] for k in runs}
    names = list(runs)
    for i in range(len(names) * (rounds + 20)):
        k = names[i % len(names)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        runs[k]()
        torch.cuda.synchronize()
        if i >= len(names) * 20:
            lat[k].append((time.perf_counter() - t0) * 1e6)
    ctx.hx_stream_status()
    by = {k: {"p50_us": float(np.percentile(v, 50)), "p99_us": float(np.percentile(v, 99)), "rounds": len(v)} for k, v in lat.items()}
    best = min(by, key=lambda k: by[k]["p50_us"])
    # the round's search kernel on its own (HIP events over back-to-back launches) against the same issue peak
    score_s = time_launches(torch, ctx.prepare(rd.score), 200)      # arguments marshalled once: the host stays ahead of an 8 us kernel
    return {"workload": "%s round: %d calls x %d x %d, %d workflows / %d nodes" % (name, rnd.calls["n"], rnd.pre["n"], rnd.dec["n"],
                                                                                  rnd.dag.n_wf, rnd.dag.n_nodes),
            "p50_us": by[best]["p50_us"], "p99_us": by[best]["p99_us"], "rounds": by[best]["rounds"], "launch": best, "by_launch": by,
            "candidates_per_s_at_p50": rnd.n_candidates / (by[best]["p50_us"] * 1e-6),
            # back-to-back launches of a kernel this short start about 10 us apart whatever its length (the kernel trace
            # in profiles/ has its duration: 8 us on the mid round); the fraction is therefore a lower bound
            "fused_search_kernel": {"launch_period_us": score_s * 1e6, "candidates_per_s": rnd.n_candidates / score_s,
                                    "frac_of_main_pipe_peak": rnd.n_candidates * MAIN_PIPE_OPS_PER_CANDIDATE / score_s / 1e12 / ALU_PEAK_TOPS},
            "calls_with_ratio_above_1.5": late}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="large", choices=["large", "mid", "stream"])
    ap.add_argument("--seed", type=int, default=1)
    ap.add_argument("--launch", default="auto", choices=["auto", "eager", "graph", "prepared", "round"],
                    help="how the timed steps are launched: the round's three library calls from the host, one launch after "
                         "the other (eager; prepared = their arguments marshalled once), as replays of a HIP graph, or as "
                         "one hx_round call (two launches: the horizon refresh rides in the search's, the ratio in the "
                         "commit's; arguments marshalled once); auto = the fastest of them in a short untimed trial")
    ap.add_argument("--eager", action="store_true", help="same as --launch eager")
    ap.add_argument("--overlap", action="store_true",
                    help="run the horizon refresh on a second stream beside the search (measured: 3-4 us slower per round "
                         "than one stream, the fork and join cost more than the small kernels they hide)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-calibration", action="store_true", help="skip the measurement of the chip's vector issue rate")
    ap.add_argument("--stream-rounds", type=int, default=1000, help="consecutive rounds of the streaming leg")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run three plain 256 MiB device copies, the known-size reference for HBM byte counters")
    ap.add_argument("--no-extras", action="store_true", help="skip the mid-round latency and critical-path legs")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: the library runs on one GPU; --gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2605_16637_amd import binding, synth
    if not os.path.exists(binding.LIB_PATH):        # loads what is built, compiles only when there is nothing
        from paper_2605_16637_amd import build
        build.build()
    ctx = binding.Context(0)
    torch.cuda.set_device(0)

    rnd = synth.make_round(args.workload if args.workload != "stream" else "stream", args.seed)
    rd = RoundOnDevice(ctx, rnd)
    C, P, D = rnd.calls["n"], rnd.pre["n"], rnd.dec["n"]
    n_cand = C * P * D

    # A short round is launch-bound on the host unless its launches are replayed from a HIP graph.  A long one
    # is not, and in a replayed graph the second kernel starts a few microseconds after the first has ended
    # (seen in the kernel trace whenever the first kernel is shorter than about 7 us): eager launches, which
    # the host enqueues ahead of the GPU, then give the higher rate.
    launch = "eager" if args.eager else args.launch
    step = rd.step_overlapped if args.overlap else rd.step
    step()
    torch.cuda.synchronize()
    modes = {"eager": lambda: step, "graph": lambda: capture(torch, step).replay,
             # the same launches with the arguments of the library calls marshalled once (not with --overlap: the
             # waits between the two streams are not library calls)
             "prepared": lambda: ctx.prepare(step),
             # the whole round as one library call
             "round": lambda: ctx.prepare(rd.round_call)}
    if args.overlap:
        del modes["prepared"], modes["round"]
    if launch == "auto":
        # whichever is fastest on this host, from a short untimed trial of each (a slow host makes eager launch-bound)
        made = {k: f() for k, f in modes.items()}
        trial = {k: time_steps(torch, f, 30, 5) for k, f in made.items()}
        launch = min(trial, key=trial.get)
        run = made[launch]
    else:
        run = modes[launch]()
    wall = time_steps(torch, run, args.steps, args.warmup)
    ctx.hx_stream_status()
    ms_per_step = wall / args.steps * 1e3
    value = n_cand * args.steps / wall
    # the dominant kernel on its own: table prepare + fused search, HIP events on the launch stream
    score_s = time_launches(torch, rd.score, max(20, min(args.steps, 200)))
    achieved = n_cand * MAIN_PIPE_OPS_PER_CANDIDATE / score_s / 1e12
    out = {
        "metric": "placement candidates scored/sec",
        "value": value, "unit": "candidates/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": {"large": "large scoring sweep: 16384 ready calls x 256 prefill x 256 decode, 8 classes",
                                "mid": "mid round: 4096 ready calls x 64 prefill x 64 decode, 4 classes",
                                "stream": "streaming round shape: 32768 ready calls x 512 x 512, 8 classes"}[args.workload],
                   "calls": C, "prefill": P, "decode": D, "candidates_per_round": n_cand,
                   "dag_nodes": rnd.dag.n_nodes, "dag_edges": rnd.dag.n_edges, "workflows": rnd.dag.n_wf,
                   # share of (call, decode instance) pairs whose KV does not fit the instance's free tokens (inputs only)
                   "infeasible_pair_fraction": float(np.mean(
                       (rnd.calls["L_in"].astype(np.int64) + rnd.calls["L_out"])[:, None]
                       > (rnd.dec["cap_tok"].astype(np.int64) - rnd.dec["used_tok"])[None, :])),
                   "step": ("[node cost + critical path (one launch)] beside [fused score+argmin] on two streams -> urgency fold -> commit"
                            if args.overlap else
                            "hx_round: [node cost + critical path] and [fused score+argmin] in one launch -> commit with the ratio (one launch)"
                            if launch == "round" else "node cost + critical path (one launch) -> fused score+argmin+ratio -> commit"),
                   "launch": {"eager": "eager, the host enqueues ahead of the GPU", "graph": "hip graph replay",
                              "prepared": "eager launches with pre-marshalled arguments, the host enqueues ahead of the GPU",
                              "round": "one hx_round call per step (two launches), arguments marshalled once, the host enqueues ahead of the GPU"}[launch],
                   "seed": args.seed},
        "roofline": {"kernel": "hx_fused_search_kernel (derives the pool's per-round tables in its own workgroups); in an hx_round step the "
                               "same search runs as hx_reveal_search_kernel, with the horizon refresh's workgroups in the same launch",
                     "bound": "alu",
                     "achieved": achieved, "peak": ALU_PEAK_TOPS,
                     "unit": "T lane-ops/s on the SIMDs' main fp32 pipe (v_max_f32, v_min3_f32: 1.5 per candidate; the v_add_f32 pairs with them on the second pipe)",
                     "frac": achieved / ALU_PEAK_TOPS,
                     "traffic": profiled_traffic("fused_search_large_sweep.txt", FUSED_SOURCES) if args.workload == "large" else None,
                     "main_pipe_ops_per_candidate": MAIN_PIPE_OPS_PER_CANDIDATE, "ops_per_candidate": OPS_PER_CANDIDATE,
                     "launch_ms": score_s * 1e3, "candidates_per_s_kernel": n_cand / score_s,
                     "frac_of_fp32_vector_peak_157.3_tflops": n_cand * OPS_PER_CANDIDATE / score_s / 1e12 / FP32_VECTOR_PEAK_TFLOPS},
    }
    if not args.no_calibration:
        cal = calibration_leg(torch)
        out["calibration"] = cal
        measured = cal["search loop on registers"]["main_pipe_lane_ops_per_s"] / 1e12
        out["roofline"]["peak_measured"] = measured
        out["roofline"]["frac_of_measured"] = achieved / measured

    if not args.no_extras:
        eager = args.eager or args.launch == "eager"
        out["round_latency"] = round_latency(torch, ctx, synth, "mid", args.seed, eager)
        out["round_latency"]["tiny"] = round_latency(torch, ctx, synth, "tiny", args.seed, eager)
        # critical-path stress: 100 000 workflows, 2.0 M nodes; rotating copies so the
        # pass does not run out of the 256 MB last-level cache
        cp = synth.make_round("cp", args.seed)
        d = cp.dag
        n_copies = 6
        sets = []
        cost_np = np.random.default_rng(args.seed).uniform(0.5, 6.0, d.n_nodes).astype(np.float32)
        for _ in range(n_copies):
            sets.append(dict(rp=dev(d.succ_row_ptr), col=dev(d.succ_col), wp=dev(d.wf_ptr), cost=dev(cost_np),
                             rem=torch.empty(d.n_nodes, device="cuda:0"), tail=torch.empty(d.n_nodes, device="cuda:0"),
                             level=torch.empty(d.n_nodes, dtype=torch.int32, device="cuda:0"),
                             hor=torch.empty(d.n_wf, device="cuda:0")))
        reps = 60
        k = [0]

        def cp_once():
            x = sets[k[0] % n_copies]
            k[0] += 1
            ctx.hx_critical_path(x["rp"], x["col"], x["cost"], x["wp"], x["rem"], x["tail"], x["level"], x["hor"])

        cp_ms = time_launches(torch, cp_once, reps, warmup=n_copies) * 1e3
        ctx.hx_stream_status()
        cp_bytes = 4 * (d.n_nodes + 1) + 4 * d.n_edges + 4 * d.n_nodes + 4 * (d.n_wf + 1) + 12 * d.n_nodes + 4 * d.n_wf
        gbs = cp_bytes / (cp_ms * 1e-3) / 1e9
        # what a plain device copy moving the same number of bytes takes (half read, half written),
        # over rotating buffers: the practical floor of a launch this small
        half = cp_bytes // 8
        bufs = [(torch.empty(half, dtype=torch.float32, device="cuda:0").fill_(1.0),
                 torch.empty(half, dtype=torch.float32, device="cuda:0")) for _ in range(n_copies)]
        j = [0]

        def copy_once():
            a, b = bufs[j[0] % n_copies]
            j[0] += 1
            b.copy_(a)

        copy_ms = time_launches(torch, copy_once, reps, warmup=n_copies) * 1e3
        del bufs
        out["critical_path"] = {"workload": "critical-path stress: %d workflows, %d nodes, %d edges" % (d.n_wf, d.n_nodes, d.n_edges),
                                "kernel": "hx_cp_local_kernel", "bound": "hbm", "launch_ms": cp_ms,
                                "algorithmic_bytes": cp_bytes, "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                "frac": gbs / HBM_PEAK_GBS, "traffic": profiled_traffic("cp_local_critical_path_stress.txt", CP_SOURCES), "rotating_copies": n_copies,
                                "plain_copy_same_bytes_ms": copy_ms}
        del sets
        # the same kernel on eight copies of the graph side by side (16 M nodes, 435 MB per pass, more than the
        # last-level cache holds): the rate once the launch ramp is amortised and blocks of several rounds overlap
        kx = 8
        off_n = (np.arange(kx, dtype=np.int64) * d.n_nodes)[:, None]
        off_e = (np.arange(kx, dtype=np.int64) * d.n_edges)[:, None]
        rp8 = np.append((d.succ_row_ptr[None, :-1] + off_e).ravel(), kx * d.n_edges).astype(np.int32)
        col8 = (d.succ_col[None, :] + off_n).ravel().astype(np.int32)
        wp8 = np.append((d.wf_ptr[None, :-1] + off_n).ravel(), kx * d.n_nodes).astype(np.int32)
        n8, w8 = kx * d.n_nodes, kx * d.n_wf
        big = [dict(rp=dev(rp8), col=dev(col8), wp=dev(wp8), cost=dev(np.tile(cost_np, kx)),
                    rem=torch.empty(n8, device="cuda:0"), tail=torch.empty(n8, device="cuda:0"),
                    level=torch.empty(n8, dtype=torch.int32, device="cuda:0"), hor=torch.empty(w8, device="cuda:0"))
               for _ in range(2)]
        kb = [0]

        def cp_big_once():
            x = big[kb[0] % 2]
            kb[0] += 1
            ctx.hx_critical_path(x["rp"], x["col"], x["cost"], x["wp"], x["rem"], x["tail"], x["level"], x["hor"])

        big_ms = time_launches(torch, cp_big_once, 20, warmup=2) * 1e3
        ctx.hx_stream_status()
        big_bytes = 4 * (n8 + 1) + 4 * kx * d.n_edges + 4 * n8 + 4 * (w8 + 1) + 12 * n8 + 4 * w8
        del big
        half = big_bytes // 8
        a8 = torch.empty(half, dtype=torch.float32, device="cuda:0").fill_(1.0)
        b8 = torch.empty(half, dtype=torch.float32, device="cuda:0")
        copy8_ms = time_launches(torch, lambda: b8.copy_(a8), 20, warmup=2) * 1e3
        del a8, b8
        out["critical_path"]["eight_graphs_side_by_side"] = {
            "nodes": n8, "launch_ms": big_ms, "algorithmic_bytes": big_bytes, "achieved": big_bytes / (big_ms * 1e-3) / 1e9,
            "unit": "GB/s", "frac": big_bytes / (big_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "plain_copy_same_bytes_ms": copy8_ms}

    if not args.no_extras:
        out["streaming"] = streaming_leg(torch, ctx, synth, binding, args.seed, rounds=args.stream_rounds)
        out["planner"] = planner_leg(torch, ctx, synth, binding, args.seed)
        out["decode_stage"] = decode_leg(torch, ctx, synth, binding, args.seed)
        out["estimate_error"] = robustness_leg(torch, ctx, synth, binding, args.seed)
    if args.calibration_copy:
        src = torch.empty(64 * 1024 * 1024, dtype=torch.float32, device="cuda:0").fill_(1.0)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        out["calibration_copy"] = {"bytes_read": src.numel() * 4, "bytes_written": src.numel() * 4, "launches": 3}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(rnd)
    ctx.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
