"""Seeded synthetic scheduling rounds.

This module only *draws inputs*: lengths, DAG shapes, pool descriptions and
instance snapshots.  It holds none of the scheduler's arithmetic and is the one
module that both the GPU path and its CPU checker are fed from.  It needs
numpy only.

The rounds stand in for the agentic traces the paper evaluates on (Sec. 7.1:
conversational chains, function-calling workflows, tree-search workflows and
their mix, each node annotated with input length, output length, parents and
workflow id).  None of those traces is reproduced here: only shape statistics
are used -- DAG size, fan-out and depth ranges, log-normal prompt and output
lengths, and heterogeneous pools given by per-class FLOP/s, memory bandwidth,
KV capacity and NIC bandwidth.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

# Model descriptor handed to the estimator at run time.  kappa follows the
# KV geometry fp16 x 32 layers x 8 KV heads x 128 dims x {K,V}; the others are
# consistent with it (8e9 active parameters, d_model 4096, fp16 weights).
MODEL = dict(
    kv_bytes_per_token=131072.0,      # kappa  [B/token]
    flops_per_token=1.6e10,           # phi    [FLOP/token]
    attn_flops_per_token2=262144.0,   # a      [FLOP/token^2]
    weight_bytes=1.6e10,              # omega  [B]
    nominal_batch=64.0,               # Bbar
)

TOKENS_PER_SEQ = 2048   # batch[d] = ceil(used_tok / TOKENS_PER_SEQ), clipped
MAX_BATCH = 256

# per-class (TFLOP/s, TB/s, KV GB, NIC GB/s)
_TYPES_2 = ([400.0, 1000.0], [2.0, 3.3], [40.0, 80.0], [25.0, 50.0])
_TYPES_4 = ([180.0, 400.0, 1000.0, 2500.0], [0.9, 2.0, 3.3, 8.0],
            [24.0, 40.0, 80.0, 288.0], [12.5, 25.0, 50.0, 100.0])


def type_table(n_types: int) -> dict:
    """Per-class rates.  2 and 4 classes are the listed ones; 8 classes are
    interpolated log-uniformly between the extremes of the 4-class table."""
    if n_types == 2:
        tf, tb, kv, nic = (np.array(x) for x in _TYPES_2)
    elif n_types == 4:
        tf, tb, kv, nic = (np.array(x) for x in _TYPES_4)
    else:
        lo = [x[0] for x in _TYPES_4]
        hi = [x[-1] for x in _TYPES_4]
        tf, tb, kv, nic = (np.geomspace(a, b, n_types) for a, b in zip(lo, hi))
    return dict(
        n_types=n_types,
        flops=(tf * 1e12).astype(np.float32),
        hbm_bw=(tb * 1e12).astype(np.float32),
        kv_bytes=kv * 1e9,
        nic_bw=(nic * 1e9).astype(np.float32),
    )


def link_table(types: dict) -> dict:
    """Effective bandwidth between two classes = the slower NIC of the two."""
    nic = types["nic_bw"]
    bw = np.minimum(nic[:, None], nic[None, :]).astype(np.float32)
    return dict(n_types=int(types["n_types"]), bw=bw, latency=None)


def gen_lengths(rng: np.random.Generator, n: int):
    """Prompt tokens ~ lognormal(median 1500, sigma 1.0) clipped to [64, 32768];
    output tokens ~ lognormal(median 300, sigma 0.8) clipped to [16, 4096]."""
    L_in = np.clip(np.rint(np.exp(np.log(1500.0) + 1.0 * rng.standard_normal(n))), 64, 32768)
    L_out = np.clip(np.rint(np.exp(np.log(300.0) + 0.8 * rng.standard_normal(n))), 16, 4096)
    return L_in.astype(np.int32), L_out.astype(np.int32)


@dataclass
class Dag:
    n_nodes: int
    n_wf: int
    wf_ptr: np.ndarray          # [n_wf+1] nodes of a workflow are contiguous
    wf_of_node: np.ndarray      # [n]
    succ_row_ptr: np.ndarray    # [n+1] successor CSR (children, increasing id)
    succ_col: np.ndarray        # [E]
    parent_row_ptr: np.ndarray  # [n+1] parent CSR (child -> parents)
    parent_col: np.ndarray      # [E]
    L_in: np.ndarray = field(default=None)
    L_out: np.ndarray = field(default=None)

    @property
    def n_edges(self) -> int:
        return int(self.succ_col.size)


def _csr(n: int, src: np.ndarray, dst: np.ndarray):
    order = np.lexsort((dst, src))
    col = dst[order].astype(np.int32)
    row_ptr = np.zeros(n + 1, np.int32)
    if src.size:
        row_ptr[1:] = np.cumsum(np.bincount(src, minlength=n))
    return row_ptr, col


def gen_dag(rng: np.random.Generator, n_wf: int, size_lo: int, size_hi: int,
            fanout_max: int, depth_max: int, p_second: float = 0.4,
            recency: float = 1.0) -> Dag:
    """Random workflow DAGs, generated parent-first.

    Node i of a workflow draws one parent (and with probability ``p_second`` a
    second, distinct one) among nodes 0..i-1 of the same workflow whose
    out-degree is below ``fanout_max`` and whose depth is below
    ``depth_max - 1``, so a longest path has at most ``depth_max`` nodes.
    ``recency`` biases the draw towards late nodes (deeper, chain-like DAGs).
    Ids are topological (parent id < child id) and workflow-contiguous.
    """
    size = rng.integers(size_lo, size_hi + 1, n_wf).astype(np.int64)
    max_n = int(size.max()) if n_wf else 0
    depth = np.zeros((n_wf, max_n), np.int16)
    outdeg = np.zeros((n_wf, max_n), np.int16)
    wf_ptr = np.zeros(n_wf + 1, np.int64)
    wf_ptr[1:] = np.cumsum(size)
    e_src, e_dst = [], []
    for i in range(1, max_n):
        act = np.nonzero(size > i)[0]
        if act.size == 0:
            break
        dep, od = depth[act, :i], outdeg[act, :i]
        ok_depth = dep < (depth_max - 1)
        valid = ok_depth & (od < fanout_max)
        none = ~valid.any(axis=1)
        valid[none] = ok_depth[none]            # fan-out cap relaxed when it cannot hold
        score = rng.random((act.size, i)) + recency * (np.arange(i)[None, :] / max(i, 1))
        s1 = np.where(valid, score, -1.0)
        p1 = s1.argmax(axis=1)
        rows = np.arange(act.size)
        new_depth = dep[rows, p1] + 1
        outdeg[act, p1] += 1
        e_src.append(wf_ptr[act] + p1); e_dst.append(wf_ptr[act] + i)
        if i >= 2 and p_second > 0:
            want = rng.random(act.size) < p_second
            valid2 = valid & (outdeg[act, :i] < fanout_max)
            valid2[rows, p1] = False
            score2 = rng.random((act.size, i))
            s2 = np.where(valid2, score2, -1.0)
            p2 = s2.argmax(axis=1)
            has = want & (s2[rows, p2] >= 0)
            sel = np.nonzero(has)[0]
            if sel.size:
                outdeg[act[sel], p2[sel]] += 1
                new_depth[sel] = np.maximum(new_depth[sel], dep[sel, p2[sel]] + 1)
                e_src.append(wf_ptr[act[sel]] + p2[sel]); e_dst.append(wf_ptr[act[sel]] + i)
        depth[act, i] = new_depth
    n = int(wf_ptr[-1])
    src = np.concatenate(e_src).astype(np.int64) if e_src else np.zeros(0, np.int64)
    dst = np.concatenate(e_dst).astype(np.int64) if e_dst else np.zeros(0, np.int64)
    srow, scol = _csr(n, src, dst)
    prow, pcol = _csr(n, dst, src)
    wf_of_node = np.repeat(np.arange(n_wf, dtype=np.int32), size)
    dag = Dag(n, n_wf, wf_ptr.astype(np.int32), wf_of_node, srow, scol, prow, pcol)
    dag.L_in, dag.L_out = gen_lengths(rng, n)
    return dag


def gen_pool(rng: np.random.Generator, P: int, D: int, n_types: int, L_in, L_out,
             near_capacity: bool):
    """Prefill and decode instance snapshots.

    Instances take classes round-robin.  backlog_tok and qd_tok are uniform on
    0..20000.  used_tok is uniform on [0, cap/2) -- or, with ``near_capacity``,
    cap minus a free amount drawn from the upper fifth of the calls' demand
    distribution, so that about one (call, decode) pair in ten does not fit.
    """
    types = type_table(n_types)
    links = link_table(types)
    kappa = MODEL["kv_bytes_per_token"]
    cap_type = np.floor(types["kv_bytes"] / kappa).astype(np.int64)
    pt = (np.arange(P) % n_types).astype(np.int32)
    dt = (np.arange(D) % n_types).astype(np.int32)
    pre = dict(n=P, flops=types["flops"][pt].copy(), hbm_bw=types["hbm_bw"][pt].copy(),
               backlog_tok=rng.integers(0, 20001, P).astype(np.int32), type=pt)
    cap = cap_type[dt]
    if near_capacity:
        demand = np.sort(np.asarray(L_in, np.int64) + np.asarray(L_out, np.int64))
        u = rng.uniform(0.8, 1.0, D)
        free = demand[np.minimum((u * demand.size).astype(np.int64), demand.size - 1)]
        used = np.maximum(cap - free, 0)
    else:
        used = (rng.random(D) * 0.5 * cap).astype(np.int64)
    batch = np.clip(-(-used // TOKENS_PER_SEQ), 0, MAX_BATCH)
    dec = dict(n=D, flops=types["flops"][dt].copy(), hbm_bw=types["hbm_bw"][dt].copy(),
               used_tok=used.astype(np.int32), cap_tok=cap.astype(np.int32),
               batch=batch.astype(np.int32), qd_tok=rng.integers(0, 20001, D).astype(np.int32), type=dt)
    return types, links, pre, dec


def gen_calls(rng: np.random.Generator, dag: Dag, C: int, leaf_fraction: float = 0.75):
    """Ready calls: nodes of the DAG, mostly leaves of the revealed graph (the
    paper's reveal rule makes a ready call a leaf), the rest interior nodes so
    that a non-zero downstream tail is exercised too."""
    outdeg = np.diff(dag.succ_row_ptr)
    leaves = np.nonzero(outdeg == 0)[0]
    inner = np.nonzero(outdeg > 0)[0]
    n_leaf = min(int(round(C * leaf_fraction)), C) if inner.size else C
    pick_leaf = rng.choice(leaves, n_leaf, replace=leaves.size < n_leaf) if n_leaf else np.zeros(0, np.int64)
    n_in = C - n_leaf
    pick_in = rng.choice(inner, n_in, replace=inner.size < n_in) if n_in else np.zeros(0, np.int64)
    node = np.concatenate([pick_leaf, pick_in]).astype(np.int32)
    rng.shuffle(node)
    return dict(n=C, node=node, wf=dag.wf_of_node[node].astype(np.int32),
                L_in=dag.L_in[node].copy(), L_out=dag.L_out[node].copy(),
                elapsed=rng.uniform(0.0, 30.0, C).astype(np.float32))


@dataclass
class Round:
    name: str
    seed: int
    model: dict
    dag: Dag
    calls: dict
    types: dict
    links: dict
    pre: dict
    dec: dict

    @property
    def n_candidates(self) -> int:
        return int(self.calls["n"]) * int(self.pre["n"]) * int(self.dec["n"])


# name: (n_wf, size_lo, size_hi, fanout_max, depth_max, p_second, recency, C, P, D, T, near_capacity)
WORKLOADS = {
    "tiny":  (8, 4, 12, 3, 5, 0.3, 0.5, 64, 4, 4, 2, False),
    "mid":   (1000, 10, 30, 4, 12, 0.4, 1.0, 4096, 64, 64, 4, False),
    "large": (4096, 10, 30, 4, 12, 0.4, 1.0, 16384, 256, 256, 8, True),
    "cp":    (100000, 8, 32, 4, 32, 0.84, 2.0, 4096, 64, 64, 4, False),
    "stream_small": (512, 4, 12, 3, 8, 0.3, 1.0, 2048, 64, 64, 8, True),
    "stream": (20000, 4, 12, 3, 8, 0.3, 1.0, 32768, 512, 512, 8, True),
}


def make_round(name: str, seed: int = 1, **override) -> Round:
    """One scheduling round of the named workload (see WORKLOADS)."""
    keys = ("n_wf", "size_lo", "size_hi", "fanout_max", "depth_max", "p_second", "recency",
            "C", "P", "D", "T", "near_capacity")
    cfg = dict(zip(keys, WORKLOADS[name]))
    cfg.update(override)
    rng = np.random.default_rng(np.random.PCG64(seed))
    dag = gen_dag(rng, cfg["n_wf"], cfg["size_lo"], cfg["size_hi"], cfg["fanout_max"],
                  cfg["depth_max"], cfg["p_second"], cfg["recency"])
    calls = gen_calls(rng, dag, cfg["C"])
    types, links, pre, dec = gen_pool(rng, cfg["P"], cfg["D"], cfg["T"],
                                      calls["L_in"], calls["L_out"], cfg["near_capacity"])
    return Round(name, seed, dict(MODEL), dag, calls, types, links, pre, dec)


def gen_intervals(rng: np.random.Generator, cap_tok, demand, stride: int, n_resident: int, n_planned: int):
    """Decode token-capacity intervals of every decode instance, fixed stride.

    Per instance: ``n_resident`` entries that hold KV now (start in the last
    20 s, release within the next 30 s; one entry may stand for a group of
    sequences released together) whose token counts split, with random
    weights, an occupancy of cap minus a free amount; the free amount is a
    U(0.2, 1) quantile of the waiting calls' demands, so a good share of the
    calls does not fit an instance right now and has to wait for releases.
    Then 0..``n_planned`` planned sequences with demands drawn like calls, that
    start within the next 10 s and hold their tokens for 1..20 s.  Entries
    beyond count[d] are filler.  Times are float32 seconds from now."""
    cap_tok = np.asarray(cap_tok, np.int64)
    demand = np.sort(np.asarray(demand, np.int64))
    D = cap_tok.size
    assert n_resident + n_planned <= stride and n_resident >= 1
    start = np.zeros((D, stride), np.float32)
    end = np.zeros((D, stride), np.float32)
    tok = np.zeros((D, stride), np.int32)
    count = np.zeros(D, np.int32)
    for d in range(D):
        free = demand[min(int(rng.uniform(0.2, 1.0) * demand.size), demand.size - 1)]
        occ0 = max(int(cap_tok[d] - free), 0)
        w = rng.random(n_resident) + 0.1
        share = np.floor(w / w.sum() * occ0).astype(np.int64)
        share[0] += occ0 - share.sum()
        k_pl = int(rng.integers(0, n_planned + 1))
        n = n_resident + k_pl
        start[d, :n_resident] = -rng.uniform(0.0, 20.0, n_resident)
        end[d, :n_resident] = rng.uniform(0.05, 30.0, n_resident)
        tok[d, :n_resident] = share
        Lp, Op = gen_lengths(rng, max(k_pl, 1))
        s_pl = rng.uniform(0.0, 10.0, k_pl)
        start[d, n_resident:n] = s_pl
        end[d, n_resident:n] = s_pl + rng.uniform(1.0, 20.0, k_pl)
        tok[d, n_resident:n] = (Lp.astype(np.int64) + Op)[:k_pl]
        count[d] = n
    return dict(stride=stride, count=count, start=start.reshape(-1), end=end.reshape(-1), tok=tok.reshape(-1))


# decode-stage workloads: (n_wf, size_lo, size_hi, Q, D, T, stride, n_resident, n_planned, lock_fraction)
DECODE_WORKLOADS = {
    "decode_tiny": (8, 4, 12, 48, 4, 2, 16, 10, 3, 0.5),
    "decode_mid": (1000, 10, 30, 4096, 64, 4, 64, 56, 6, 0.5),
    "decode_large": (4096, 10, 30, 16384, 256, 8, 128, 112, 12, 0.5),
}


def make_decode_round(name: str, seed: int = 1, **override):
    """One decode-stage round: a queue of calls whose KV has arrived (about
    half of them locked to an instance), the decode table and its intervals.
    Returns (Round, lock, intervals); the Round's prefill side is a 1-instance stub."""
    keys = ("n_wf", "size_lo", "size_hi", "Q", "D", "T", "stride", "n_resident", "n_planned", "lock_fraction")
    cfg = dict(zip(keys, DECODE_WORKLOADS[name]))
    cfg.update(override)
    rng = np.random.default_rng(np.random.PCG64(seed))
    dag = gen_dag(rng, cfg["n_wf"], cfg["size_lo"], cfg["size_hi"], 4, 12, 0.4, 1.0)
    calls = gen_calls(rng, dag, cfg["Q"])
    types, links, pre, dec = gen_pool(rng, 1, cfg["D"], cfg["T"], calls["L_in"], calls["L_out"], False)
    iv = gen_intervals(rng, dec["cap_tok"], calls["L_in"].astype(np.int64) + calls["L_out"], cfg["stride"],
                       cfg["n_resident"], cfg["n_planned"])
    lock = np.where(rng.random(cfg["Q"]) < cfg["lock_fraction"], rng.integers(0, cfg["D"], cfg["Q"]), -1).astype(np.int32)
    return Round(name, seed, dict(MODEL), dag, calls, types, links, pre, dec), lock, iv


class StreamGen:
    """Rounds of a live system: every round reveals 0..8 new calls per live
    workflow (parents among that workflow's recent nodes), a workflow that has
    reached its final size retires and a fresh one takes its slot, and the
    pool drains by per-instance amounts proportional to instance speed.

    Structure only; which placements are chosen is not known here.
    """

    def __init__(self, seed: int, n_live: int, final_lo: int = 10, final_hi: int = 30,
                 max_new: int = 8, ring: int = 8):
        self.rng = np.random.default_rng(np.random.PCG64(seed))
        self.n_live, self.max_new, self.ring = n_live, max_new, ring
        self.final_lo, self.final_hi = final_lo, final_hi
        self.n_nodes = 0
        self.n_wf = 0
        self.slot_wf = np.full(n_live, -1, np.int64)       # workflow id in each live slot
        self.slot_size = np.zeros(n_live, np.int64)
        self.slot_final = np.zeros(n_live, np.int64)
        self.recent = np.full((n_live, ring), -1, np.int64)  # recent node ids per slot
        self.recent_n = np.zeros(n_live, np.int64)

    def next_batch(self):
        """Returns dict(n_new, parent_row_ptr, parent_col, wf, L_in, L_out,
        n_wf_total).  New nodes get ids n_nodes.. in slot order; parents always
        have smaller ids."""
        rng = self.rng
        done = (self.slot_wf < 0) | (self.slot_size >= self.slot_final)
        k = int(done.sum())
        if k:
            self.slot_wf[done] = self.n_wf + np.arange(k)
            self.n_wf += k
            self.slot_size[done] = 0
            self.slot_final[done] = rng.integers(self.final_lo, self.final_hi + 1, k)
            self.recent[done] = -1
            self.recent_n[done] = 0
        new = rng.integers(0, self.max_new + 1, self.n_live)
        new = np.minimum(new, self.slot_final - self.slot_size)
        new = np.where(self.slot_size == 0, np.maximum(new, 1), new)   # a fresh workflow reveals a source
        total = int(new.sum())
        slot = np.repeat(np.arange(self.n_live), new)
        first = np.zeros(self.n_live + 1, np.int64); first[1:] = np.cumsum(new)
        ids = self.n_nodes + np.arange(total)
        # parents: up to 2 distinct draws from the slot's ring of recent nodes
        # (as it stood before this round); sources of fresh workflows have none
        rn = self.recent_n[slot]
        has = rn > 0
        r1 = (rng.random(total) * np.maximum(rn, 1)).astype(np.int64)
        r2 = (rng.random(total) * np.maximum(rn, 1)).astype(np.int64)
        two = has & (rng.random(total) < 0.3) & (r2 != r1)
        p1 = self.recent[slot, np.minimum(r1, self.ring - 1)]
        p2 = self.recent[slot, np.minimum(r2, self.ring - 1)]
        cnt = has.astype(np.int64) + two.astype(np.int64)
        prow = np.zeros(total + 1, np.int64); prow[1:] = np.cumsum(cnt)
        pcol = np.empty(int(prow[-1]), np.int64)
        pcol[prow[:-1][has]] = p1[has]
        pcol[prow[:-1][two] + 1] = p2[two]
        L_in, L_out = gen_lengths(rng, total)
        # update rings: the j-th new node of a slot overwrites ring position
        # (nodes seen so far + j) mod ring
        for j in range(self.max_new):
            m = np.nonzero(new > j)[0]
            if m.size == 0:
                break
            self.recent[m, (self.slot_size[m] + j) % self.ring] = self.n_nodes + first[:-1][m] + j
        self.recent_n = np.minimum(self.recent_n + new, self.ring)
        self.slot_size += new
        self.n_nodes += total
        return dict(n_new=total, parent_row_ptr=prow.astype(np.int32), parent_col=pcol.astype(np.int32),
                    wf=self.slot_wf[slot].astype(np.int32), L_in=L_in, L_out=L_out,
                    n_wf_total=self.n_wf, ids=ids.astype(np.int32))

    def drains(self, pre: dict, dec: dict, types: dict, scale: float = 1.0):
        """Per-round drain amounts, proportional to instance speed."""
        f = pre["flops"].astype(np.float64) / float(types["flops"].max())
        g = dec["hbm_bw"].astype(np.float64) / float(types["hbm_bw"].max())
        rng = self.rng
        dp = (scale * 60000.0 * f * rng.uniform(0.8, 1.2, f.size)).astype(np.int32)
        dq = (scale * 20000.0 * g * rng.uniform(0.8, 1.2, g.size)).astype(np.int32)
        rl = (scale * 40000.0 * g * rng.uniform(0.8, 1.2, g.size)).astype(np.int32)
        return dp, dq, rl
