"""ctypes front of the CPU oracle (``hx_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by the tests, by the smoke check and by the
CPU-baseline leg of the benchmark.  The product path never touches this module.

The wrappers below only marshal numpy arrays; all arithmetic of the method is
in the C file.  The one piece of logic that lives here is structural: turning
parent lists into successor lists, so that "incremental append" can be checked
against its definition (a full recomputation on the grown graph).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hx_oracle.c")
_LIB = os.path.join(_HERE, "libhx_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C99, -O2, OpenMP over calls)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-Wall", "-Wextra", "-fopenmp", "-shared", "-fPIC",
             "-o", _LIB, _SRC, "-lm"])
    return _LIB


def build_sanitized(out: str) -> str:
    """The same source with AddressSanitizer and UndefinedBehaviorSanitizer, every
    finding fatal (for a test that runs the pins against it; load it by
    putting its path in HXO_LIB with libasan preloaded)."""
    subprocess.check_call(
        ["gcc", "-O1", "-g", "-std=c99", "-Wall", "-Wextra", "-fopenmp", "-shared", "-fPIC",
         "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
         "-o", out, _SRC, "-lm"])
    return out


class _Model(C.Structure):
    _fields_ = [("kv_bytes_per_token", C.c_double), ("flops_per_token", C.c_double),
                ("attn_flops_per_token2", C.c_double), ("weight_bytes", C.c_double),
                ("nominal_batch", C.c_double)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(os.environ.get("HXO_LIB") or build())      # HXO_LIB: a build of the same source to use instead
        _lib.hxo_score_one.restype = C.c_double
        _lib.hxo_candidate_cost.restype = C.c_double
        for name in ("hxo_prefill_wait", "hxo_prefill_time", "hxo_transfer_time",
                     "hxo_decode_step", "hxo_decode_wait", "hxo_decode_token_time", "hxo_decode_start"):
            getattr(_lib, name).restype = C.c_double
    return _lib


def _model(m) -> _Model:
    return _Model(float(m["kv_bytes_per_token"]), float(m["flops_per_token"]),
                  float(m["attn_flops_per_token2"]), float(m["weight_bytes"]),
                  float(m["nominal_batch"]))


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


@dataclass
class ScoreResult:
    best_p: np.ndarray
    best_d: np.ndarray
    best_cost: np.ndarray
    second: np.ndarray
    cost: np.ndarray | None
    feas: np.ndarray | None


def _tables(pre, dec, links):
    T = int(links["n_types"])
    t = dict(
        pF=_f32(pre["flops"]), pB=_f32(pre["hbm_bw"]), pbl=_i32(pre["backlog_tok"]), pty=_i32(pre["type"]),
        dF=_f32(dec["flops"]), dB=_f32(dec["hbm_bw"]), dus=_i32(dec["used_tok"]), dcap=_i32(dec["cap_tok"]),
        dba=_i32(dec["batch"]), dqd=_i32(dec["qd_tok"]), dty=_i32(dec["type"]),
        bw=_f32(links["bw"]).reshape(-1),
        lat=None if links.get("latency") is None else _f32(links["latency"]).reshape(-1), T=T)
    assert t["bw"].size == T * T
    return t


def score(model, L_in, L_out, pre, dec, links, want_cost=False, want_feas=False, nthreads=0) -> ScoreResult:
    """R7/R8 over all (call, prefill, decode) candidates."""
    L_in, L_out = _i32(L_in), _i32(L_out)
    t = _tables(pre, dec, links)
    Cn, P, D = L_in.size, t["pF"].size, t["dF"].size
    cost = np.empty((Cn, P, D), np.float64) if want_cost else None
    feas = np.empty((Cn, D), np.uint8) if want_feas else None
    bp = np.empty(Cn, np.int32); bd = np.empty(Cn, np.int32)
    bc = np.empty(Cn, np.float64); sc = np.empty(Cn, np.float64)
    m = _model(model)
    rc = lib().hxo_score(C.byref(m), Cn, _p(L_in), _p(L_out),
                         P, _p(t["pF"]), _p(t["pB"]), _p(t["pbl"]), _p(t["pty"]),
                         D, _p(t["dF"]), _p(t["dB"]), _p(t["dus"]), _p(t["dcap"]), _p(t["dba"]),
                         _p(t["dqd"]), _p(t["dty"]), t["T"], _p(t["bw"]), _p(t["lat"]),
                         _p(cost), _p(feas), _p(bp), _p(bd), _p(bc), _p(sc), int(nthreads))
    if rc:
        raise ValueError(f"hxo_score failed: {rc}")
    return ScoreResult(bp, bd, bc, sc, cost, feas)


def score_one(model, L, O, p, d, pre, dec, links) -> float:
    """R7 for one candidate, by index."""
    t = _tables(pre, dec, links)
    m = _model(model)
    return float(lib().hxo_score_one(C.byref(m), C.c_int32(int(L)), C.c_int32(int(O)),
                                     C.c_int32(int(p)), _p(t["pF"]), _p(t["pB"]), _p(t["pbl"]), _p(t["pty"]),
                                     C.c_int32(int(d)), _p(t["dF"]), _p(t["dB"]), _p(t["dus"]), _p(t["dcap"]),
                                     _p(t["dba"]), _p(t["dqd"]), _p(t["dty"]),
                                     t["T"], _p(t["bw"]), _p(t["lat"])))


def select(cost):
    """R8 on an existing [C,P,D] fp64 tensor."""
    cost = _f64(cost)
    Cn, P, D = cost.shape
    bp = np.empty(Cn, np.int32); bd = np.empty(Cn, np.int32); bc = np.empty(Cn, np.float64)
    rc = lib().hxo_select(Cn, P, D, _p(cost), _p(bp), _p(bd), _p(bc))
    if rc:
        raise ValueError(f"hxo_select failed: {rc}")
    return bp, bd, bc


def node_cost(model, L_in, L_out, types, links):
    """R9: standalone cost of each call on its best class pair."""
    L_in, L_out = _i32(L_in), _i32(L_out)
    tF, tB = _f32(types["flops"]), _f32(types["hbm_bw"])
    T = tF.size
    bw = _f32(links["bw"]).reshape(-1)
    lat = None if links.get("latency") is None else _f32(links["latency"]).reshape(-1)
    out = np.empty(L_in.size, np.float64)
    m = _model(model)
    rc = lib().hxo_node_cost(C.byref(m), L_in.size, _p(L_in), _p(L_out), T, _p(tF), _p(tB),
                             _p(bw), _p(lat), _p(out))
    if rc:
        raise ValueError(f"hxo_node_cost failed: {rc}")
    return out


def critical_path(row_ptr, col, cost, wf_ptr, round_f32=True):
    """R10.  Returns (rem, tail, level, horizon); rem/tail/horizon as fp64
    holders of (when round_f32) exact fp32 values."""
    row_ptr, col, wf_ptr = _i32(row_ptr), _i32(col), _i32(wf_ptr)
    cost = _f64(cost)
    n, n_wf = row_ptr.size - 1, wf_ptr.size - 1
    rem = np.zeros(n, np.float64); tail = np.zeros(n, np.float64)
    level = np.zeros(n, np.int32); hor = np.zeros(max(n_wf, 0), np.float64)
    rc = lib().hxo_critical_path(n, _p(row_ptr), _p(col), _p(cost), n_wf, _p(wf_ptr),
                                 1 if round_f32 else 0, _p(rem), _p(tail), _p(level), _p(hor))
    if rc == -2:
        raise ValueError("not a DAG")
    if rc:
        raise ValueError(f"hxo_critical_path failed: {rc}")
    return rem, tail, level, hor


def successors_from_parents(n, parent_row_ptr, parent_col):
    """Structure only: transpose child->parents lists into a successor CSR
    (successors of a node in increasing id)."""
    parent_row_ptr, parent_col = _i32(parent_row_ptr), _i32(parent_col)
    child = np.repeat(np.arange(n, dtype=np.int32), np.diff(parent_row_ptr))
    order = np.lexsort((child, parent_col))
    col = child[order].astype(np.int32)
    counts = np.bincount(parent_col, minlength=n) if parent_col.size else np.zeros(n, np.int64)
    row_ptr = np.zeros(n + 1, np.int32)
    row_ptr[1:] = np.cumsum(counts)
    return row_ptr, col


def critical_path_by_parents(parent_row_ptr, parent_col, cost, wf_of_node, n_wf, round_f32=True):
    """R10 on a graph given as parent lists with a per-node workflow id: the
    definition the incremental append must reproduce after every batch."""
    n = len(cost)
    row_ptr, col = successors_from_parents(n, parent_row_ptr, parent_col)
    rem, tail, level, _ = critical_path(row_ptr, col, cost, np.zeros(1, np.int32), round_f32)
    hor = np.zeros(n_wf, np.float64)
    wf = _i32(wf_of_node)
    rc = lib().hxo_horizon_by_id(n, _p(rem), _p(wf), n_wf, _p(hor))
    if rc:
        raise ValueError("workflow id out of range")
    return rem, tail, level, hor


def critical_path_revealed(parent_row_ptr, parent_col, cost, wf_of_node, n_wf, round_f32=True, out=None):
    """R10 on a graph in reveal order (every parent id below its child's), one
    pass from the last node to the first; same results as critical_path_by_parents.
    out: optional (rem f64, tail f64, level i32, horizon f64) buffers at least as
    long as needed, reused by callers that repeat the pass on a growing graph
    (the results are views of their heads)."""
    prow, pcol, wf = _i32(parent_row_ptr), _i32(parent_col), _i32(wf_of_node)
    cost = _f64(cost)
    n = cost.size
    if out is None:
        rem = np.empty(n, np.float64); tail = np.empty(n, np.float64)
        level = np.empty(n, np.int32); hor = np.empty(n_wf, np.float64)
    else:
        rem, tail, level, hor = out[0][:n], out[1][:n], out[2][:n], out[3][:n_wf]
        assert rem.dtype == np.float64 and tail.dtype == np.float64 and level.dtype == np.int32 and hor.dtype == np.float64
        assert rem.size == n and tail.size == n and level.size == n and hor.size == n_wf
    rc = lib().hxo_critical_path_revealed(n, _p(prow), _p(pcol), _p(cost), _p(wf), int(n_wf),
                                          1 if round_f32 else 0, _p(rem), _p(tail), _p(level), _p(hor))
    if rc:
        raise ValueError("not in reveal order, or a workflow id out of range")
    return rem, tail, level, hor


def urgency(elapsed, best_cost, node, wf, tail, horizon):
    """R11 / Eq. (2)."""
    elapsed, best_cost, tail, horizon = _f64(elapsed), _f64(best_cost), _f64(tail), _f64(horizon)
    node, wf = _i32(node), _i32(wf)
    out = np.empty(elapsed.size, np.float64)
    with np.errstate(all="ignore"):
        lib().hxo_urgency(elapsed.size, _p(elapsed), _p(best_cost), _p(node), _p(wf),
                          _p(tail), _p(horizon), _p(out))
    return out


def commit(L_in, L_out, best_p, best_d, backlog_tok, used_tok, batch, qd_tok,
           drain_prefill, drain_decode_q, release_tok, tokens_per_seq=2048, max_batch=256):
    """R12.  Returns new (backlog_tok, used_tok, batch, qd_tok) and the status."""
    L_in, L_out, best_p, best_d = _i32(L_in), _i32(L_out), _i32(best_p), _i32(best_d)
    bl, us, ba, qd = (_i32(x).copy() for x in (backlog_tok, used_tok, batch, qd_tok))
    dp, dq, rl = _i32(drain_prefill), _i32(drain_decode_q), _i32(release_tok)
    rc = lib().hxo_commit(L_in.size, _p(L_in), _p(L_out), _p(best_p), _p(best_d),
                          bl.size, _p(bl), us.size, _p(us), _p(ba), _p(qd),
                          _p(dp), _p(dq), _p(rl), int(tokens_per_seq), int(max_batch))
    return bl, us, ba, qd, rc


def rank(ratio):
    """R14: position of every call by decreasing ratio, equal ratios by increasing index."""
    ratio = _f64(ratio)
    out = np.empty(ratio.size, np.int32)
    rc = lib().hxo_rank(ratio.size, _p(ratio), _p(out))
    if rc:
        raise ValueError(f"hxo_rank failed: {rc}")
    return out


@dataclass
class PlanResult:
    best_p: np.ndarray
    best_d: np.ndarray
    best_cost: np.ndarray
    ratio: np.ndarray
    rank: np.ndarray
    backlog_tok: np.ndarray
    used_tok: np.ndarray
    batch: np.ndarray
    qd_tok: np.ndarray


def plan_greedy(model, L_in, L_out, elapsed, node, wf, tail, horizon, pre, dec, links,
                tokens_per_seq=2048, max_batch=256) -> PlanResult:
    """R13: the recomputing greedy loop; returns the plan and the simulated state it leaves."""
    L_in, L_out, node, wf = _i32(L_in), _i32(L_out), _i32(node), _i32(wf)
    elapsed, tail, horizon = _f64(elapsed), _f64(tail), _f64(horizon)
    t = _tables(pre, dec, links)
    bl, us, ba, qd = t["pbl"].copy(), t["dus"].copy(), t["dba"].copy(), t["dqd"].copy()
    Cn = L_in.size
    bp = np.empty(Cn, np.int32); bd = np.empty(Cn, np.int32); rk = np.empty(Cn, np.int32)
    bc = np.empty(Cn, np.float64); rt = np.empty(Cn, np.float64)
    m = _model(model)
    with np.errstate(all="ignore"):
        rc = lib().hxo_plan_greedy(C.byref(m), Cn, _p(L_in), _p(L_out), _p(elapsed), _p(node), _p(wf), _p(tail), _p(horizon),
                                   t["pF"].size, _p(t["pF"]), _p(t["pB"]), _p(bl), _p(t["pty"]),
                                   t["dF"].size, _p(t["dF"]), _p(t["dB"]), _p(us), _p(t["dcap"]), _p(ba), _p(qd), _p(t["dty"]),
                                   t["T"], _p(t["bw"]), _p(t["lat"]), int(tokens_per_seq), int(max_batch),
                                   _p(bp), _p(bd), _p(bc), _p(rt), _p(rk))
    if rc:
        raise ValueError(f"hxo_plan_greedy failed: {rc}")
    return PlanResult(bp, bd, bc, rt, rk, bl, us, ba, qd)


# ---- decode stage (R22-R26) -------------------------------------------------------
def decode_start(m_tok, T, cap_tok, iv_start, iv_end, iv_tok) -> float:
    """R23: earliest capacity-feasible start of m_tok tokens for T seconds on one instance."""
    s, e, k = _f64(iv_start), _f64(iv_end), _i32(iv_tok)
    return float(lib().hxo_decode_start(C.c_int32(int(m_tok)), C.c_double(float(T)), C.c_int32(int(cap_tok)),
                                        C.c_int32(s.size), _p(s), _p(e), _p(k)))


@dataclass
class DecodeScore:
    best_d: np.ndarray
    best_start: np.ndarray
    best_cost: np.ndarray
    start: np.ndarray | None
    cost: np.ndarray | None


def _intervals(iv, D):
    stride = int(iv["stride"])
    cnt = _i32(iv["count"]).copy()
    s, e, k = _f64(iv["start"]).reshape(-1).copy(), _f64(iv["end"]).reshape(-1).copy(), _i32(iv["tok"]).reshape(-1).copy()
    assert cnt.size == D and s.size == e.size == k.size == D * stride and (cnt <= stride).all() and (cnt >= 0).all()
    return stride, cnt, s, e, k


def _decode_score(fn, extra, model, L_in, L_out, lock, dec, iv, want_all):
    L_in, L_out = _i32(L_in), _i32(L_out)
    lock = None if lock is None else _i32(lock)
    dF, dB, dus, dcap, dba = _f32(dec["flops"]), _f32(dec["hbm_bw"]), _i32(dec["used_tok"]), _i32(dec["cap_tok"]), _i32(dec["batch"])
    Q, D = L_in.size, dF.size
    stride, cnt, s, e, k = _intervals(iv, D)
    bd = np.empty(Q, np.int32); bs = np.empty(Q, np.float64); bc = np.empty(Q, np.float64)
    st = np.empty((Q, D), np.float64) if want_all else None
    co = np.empty((Q, D), np.float64) if want_all else None
    m = _model(model)
    rc = fn(C.byref(m), Q, _p(L_in), _p(L_out), _p(lock), D, _p(dF), _p(dB), _p(dus), _p(dcap), _p(dba),
            stride, _p(cnt), _p(s), _p(e), _p(k), *extra, _p(st), _p(co), _p(bd), _p(bs), _p(bc))
    if rc:
        raise ValueError(f"decode score failed: {rc}")
    return DecodeScore(bd, bs, bc, st, co)


def decode_score(model, L_in, L_out, lock, dec, iv, want_all=False) -> DecodeScore:
    """R24/R25 over all (call, decode instance) pairs."""
    return _decode_score(lib().hxo_decode_score, (), model, L_in, L_out, lock, dec, iv, want_all)


def decode_score_bracket(model, L_in, L_out, lock, dec, iv, t_scale, t_shift, want_all=False) -> DecodeScore:
    """Not the method: decode_score with every decode time replaced by
    max(0, t_scale * T + t_shift); only the parity test of a finished decode plan uses it."""
    return _decode_score(lib().hxo_decode_score_bracket, (C.c_double(float(t_scale)), C.c_double(float(t_shift))),
                         model, L_in, L_out, lock, dec, iv, want_all)


@dataclass
class DecodePlan:
    best_d: np.ndarray
    best_start: np.ndarray
    best_cost: np.ndarray
    ratio: np.ndarray
    rank: np.ndarray
    count: np.ndarray
    start: np.ndarray
    end: np.ndarray
    tok: np.ndarray


def decode_plan_greedy(model, L_in, L_out, lock, elapsed, node, wf, tail, horizon, dec, iv) -> DecodePlan:
    """R26: recomputing greedy of the decode stage; returns the plan and the extended interval lists."""
    L_in, L_out, node, wf = _i32(L_in), _i32(L_out), _i32(node), _i32(wf)
    lock = None if lock is None else _i32(lock)
    elapsed, tail, horizon = _f64(elapsed), _f64(tail), _f64(horizon)
    dF, dB, dus, dcap, dba = _f32(dec["flops"]), _f32(dec["hbm_bw"]), _i32(dec["used_tok"]), _i32(dec["cap_tok"]), _i32(dec["batch"])
    Q, D = L_in.size, dF.size
    stride, cnt, s, e, k = _intervals(iv, D)
    bd = np.empty(Q, np.int32); rk = np.empty(Q, np.int32)
    bs = np.empty(Q, np.float64); bc = np.empty(Q, np.float64); rt = np.empty(Q, np.float64)
    m = _model(model)
    with np.errstate(all="ignore"):
        rc = lib().hxo_decode_plan_greedy(C.byref(m), Q, _p(L_in), _p(L_out), _p(lock), _p(elapsed), _p(node), _p(wf),
                                          _p(tail), _p(horizon), D, _p(dF), _p(dB), _p(dus), _p(dcap), _p(dba),
                                          stride, _p(cnt), _p(s), _p(e), _p(k), _p(bd), _p(bs), _p(bc), _p(rt), _p(rk))
    if rc:
        raise ValueError(f"hxo_decode_plan_greedy failed: {rc}")
    return DecodePlan(bd, bs, bc, rt, rk, cnt, s.reshape(D, stride), e.reshape(D, stride), k.reshape(D, stride))


# scalar term accessors, for the round-number pins
def term(name, model, *args):
    m = _model(model)
    f = getattr(lib(), "hxo_" + name)
    conv = []
    for a in args:
        conv.append(C.c_int32(a) if isinstance(a, (int, np.integer)) else C.c_double(float(a)))
    return float(f(C.byref(m), *conv))


def feasible(L, O, used, cap) -> bool:
    return bool(lib().hxo_feasible(C.c_int32(L), C.c_int32(O), C.c_int32(used), C.c_int32(cap)))
