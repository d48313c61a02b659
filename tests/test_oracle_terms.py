"""Pins of the oracle's latency terms (no GPU).

The paper describes the estimator's terms (Sec. 4.2, Sec. 5.3, Sec. 5.4) but
prints no values; these tests pin the oracle to hand-worked round-number cases,
to the decomposition of a candidate into its terms, and to the properties the
paper's prose fixes (queues, lower bandwidth and occupancy only ever delay).
"""
import math

import numpy as np
import pytest

from oracle import hx_oracle as o
from paper_2605_16637_amd import synth
from helpers import ROUND_MODEL, one_pool, random_pool, read_kv, read_rows

G = read_kv("round_numbers.txt")
TOL = 1e-12


def test_prefill_wait_round():
    assert o.term("prefill_wait", ROUND_MODEL, 2000, 1e13) == pytest.approx(G["prefill_wait"], rel=TOL)


def test_prefill_time_round():
    assert o.term("prefill_time", ROUND_MODEL, 1000, 1e13, 1e12) == pytest.approx(G["prefill_time_compute"], rel=TOL)
    m = dict(ROUND_MODEL, weight_bytes=4e10)
    assert o.term("prefill_time", m, 1000, 1e15, 1e12) == pytest.approx(G["prefill_time_memory"], rel=TOL)


def test_prefill_time_quadratic_term():
    # with phi = omega = kappa = 0 only a*L^2/F is left: doubling L quadruples it
    m = dict(ROUND_MODEL, flops_per_token=0.0, weight_bytes=0.0, kv_bytes_per_token=0.0)
    t1 = o.term("prefill_time", m, 1000, 1e13, 1e12)
    t2 = o.term("prefill_time", m, 2000, 1e13, 1e12)
    assert t1 == pytest.approx(0.1, rel=TOL) and t2 == pytest.approx(0.4, rel=TOL)


def test_transfer_round_and_table_orientation():
    assert o.term("transfer_time", ROUND_MODEL, 1000, 1e9, 0.05) == pytest.approx(G["transfer_time"], rel=TOL)
    # two classes, asymmetric table: the row is the prefill class, the column the decode class
    pre = dict(flops=[1e13, 1e13], hbm_bw=[1e12, 1e12], backlog_tok=[0, 0], type=[0, 1])
    dec = dict(flops=[1e13, 1e13], hbm_bw=[1e12, 1e12], used_tok=[0, 0], cap_tok=[10**6] * 2,
               batch=[0, 0], qd_tok=[0, 0], type=[0, 1])
    links = dict(n_types=2, bw=np.array([[4e9, 1e9], [2e9, 4e9]], np.float32), latency=None)
    r = o.score(ROUND_MODEL, [1000], [100], pre, dec, links, want_cost=True)
    base = o.score_one(ROUND_MODEL, 1000, 100, 0, 0, pre, dec, links) - 1e8 / 4e9
    assert r.cost[0, 0, 1] - base == pytest.approx(G["transfer_0_to_1"], rel=1e-6)
    assert r.cost[0, 1, 0] - base == pytest.approx(G["transfer_1_to_0"], rel=1e-6)


def test_decode_terms_round():
    assert o.term("decode_step", ROUND_MODEL, 100, 10000, 1e13, 1e12) == pytest.approx(G["decode_step"], rel=TOL)
    assert o.term("decode_wait", ROUND_MODEL, 50, 100, 10000, 1e13, 1e12) == pytest.approx(G["decode_wait"], rel=TOL)
    assert o.term("decode_token_time", ROUND_MODEL, 1000, 100, 100, 10000, 1e13, 1e12) == \
        pytest.approx(G["decode_token_time"], rel=TOL)
    assert o.term("decode_token_time", ROUND_MODEL, 1000, 100, 100, 10000, 1e15, 1e12) == \
        pytest.approx(G["decode_token_time_memory"], rel=TOL)


def test_candidate_round():
    # rates pass through fp32 tables (1e13 is not an fp32 number): 1e-6 relative
    pre, dec, links = one_pool()
    r = o.score(ROUND_MODEL, [1000], [100], pre, dec, links, want_cost=True)
    assert r.cost[0, 0, 0] == pytest.approx(G["candidate_ready_dominates"], rel=1e-6)
    pre, dec, links = one_pool(qd=500)
    r = o.score(ROUND_MODEL, [1000], [100], pre, dec, links, want_cost=True)
    assert r.cost[0, 0, 0] == pytest.approx(G["candidate_wait_dominates"], rel=1e-6)
    assert (r.best_p[0], r.best_d[0]) == (0, 0)


def test_candidate_is_sum_of_its_terms():
    # R7 recomposed from the term functions for random inputs
    rng = np.random.default_rng(5)
    M = synth.MODEL
    for _ in range(50):
        types, pre, dec, links = random_pool(rng, 1, 1, 1)
        dec["cap_tok"] = np.array([2 * 10**6], np.int32)
        L, O = int(rng.integers(64, 32768)), int(rng.integers(16, 4096))
        F, B = float(pre["flops"][0]), float(pre["hbm_bw"][0])
        ready = (o.term("prefill_wait", M, int(pre["backlog_tok"][0]), F)
                 + o.term("prefill_time", M, L, F, B)
                 + o.term("transfer_time", M, L, float(links["bw"][0, 0]), float(links["latency"][0, 0])))
        avail = o.term("decode_wait", M, int(dec["qd_tok"][0]), int(dec["batch"][0]), int(dec["used_tok"][0]), F, B)
        tdec = O * o.term("decode_token_time", M, L, O, int(dec["batch"][0]), int(dec["used_tok"][0]), F, B)
        got = o.score_one(M, L, O, 0, 0, pre, dec, links)
        assert got == pytest.approx(max(ready, avail) + tdec, rel=1e-14)


def test_feasibility_boundary_is_exact():
    # Eq. (3),(4): demand L + O against the capacity still free
    assert o.feasible(1000, 100, 0, 1100)
    assert not o.feasible(1000, 100, 0, 1099)
    assert o.feasible(1000, 100, 500, 1600)
    assert not o.feasible(1000, 100, 501, 1600)
    # no int32 wrap-around
    assert not o.feasible(2**31 - 1, 2**31 - 1, 2**31 - 1, 2**31 - 1)
    pre, dec, links = one_pool(used=10000, cap=11099)
    r = o.score(ROUND_MODEL, [1000], [100], pre, dec, links, want_cost=True, want_feas=True)
    assert math.isinf(r.cost[0, 0, 0]) and r.feas[0, 0] == 0
    assert (r.best_p[0], r.best_d[0]) == (-1, -1) and math.isinf(r.best_cost[0])
    pre, dec, links = one_pool(used=10000, cap=11100)
    r = o.score(ROUND_MODEL, [1000], [100], pre, dec, links, want_feas=True)
    assert r.feas[0, 0] == 1 and r.best_p[0] == 0


def test_worked_example_table():
    rows = read_rows("worked_example.txt")
    M = synth.MODEL
    types = synth.type_table(2)
    links = synth.link_table(types)
    cap = np.floor(types["kv_bytes"] / M["kv_bytes_per_token"]).astype(np.int32)
    assert list(cap) == [305175, 610351]
    pre = dict(flops=types["flops"], hbm_bw=types["hbm_bw"], backlog_tok=[8000, 16000], type=[0, 1])
    dec = dict(flops=types["flops"], hbm_bw=types["hbm_bw"], used_tok=[100000, 600000], cap_tok=cap,
               batch=[16, 32], qd_tok=[0, 640], type=[0, 1])
    calls = [r for r in rows if r[0] in ("c0", "c1", "c2")]
    L = [int(r[1]) for r in calls]
    O = [int(r[2]) for r in calls]
    res = o.score(M, L, O, pre, dec, links, want_cost=True)
    for i, r in enumerate(calls):
        want = np.array([float(x) for x in r[3:7]])
        got = res.cost[i].reshape(-1)
        assert np.array_equal(np.isinf(want), np.isinf(got))
        fin = np.isfinite(want)
        assert np.allclose(got[fin], want[fin], rtol=0, atol=6e-7)
        assert (res.best_p[i], res.best_d[i]) == (int(r[7]), int(r[8]))
    nc = o.node_cost(M, L, O, types, links)
    want_nc = [float(x) for x in [r for r in rows if r[0] == "node_cost"][0][1:]]
    assert np.allclose(nc, want_nc, rtol=0, atol=6e-7)
    # critical path of the fan-out c0 -> {c1, c2} on those costs
    rem, tail, level, hor = o.critical_path([0, 2, 2, 2], [1, 2], nc, [0, 3], round_f32=False)
    get = lambda k: [float(x) for x in [r for r in rows if r[0] == k][0][1:]]
    assert np.allclose(rem, get("rem"), atol=6e-7) and np.allclose(tail, get("tail"), atol=6e-7)
    assert list(level) == [int(x) for x in get("level")]
    assert hor[0] == pytest.approx(get("horizon")[0], abs=6e-7)
    ratio = o.urgency([1.0], [res.best_cost[2]], [2], [0], tail, hor)
    assert ratio[0] == pytest.approx(get("ratio_c2")[0], abs=6e-7)


def test_urgency_round():
    # Eq. (2) with the tail of the call's node
    r = o.urgency([2.0], [3.0], [0], [0], [1.0], [4.0])
    assert r[0] == pytest.approx(G["urgency"], rel=TOL)
    # a leaf of the revealed DAG: exactly Eq. (2)
    r = o.urgency([2.0], [3.0], [0], [0], [0.0], [4.0])
    assert r[0] == pytest.approx((2.0 + 3.0) / 4.0, rel=TOL)
    # node and workflow indices are not swapped
    r = o.urgency([0.0], [1.0], [1], [0], [10.0, 20.0], [7.0, 1e9])
    assert r[0] == pytest.approx(21.0 / 7.0, rel=TOL)
    # a workflow without a horizon (Eq. (2) is undefined there): as urgent as can be, also for a zero numerator
    r = o.urgency([2.0, 0.0], [3.0, 0.0], [0, 0], [0, 0], [0.0], [0.0])
    assert np.isposinf(r).all()
    # nothing feasible: +inf over any horizon
    assert np.isposinf(o.urgency([2.0], [np.inf], [0], [0], [0.0], [4.0])[0])


@pytest.mark.parametrize("field,side", [("backlog_tok", "pre"), ("qd_tok", "dec"), ("used_tok", "dec"), ("batch", "dec")])
def test_cost_monotone_in_load(field, side):
    # queues, occupancy and batch only ever delay (Sec. 4.2 resource model)
    rng = np.random.default_rng(11)
    M = synth.MODEL
    types, pre, dec, links = random_pool(rng, 3, 3, 2)
    dec["cap_tok"] = np.full(3, 2 * 10**6, np.int32)
    L, O = [700, 5000, 30000], [50, 400, 3000]
    base = o.score(M, L, O, pre, dec, links, want_cost=True).cost
    tab = pre if side == "pre" else dec
    for bump in (1, 100, 10000):
        t2 = dict(tab); t2[field] = np.asarray(tab[field]) + bump
        c2 = o.score(M, L, O, t2 if side == "pre" else pre, t2 if side == "dec" else dec, links, want_cost=True).cost
        assert (c2 >= base).all()
    assert (c2 > base).any()


def test_cost_antimonotone_in_rates_and_bandwidth():
    rng = np.random.default_rng(12)
    M = synth.MODEL
    types, pre, dec, links = random_pool(rng, 3, 3, 2)
    dec["cap_tok"] = np.full(3, 2 * 10**6, np.int32)
    L, O = [700, 5000, 30000], [50, 400, 3000]
    base = o.score(M, L, O, pre, dec, links, want_cost=True).cost
    for key, side in (("flops", "pre"), ("hbm_bw", "pre"), ("flops", "dec"), ("hbm_bw", "dec")):
        tab = dict(pre if side == "pre" else dec)
        tab[key] = (np.asarray(tab[key]) * 1.5).astype(np.float32)
        c2 = o.score(M, L, O, tab if side == "pre" else pre, tab if side == "dec" else dec, links, want_cost=True).cost
        assert (c2 <= base).all()
    l2 = dict(links, bw=links["bw"] * 0.5)        # cross-class transfers over a slower link cost more
    c2 = o.score(M, L, O, pre, dec, l2, want_cost=True).cost
    assert (c2 >= base).all()
    d0 = dict(dec, qd_tok=np.zeros(3, np.int32))   # no decode queue: the transfer is on the critical path
    b0 = o.score(M, L, O, pre, d0, links, want_cost=True).cost
    c0 = o.score(M, L, O, pre, d0, l2, want_cost=True).cost
    assert (c0 > b0).all()


def test_scaling_all_rates_scales_all_costs():
    # a uniform multiplicative error on every estimate leaves every choice
    # unchanged (cf. the robustness experiment, Sec. 7.6)
    rng = np.random.default_rng(13)
    M = synth.MODEL
    types, pre, dec, links = random_pool(rng, 4, 4, 3)
    links["latency"] = None
    L, O = synth.gen_lengths(rng, 40)
    base = o.score(M, L, O, pre, dec, links, want_cost=True)
    k = 2.0   # power of two: fp32 rates scale exactly
    p2 = dict(pre, flops=pre["flops"] * k, hbm_bw=pre["hbm_bw"] * k)
    d2 = dict(dec, flops=dec["flops"] * k, hbm_bw=dec["hbm_bw"] * k)
    l2 = dict(links, bw=links["bw"] * k)
    sc = o.score(M, L, O, p2, d2, l2, want_cost=True)
    fin = np.isfinite(base.cost)
    assert np.array_equal(fin, np.isfinite(sc.cost))
    assert np.allclose(sc.cost[fin] * k, base.cost[fin], rtol=1e-14)
    assert np.array_equal(sc.best_p, base.best_p) and np.array_equal(sc.best_d, base.best_d)


def test_node_cost_round():
    links = dict(n_types=1, bw=np.array([[1e9]], np.float32), latency=None)
    types = dict(flops=np.array([1e13], np.float32), hbm_bw=np.array([1e12], np.float32))
    nc = o.node_cost(ROUND_MODEL, [1000], [100], types, links)
    assert nc[0] == pytest.approx(G["node_cost_memory_bound_decode"], rel=1e-6)
    types = dict(flops=np.array([1e10], np.float32), hbm_bw=np.array([1e12], np.float32))
    nc = o.node_cost(ROUND_MODEL, [1000], [100], types, links)
    assert nc[0] == pytest.approx(G["node_cost_compute_bound_decode"], rel=1e-6)


def test_node_cost_is_best_pair_on_idle_pool():
    # R9 = min over class pairs of R7 on an idle pool holding one instance per class
    rng = np.random.default_rng(14)
    M = synth.MODEL
    T = 3
    types, _, _, links = random_pool(rng, 1, 1, T)
    L, O = synth.gen_lengths(rng, 30)
    ty = np.arange(T, dtype=np.int32)
    pre = dict(flops=types["flops"], hbm_bw=types["hbm_bw"], backlog_tok=np.zeros(T, np.int32), type=ty)
    dec = dict(flops=types["flops"], hbm_bw=types["hbm_bw"], used_tok=np.zeros(T, np.int32),
               cap_tok=np.full(T, 2**30, np.int32), batch=np.zeros(T, np.int32), qd_tok=np.zeros(T, np.int32), type=ty)
    r = o.score(M, L, O, pre, dec, links)
    nc = o.node_cost(M, L, O, types, links)
    assert np.allclose(nc, r.best_cost, rtol=1e-14)
