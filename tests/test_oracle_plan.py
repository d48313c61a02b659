"""Pins of the oracle's ordering and recomputing-greedy loop (Algorithm 1 main
loop; Sec. 5.3: pick the most urgent call, give it the pair with the earliest
projected decode finish, update the simulated availability, recompute).  No GPU."""
import numpy as np
import pytest

from oracle import hx_oracle as o
from paper_2605_16637_amd import synth
from helpers import ROUND_MODEL, random_pool, read_kv

G = read_kv("round_numbers.txt")


def test_rank_is_a_stable_descending_sort():
    rng = np.random.default_rng(51)
    r = rng.choice([0.5, 1.0, 2.0, np.inf, 3.25], 200)      # many ties, some calls with nothing feasible
    rank = o.rank(r)
    order = np.argsort(-r, kind="stable")                    # ties keep increasing index
    want = np.empty(200, np.int64); want[order] = np.arange(200)
    assert np.array_equal(rank, want)
    assert sorted(rank) == list(range(200))


def test_greedy_hand_worked_conflict():
    pre = dict(flops=[1e13, 1e13], hbm_bw=[1e12, 1e12], backlog_tok=[0, 0], type=[0, 0])
    dec = dict(flops=[1e13], hbm_bw=[1e12], used_tok=[0], cap_tok=[10**6], batch=[0], qd_tok=[0], type=[0])
    links = dict(n_types=1, bw=np.array([[1e9]], np.float32), latency=np.array([[0.05]], np.float32))
    r = o.plan_greedy(ROUND_MODEL, [1000, 1000], [100, 100], [1.0, 5.0], [0, 1], [0, 0], [0.0, 0.0], [10.0],
                      pre, dec, links)
    # call 1 (elapsed 5) is A, call 0 is B
    assert list(r.rank) == [1, 0]
    assert (r.best_p[1], r.best_d[1]) == (0, 0) and (r.best_p[0], r.best_d[0]) == (1, 0)
    assert r.best_cost[1] == pytest.approx(G["greedy_A_cost"], rel=1e-6)
    assert r.ratio[1] == pytest.approx(G["greedy_A_ratio"], rel=1e-6)
    assert r.best_cost[0] == pytest.approx(G["greedy_B_cost"], rel=1e-6)
    assert r.ratio[0] == pytest.approx(G["greedy_B_ratio"], rel=1e-6)
    assert list(r.backlog_tok) == [1000, 1000] and list(r.used_tok) == [2200] and list(r.qd_tok) == [200]
    assert list(r.batch) == [2]
    # a one-pass plan on the snapshot would have sent both calls to prefill 0
    snap = o.score(ROUND_MODEL, [1000, 1000], [100, 100], pre, dec, links)
    assert list(snap.best_p) == [0, 0]


def test_greedy_steps_are_argmins_on_the_evolving_state():
    # 3 calls x 2 x 2 (and a few larger cases): replay the plan in rank order with the
    # enumeration oracle (hxo_score) on a state updated by hand; every pick is the
    # most urgent remaining call and its pair the first minimum over all pairs
    rng = np.random.default_rng(52)
    M = synth.MODEL
    for C, P, D, T in [(3, 2, 2, 2), (8, 3, 4, 2), (12, 4, 4, 3)]:
        types, pre, dec, links = random_pool(rng, P, D, T)
        dec["cap_tok"] = (dec["used_tok"] + rng.integers(3000, 40000, D)).astype(np.int32)   # tight: some calls stop fitting
        L, O = synth.gen_lengths(rng, C)
        elapsed = rng.uniform(0, 20, C); tail = rng.uniform(0, 5, C); hor = rng.uniform(5, 50, 2)
        node = np.arange(C, dtype=np.int32); wf = rng.integers(0, 2, C).astype(np.int32)
        r = o.plan_greedy(M, L, O, elapsed, node, wf, tail, hor, pre, dec, links)
        assert sorted(r.rank) == list(range(C))
        state_p = {k: np.array(v).copy() for k, v in pre.items()}
        state_d = {k: np.array(v).copy() for k, v in dec.items()}
        alive = list(range(C))
        for k in range(C):
            c = int(np.nonzero(r.rank == k)[0][0])
            s = o.score(M, L[alive], O[alive], state_p, state_d, links)
            with np.errstate(all="ignore"):
                R = (elapsed[alive] + s.best_cost + tail[node[alive]]) / hor[wf[alive]]
            i = alive.index(c)
            assert i == int(np.argmax(R))                                   # first maximum = lowest index among ties
            assert (r.best_p[c], r.best_d[c]) == (s.best_p[i], s.best_d[i]) and r.best_cost[c] == s.best_cost[i]
            assert r.ratio[c] == R[i] or (np.isinf(r.ratio[c]) and np.isinf(R[i]))
            if s.best_p[i] >= 0:
                p, d = s.best_p[i], s.best_d[i]
                state_p["backlog_tok"][p] += L[c]
                state_d["qd_tok"][d] += O[c]; state_d["used_tok"][d] += L[c] + O[c]
                state_d["batch"][d] = min(256, -(-int(state_d["used_tok"][d]) // 2048))
            alive.remove(c)
        assert np.array_equal(r.backlog_tok, state_p["backlog_tok"]) and np.array_equal(r.used_tok, state_d["used_tok"])
        assert np.array_equal(r.batch, state_d["batch"]) and np.array_equal(r.qd_tok, state_d["qd_tok"])
        # a call that fits nowhere (from the start, or once earlier picks took the room) has
        # infinite ratio when it is picked and is never placed
        none = r.best_p < 0
        assert np.isinf(r.ratio[none]).all() and (r.best_d[none] < 0).all()


def test_greedy_of_one_call_is_the_plain_search():
    rnd = synth.make_round("tiny", 2)
    c = rnd.calls
    s = o.score(rnd.model, c["L_in"][:1], c["L_out"][:1], rnd.pre, rnd.dec, rnd.links)
    r = o.plan_greedy(rnd.model, c["L_in"][:1], c["L_out"][:1], [3.0], [0], [0], [1.5], [20.0], rnd.pre, rnd.dec, rnd.links)
    assert (r.best_p[0], r.best_d[0], r.best_cost[0]) == (s.best_p[0], s.best_d[0], s.best_cost[0])
    assert r.ratio[0] == pytest.approx((3.0 + s.best_cost[0] + 1.5) / 20.0, rel=1e-14) and r.rank[0] == 0
