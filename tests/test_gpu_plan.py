"""GPU parity of the planner around the scoring loop: one-pass ordering and the
recomputing greedy loop (Algorithm 1 main loop; Sec. 5.3), through the C ABI.

The greedy sequence is chaotic under fp32 near-ties (a different pick changes
every later state), so the plan is checked step by step: the oracle replays the
GPU's order on its own copy of the state, and at every step the GPU's call must
be a most-urgent one and its pair an earliest-finish one up to the fp32
tolerance; only then is it applied to the oracle's state.  Integer state must
agree exactly at the end."""
import numpy as np
import pytest

from oracle import hx_oracle as o
from paper_2605_16637_amd import synth
from gpu_helpers import REL, assert_costs_close, dev
from helpers import random_pool

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    from paper_2605_16637_amd import binding
    c = binding.Context(0)
    yield c
    c.close()


@pytest.mark.parametrize("C", [1, 7, 2048, 2049, 16384, 16385, 40000, 100003])
def test_rank_matches_oracle(ctx, C):
    import torch
    rng = np.random.default_rng(60 + C)
    r = rng.choice(np.concatenate([rng.uniform(0.1, 5.0, 50), [np.inf, 2.0, 2.0]]), C).astype(np.float32)
    want = o.rank(r.astype(np.float64)) if C <= 2049 else None
    rank = torch.full((C,), -1, dtype=torch.int32, device="cuda:0")
    ctx.hx_rank(dev(r), rank)
    ctx.hx_stream_status()
    got = rank.cpu().numpy()
    if want is None:        # the quadratic oracle is too slow here: a stable sort gives the same definition
        order = np.argsort(-r.astype(np.float64), kind="stable")
        want = np.empty(C, np.int64); want[order] = np.arange(C)
    assert np.array_equal(got, want)


def run_greedy(ctx, model, L, O, elapsed, node, wf, tail, hor, pre, dec, links):
    import torch
    from paper_2605_16637_amd import binding
    C, P, D = len(L), len(pre["flops"]), len(dec["flops"])
    calls = binding.to_device(dict(n=C, L_in=np.asarray(L, np.int32), L_out=np.asarray(O, np.int32),
                                   node=np.asarray(node, np.int32), wf=np.asarray(wf, np.int32),
                                   elapsed=np.asarray(elapsed, np.float32)))
    dp = binding.to_device({**{k: np.asarray(v) for k, v in pre.items()}, "n": P})
    dd = binding.to_device({**{k: np.asarray(v) for k, v in dec.items()}, "n": D})
    dl = binding.to_device(links)
    i32 = dict(dtype=torch.int32, device="cuda:0")
    bp, bd, rk = torch.full((C,), -9, **i32), torch.full((C,), -9, **i32), torch.full((C,), -9, **i32)
    bc, rt = torch.full((C,), -9.0, device="cuda:0"), torch.full((C,), -9.0, device="cuda:0")
    st = [torch.full((P,), -9, **i32)] + [torch.full((D,), -9, **i32) for _ in range(3)]
    ctx.hx_plan_greedy(model, calls, dp, dd, dl, dev(np.asarray(tail, np.float32)), dev(np.asarray(hor, np.float32)),
                       bp, bd, bc, rt, rk, *st)
    ctx.hx_stream_status()
    return [x.cpu().numpy() for x in (bp, bd, bc, rt, rk, *st)]


def check_plan_stepwise(model, L, O, elapsed, node, wf, tail, hor, pre, dec, links, got):
    gp, gd, gc, gr, grank, g_bl, g_us, g_ba, g_qd = got
    C = len(L)
    assert sorted(grank) == list(range(C))
    sp = {k: np.array(v).copy() for k, v in pre.items()}
    sd = {k: np.array(v).copy() for k, v in dec.items()}
    alive = list(range(C))
    elapsed = np.asarray(elapsed, np.float32).astype(np.float64)
    tail = np.asarray(tail, np.float32).astype(np.float64); hor = np.asarray(hor, np.float32).astype(np.float64)
    L, O = np.asarray(L), np.asarray(O)
    for k in range(C):
        c = int(np.nonzero(grank == k)[0][0])
        s = o.score(model, L[alive], O[alive], sp, sd, links)
        with np.errstate(all="ignore"):
            R = (elapsed[alive] + s.best_cost + tail[np.asarray(node)[alive]]) / hor[np.asarray(wf)[alive]]
        i = alive.index(c)
        # the picked call is a most urgent one (exactly, or within the fp32 tolerance of the largest ratio)
        top = R.max()
        assert (np.isinf(top) and np.isinf(R[i])) or R[i] >= top * (1 - 2 * REL), f"step {k}: call {c} ratio {R[i]} vs {top}"
        if np.isinf(R[i]):
            assert (gp[c], gd[c]) == (-1, -1) and np.isinf(gc[c]) and np.isinf(gr[c])
            # among calls with nothing feasible the lowest index goes first
            assert c == min(a for a, r in zip(alive, R) if np.isinf(r))
        else:
            assert gp[c] >= 0 and gd[c] >= 0
            alt = o.score_one(model, L[c], O[c], gp[c], gd[c], sp, sd, links)
            assert np.isfinite(alt) and alt <= s.best_cost[i] * (1 + REL), f"step {k}: pair of call {c}"
            assert abs(gc[c] - alt) <= REL * alt
            want_r = (elapsed[c] + alt + tail[node[c]]) / hor[wf[c]]
            assert abs(gr[c] - want_r) <= REL * want_r
            p, d = int(gp[c]), int(gd[c])
            sp["backlog_tok"][p] += L[c]
            sd["qd_tok"][d] += O[c]; sd["used_tok"][d] += L[c] + O[c]
            sd["batch"][d] = min(256, -(-int(sd["used_tok"][d]) // 2048))
        alive.remove(c)
    assert np.array_equal(g_bl, sp["backlog_tok"]) and np.array_equal(g_us, sd["used_tok"])
    assert np.array_equal(g_ba, sd["batch"]) and np.array_equal(g_qd, sd["qd_tok"])


@pytest.mark.parametrize("C,P,D,T,seed", [(3, 2, 2, 2, 1), (24, 8, 8, 3, 2), (64, 8, 10, 3, 3), (40, 64, 64, 4, 4),
                                          (130, 20, 33, 8, 5), (16, 256, 256, 8, 6),
                                          # the queue and pool bench.py times
                                          (256, 64, 64, 4, 7),
                                          # pools searched class by class (more than 64 x 64 pairs)
                                          (60, 100, 90, 5, 8), (48, 70, 256, 3, 9)])
def test_greedy_plan_matches_oracle(ctx, C, P, D, T, seed):
    rng = np.random.default_rng(70 + seed)
    model = synth.MODEL
    types, pre, dec, links = random_pool(rng, P, D, T)
    # tight capacities: calls stop fitting as the plan fills the pool
    dec["cap_tok"] = (dec["used_tok"] + rng.integers(2000, 60000, D)).astype(np.int32)
    L, O = synth.gen_lengths(rng, C)
    elapsed = rng.uniform(0, 20, C).astype(np.float32)
    n_nodes, n_wf = C + 5, 4
    node = rng.permutation(n_nodes)[:C].astype(np.int32); wf = rng.integers(0, n_wf, C).astype(np.int32)
    tail = rng.uniform(0, 5, n_nodes).astype(np.float32); hor = rng.uniform(5, 50, n_wf).astype(np.float32)
    got = run_greedy(ctx, model, L, O, elapsed, node, wf, tail, hor, pre, dec, links)
    check_plan_stepwise(model, L, O, elapsed, node, wf, tail, hor, pre, dec, links, got)
    # and, when no near-tie occurred, the oracle's own plan is the same plan
    want = o.plan_greedy(model, L, O, elapsed, node, wf, tail, hor, pre, dec, links)
    if np.array_equal(got[4], want.rank):
        assert np.array_equal(got[0], want.best_p) and np.array_equal(got[1], want.best_d)
        assert_costs_close(got[2], want.best_cost, "plan cost"); assert_costs_close(got[3], want.ratio, "plan ratio")
        assert np.array_equal(got[5], want.backlog_tok) and np.array_equal(got[6], want.used_tok)


def test_greedy_hand_worked_conflict_on_gpu(ctx):
    from helpers import ROUND_MODEL, read_kv
    G = read_kv("round_numbers.txt")
    pre = dict(flops=np.array([1e13, 1e13], np.float32), hbm_bw=np.array([1e12, 1e12], np.float32),
               backlog_tok=np.zeros(2, np.int32), type=np.zeros(2, np.int32))
    dec = dict(flops=np.array([1e13], np.float32), hbm_bw=np.array([1e12], np.float32), used_tok=np.zeros(1, np.int32),
               cap_tok=np.array([10**6], np.int32), batch=np.zeros(1, np.int32), qd_tok=np.zeros(1, np.int32),
               type=np.zeros(1, np.int32))
    links = dict(n_types=1, bw=np.array([[1e9]], np.float32), latency=np.array([[0.05]], np.float32))
    gp, gd, gc, gr, grank, bl, us, ba, qd = run_greedy(ctx, ROUND_MODEL, [1000, 1000], [100, 100], [1.0, 5.0], [0, 1], [0, 0],
                                                        [0.0, 0.0], [10.0], pre, dec, links)
    assert list(grank) == [1, 0] and list(gp) == [1, 0] and list(gd) == [0, 0]
    assert gc[1] == pytest.approx(G["greedy_A_cost"], rel=REL) and gc[0] == pytest.approx(G["greedy_B_cost"], rel=REL)
    assert gr[1] == pytest.approx(G["greedy_A_ratio"], rel=REL) and gr[0] == pytest.approx(G["greedy_B_ratio"], rel=REL)
    assert list(bl) == [1000, 1000] and list(us) == [2200] and list(qd) == [200] and list(ba) == [2]


@pytest.mark.parametrize("P,D", [(6, 5), (96, 80)])
def test_greedy_breaks_exact_ties_by_lowest_index(ctx, P, D):
    # identical instances on both sides (two classes, all of a class in the same state): every call sees exact ties
    # over many pairs; the plan has to be the oracle's pair for pair, the lowest (p, d) among equals at every step --
    # on a small pool (searched pair by pair) and on a large one (searched class by class)
    rng = np.random.default_rng(P)
    C = 40
    tp, td = (np.arange(P) % 2).astype(np.int32), (np.arange(D) % 2).astype(np.int32)
    F, B = np.array([4e14, 1e15], np.float32), np.array([2e12, 3.3e12], np.float32)
    pre = dict(flops=F[tp], hbm_bw=B[tp], backlog_tok=np.zeros(P, np.int32), type=tp)
    dec = dict(flops=F[td], hbm_bw=B[td], used_tok=np.full(D, 4096, np.int32), cap_tok=np.full(D, 10**6, np.int32),
               batch=np.full(D, 2, np.int32), qd_tok=np.zeros(D, np.int32), type=td)
    links = dict(n_types=2, bw=np.array([[5e10, 2.5e10], [2.5e10, 1e11]], np.float32), latency=np.zeros((2, 2), np.float32))
    L, O = synth.gen_lengths(rng, C)
    elapsed = rng.uniform(0, 20, C).astype(np.float32)
    node = np.arange(C, dtype=np.int32); wf = (np.arange(C) % 4).astype(np.int32)
    tail = rng.uniform(0, 5, C).astype(np.float32); hor = rng.uniform(5, 50, 4).astype(np.float32)
    got = run_greedy(ctx, synth.MODEL, L, O, elapsed, node, wf, tail, hor, pre, dec, links)
    want = o.plan_greedy(synth.MODEL, L, O, elapsed, node, wf, tail, hor, pre, dec, links)
    assert np.array_equal(got[4], want.rank)
    assert np.array_equal(got[0], want.best_p) and np.array_equal(got[1], want.best_d)
    assert_costs_close(got[2], want.best_cost, "plan cost")
    # the first call placed had the whole pool to choose from, all instances of a class equal: it took the first of its classes
    first = int(np.argmin(got[4]))
    assert got[0][first] < 2 and got[1][first] < 2


def test_planner_limits_and_empty_inputs(ctx):
    import torch
    from paper_2605_16637_amd import binding
    rng = np.random.default_rng(80)
    types, pre, dec, links = random_pool(rng, 4, 4, 2)
    L, O = synth.gen_lengths(rng, 5)
    # an empty decode pool: nothing is feasible, calls are ranked by index, the state comes back unchanged
    none = {k: np.asarray(v)[:0] for k, v in dec.items()}
    got = run_greedy(ctx, synth.MODEL, L, O, np.ones(5), np.arange(5), np.zeros(5, int), np.zeros(5), [9.0], pre, none, links)
    assert (got[0] == -1).all() and np.isinf(got[2]).all() and list(got[4]) == [0, 1, 2, 3, 4]
    assert np.array_equal(got[5], pre["backlog_tok"])
    # beyond the queue length the planner takes
    C = 1025
    big = binding.to_device(dict(n=C, L_in=np.ones(C, np.int32), L_out=np.ones(C, np.int32), node=np.zeros(C, np.int32),
                                 wf=np.zeros(C, np.int32), elapsed=np.zeros(C, np.float32)))
    i32 = dict(dtype=torch.int32, device="cuda:0")
    out = [torch.empty(C, **i32), torch.empty(C, **i32), torch.empty(C, device="cuda:0"), torch.empty(C, device="cuda:0"),
           torch.empty(C, **i32)]
    pre["n"], dec["n"] = 4, 4
    with pytest.raises(binding.HxError) as e:
        ctx.hx_plan_greedy(synth.MODEL, big, binding.to_device(pre), binding.to_device(dec), binding.to_device(links),
                           dev(np.zeros(1, np.float32)), dev(np.ones(1, np.float32)), *out)
    assert e.value.code == -2


def test_greedy_rescans_everything_when_a_commit_lowers_a_term(ctx):
    # The snapshot's batch of a decode instance may stand above what the batch rule gives for its occupancy (the
    # interface only asks for batch >= 0).  The first commit on that instance then lowers its per-token time, pairs
    # on it get cheaper, and calls whose current pair is elsewhere must move there: the plan is Algorithm 1's full
    # recomputation only if those calls are scored again.  Compute-bound decode (large FLOP per token) makes the
    # batch term the one that counts; two decode classes, the fast instance starting with the inflated batch.
    rng = np.random.default_rng(91)
    model = dict(synth.MODEL); model["flops_per_token"] = 4e11
    P, D, C = 6, 2, 24
    tp = (np.arange(P) % 2).astype(np.int32); td = np.array([1, 0], np.int32)
    F, B = np.array([4e14, 1e15], np.float32), np.array([2e12, 3.3e12], np.float32)
    pre = dict(flops=F[tp], hbm_bw=B[tp], backlog_tok=rng.integers(0, 3000, P).astype(np.int32), type=tp)
    L, O = synth.gen_lengths(rng, C)
    dec = dict(flops=F[td], hbm_bw=B[td], used_tok=np.array([20000, 20000], np.int32),
               cap_tok=np.array([10**6, 20000 + int(np.median(L + O)) * 6], np.int32),
               batch=np.array([150, 12], np.int32), qd_tok=np.array([500, 500], np.int32), type=td)
    links = dict(n_types=2, bw=np.array([[5e10, 2.5e10], [2.5e10, 1e11]], np.float32), latency=np.zeros((2, 2), np.float32))
    elapsed = rng.uniform(0, 20, C).astype(np.float32)
    node = np.arange(C, dtype=np.int32); wf = (np.arange(C) % 4).astype(np.int32)
    tail = rng.uniform(0, 5, C).astype(np.float32); hor = rng.uniform(5, 50, 4).astype(np.float32)
    want = o.plan_greedy(model, L, O, elapsed, node, wf, tail, hor, pre, dec, links)
    # the case is what it is meant to be: on the snapshot every call prefers instance 1; once a call has gone to
    # instance 0 its batch falls from 150 and most of the remaining calls follow
    snap = o.score(model, L, O, pre, dec, links)
    assert (snap.best_d == 1).all() and want.batch[0] < 150 and (want.best_d == 0).sum() > C // 2
    got = run_greedy(ctx, model, L, O, elapsed, node, wf, tail, hor, pre, dec, links)
    check_plan_stepwise(model, L, O, elapsed, node, wf, tail, hor, pre, dec, links, got)
    assert np.array_equal(got[4], want.rank)
    assert np.array_equal(got[0], want.best_p) and np.array_equal(got[1], want.best_d)
    assert_costs_close(got[2], want.best_cost, "plan cost")
    assert np.array_equal(got[7], want.batch) and np.array_equal(got[6], want.used_tok)
