"""Pins of the oracle's horizon pass (Sec. 5.1: H_w(t) is the isolated
completion time of the revealed sub-DAG, i.e. its longest cost-weighted path;
it is recomputed when calls are revealed and can only grow).  No GPU."""
import itertools

import numpy as np
import pytest

from oracle import hx_oracle as o
from paper_2605_16637_amd import synth


def brute_force(n, row_ptr, col, cost):
    """Enumerate every path; rem = heaviest path starting at v, level = most
    edges on a path starting at v."""
    succ = [list(col[row_ptr[v]:row_ptr[v + 1]]) for v in range(n)]
    rem = np.zeros(n); level = np.zeros(n, np.int64)

    def walk(v, weight, edges, start):
        weight += cost[v]
        rem[start] = max(rem[start], weight)
        level[start] = max(level[start], edges)
        for u in succ[v]:
            walk(u, weight, edges + 1, start)

    for v in range(n):
        walk(v, 0.0, 0, v)
    return rem, level


def small_dag(rng, n, p_edge):
    src, dst = [], []
    for i, j in itertools.combinations(range(n), 2):
        if rng.random() < p_edge:
            src.append(i); dst.append(j)
    src, dst = np.array(src, np.int64), np.array(dst, np.int64)
    order = np.lexsort((dst, src))
    row_ptr = np.zeros(n + 1, np.int32)
    if src.size:
        row_ptr[1:] = np.cumsum(np.bincount(src, minlength=n))
    return row_ptr, dst[order].astype(np.int32)


def test_against_path_enumeration():
    rng = np.random.default_rng(31)
    for trial in range(40):
        n = int(rng.integers(1, 13))
        row_ptr, col = small_dag(rng, n, rng.uniform(0.1, 0.5))
        cost = rng.uniform(0.1, 5.0, n)
        rem, tail, level, hor = o.critical_path(row_ptr, col, cost, [0, n], round_f32=False)
        brem, blevel = brute_force(n, row_ptr, col, cost)
        assert np.allclose(rem, brem, rtol=1e-13)
        assert np.array_equal(level, blevel)
        assert np.allclose(tail, brem - cost, rtol=1e-12, atol=1e-12)
        assert hor[0] == pytest.approx(brem.max(), rel=1e-13)


def test_chain_is_a_suffix_sum():
    n = 50
    rng = np.random.default_rng(32)
    cost32 = rng.uniform(0.1, 5.0, n).astype(np.float32)
    row_ptr = np.minimum(np.arange(n + 1), n - 1).astype(np.int32)
    col = np.arange(1, n, dtype=np.int32)
    rem, tail, level, hor = o.critical_path(row_ptr, col, cost32.astype(np.float64), [0, n], round_f32=True)
    # fp32 running sum from the sink up: one rounding per node
    acc = np.float32(0)
    want = np.zeros(n, np.float32)
    for v in range(n - 1, -1, -1):
        acc = np.float32(cost32[v] + acc)
        want[v] = acc
    assert np.array_equal(rem.astype(np.float32), want) and np.array_equal(rem, want.astype(np.float64))
    assert np.array_equal(level, np.arange(n - 1, -1, -1))
    assert hor[0] == want[0]
    # in fp64 the same chain is the exact suffix sum
    rem64, *_ = o.critical_path(row_ptr, col, cost32.astype(np.float64), [0, n], round_f32=False)
    assert np.allclose(rem64, np.cumsum(cost32[::-1].astype(np.float64))[::-1], rtol=1e-14)


def test_star_and_isolated_nodes():
    # root 0 -> leaves 1..5, node 6 isolated, in a second workflow
    cost = np.array([2.0, 1.0, 7.0, 3.0, 0.5, 4.0, 9.0])
    row_ptr = np.array([0, 5, 5, 5, 5, 5, 5, 5], np.int32)
    col = np.arange(1, 6, dtype=np.int32)
    rem, tail, level, hor = o.critical_path(row_ptr, col, cost, [0, 6, 7], round_f32=False)
    assert rem[0] == 9.0 and tail[0] == 7.0 and level[0] == 1
    assert np.array_equal(rem[1:], cost[1:]) and not tail[1:].any() and not level[1:].any()
    assert list(hor) == [9.0, 9.0]
    # an empty workflow has horizon 0
    *_, hor = o.critical_path(row_ptr, col, cost, [0, 6, 6, 7], round_f32=False)
    assert list(hor) == [9.0, 0.0, 9.0]


def test_numbering_does_not_matter():
    # the oracle does not rely on parent id < child id
    rnd = synth.make_round("tiny", seed=4)
    d = rnd.dag
    rng = np.random.default_rng(33)
    cost = rng.uniform(0.5, 3.0, d.n_nodes)
    rem, tail, level, _ = o.critical_path(d.succ_row_ptr, d.succ_col, cost, d.wf_ptr)
    perm = rng.permutation(d.n_nodes)            # new id of old node v is perm[v]
    inv = np.argsort(perm)
    deg = np.diff(d.succ_row_ptr)[inv]
    rp = np.zeros(d.n_nodes + 1, np.int32); rp[1:] = np.cumsum(deg)
    col = np.concatenate([perm[d.succ_col[d.succ_row_ptr[v]:d.succ_row_ptr[v + 1]]] for v in inv]).astype(np.int32)
    rem2, tail2, level2, _ = o.critical_path(rp, col, cost[inv], [0, d.n_nodes])
    assert np.array_equal(rem2[perm], rem) and np.array_equal(tail2[perm], tail) and np.array_equal(level2[perm], level)


def test_edge_invariants_on_a_mid_round():
    rnd = synth.make_round("mid", seed=1)
    d = rnd.dag
    cost = o.node_cost(rnd.model, d.L_in, d.L_out, rnd.types, rnd.links).astype(np.float32)
    rem, tail, level, hor = o.critical_path(d.succ_row_ptr, d.succ_col, cost.astype(np.float64), d.wf_ptr)
    src = np.repeat(np.arange(d.n_nodes), np.diff(d.succ_row_ptr))
    dst = d.succ_col
    # remaining latency is monotone along edges; every rem is one fp32 add
    assert (rem[src] > rem[dst]).all()
    assert (rem[src] >= (cost[src] + rem[dst].astype(np.float32)).astype(np.float64)).all()
    assert np.array_equal(rem.astype(np.float32), cost + tail.astype(np.float32))
    assert (level[src] >= level[dst] + 1).all()
    tight = np.zeros(d.n_nodes, bool); tight[src[level[src] == level[dst] + 1]] = True
    inner = np.diff(d.succ_row_ptr) > 0
    assert tight[inner].all() and not level[~inner].any() and not tail[~inner].any()
    assert level.max() <= 11                        # depth_max = 12 nodes
    wf = d.wf_of_node
    assert (hor[wf] >= rem).all()
    roots = np.diff(d.parent_row_ptr) == 0
    hmax = np.zeros(d.n_wf); np.maximum.at(hmax, wf[roots], rem[roots])
    assert np.array_equal(hmax, hor)                # a horizon is attained at a source


def test_horizon_only_grows_under_reveal():
    # reveal a workflow node by node: H never shrinks, and the parent-list form
    # equals the successor-list form
    rnd = synth.make_round("tiny", seed=5)
    d = rnd.dag
    rng = np.random.default_rng(34)
    cost = rng.uniform(0.5, 3.0, d.n_nodes).astype(np.float32).astype(np.float64)
    full = o.critical_path(d.succ_row_ptr, d.succ_col, cost, d.wf_ptr)
    by_par = o.critical_path_by_parents(d.parent_row_ptr, d.parent_col, cost, d.wf_of_node, d.n_wf)
    for a, b in zip(full, by_par):
        assert np.array_equal(a, b)
    prev = np.zeros(d.n_wf)
    for k in range(1, d.n_nodes + 1):
        prow = d.parent_row_ptr[:k + 1]
        pcol = d.parent_col[:prow[-1]]
        *_, hor = o.critical_path_by_parents(prow, pcol, cost[:k], d.wf_of_node[:k], d.n_wf)
        assert (hor >= prev).all()
        prev = hor
    assert np.array_equal(prev, full[3])


def test_cycle_is_reported():
    with pytest.raises(ValueError, match="not a DAG"):
        o.critical_path([0, 1, 2, 3], [1, 2, 0], [1.0, 1.0, 1.0], [0, 3])
    with pytest.raises(ValueError, match="not a DAG"):
        o.critical_path([0, 1], [0], [1.0], [0, 1])


def test_reveal_order_pass_against_path_enumeration_and_the_depth_first_form():
    # the one-pass form used on long-lived graphs: same values as enumerating every path (<= 12 nodes),
    # same bits as the depth-first form on streamed graphs, fp64 and fp32-rounding modes
    rng = np.random.default_rng(35)
    for trial in range(40):
        n = int(rng.integers(1, 13))
        row_ptr, col = small_dag(rng, n, rng.uniform(0.1, 0.5))          # edges i -> j with i < j: reveal order
        cost = rng.uniform(0.1, 5.0, n)
        src = np.repeat(np.arange(n), np.diff(row_ptr))
        order = np.lexsort((src, col))
        prow = np.zeros(n + 1, np.int32); prow[1:] = np.cumsum(np.bincount(col, minlength=n)) if col.size else 0
        pcol = src[order].astype(np.int32)
        wf = rng.integers(0, 3, n).astype(np.int32)
        rem, tail, level, hor = o.critical_path_revealed(prow, pcol, cost, wf, 3, round_f32=False)
        brem, blevel = brute_force(n, row_ptr, col, cost)
        assert np.allclose(rem, brem, rtol=1e-13) and np.array_equal(level, blevel)
        assert np.allclose(tail, brem - cost, rtol=1e-12, atol=1e-12)
        for w in range(3):
            assert hor[w] == pytest.approx(brem[wf == w].max() if (wf == w).any() else 0.0, rel=1e-13)
    gen = synth.StreamGen(3, 200, final_lo=6, final_hi=20)
    prow = np.zeros(1, np.int32); pcol = np.zeros(0, np.int32); wf = np.zeros(0, np.int32)
    for r in range(12):
        b = gen.next_batch()
        prow = np.concatenate([prow, prow[-1] + b["parent_row_ptr"][1:]]).astype(np.int32)
        pcol = np.concatenate([pcol, b["parent_col"]]); wf = np.concatenate([wf, b["wf"]])
    cost = rng.uniform(0.05, 9.0, wf.size).astype(np.float32).astype(np.float64)
    for mode in (True, False):
        a = o.critical_path_by_parents(prow, pcol, cost, wf, gen.n_wf, round_f32=mode)
        b = o.critical_path_revealed(prow, pcol, cost, wf, gen.n_wf, round_f32=mode)
        for x, y in zip(a, b):
            assert np.array_equal(x, y)
    assert a[2].max() >= 5                                  # deep enough to mean something
    # a parent that is not older than its child is refused
    with pytest.raises(ValueError):
        o.critical_path_revealed([0, 1, 1], [1], [1.0, 1.0], [0, 0], 1)
