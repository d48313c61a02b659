"""GPU parity of the scoring path (fused search, materialised tensor, select,
projected ratio) against the CPU oracle, through the C ABI."""
import numpy as np
import pytest

from oracle import hx_oracle as o
from paper_2605_16637_amd import synth
from gpu_helpers import REL, assert_costs_close, assert_search_matches, dev, dev_tables, fused
from helpers import random_pool

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    from paper_2605_16637_amd import binding
    c = binding.Context(0)
    yield c
    c.close()


def oracle_round(rnd, **kw):
    return o.score(rnd.model, rnd.calls["L_in"], rnd.calls["L_out"], rnd.pre, rnd.dec, rnd.links, **kw)


@pytest.mark.parametrize("name,seed", [("tiny", 1), ("tiny", 2), ("tiny", 3), ("mid", 1), ("mid", 2)])
def test_fused_search_matches_oracle(ctx, name, seed):
    rnd = synth.make_round(name, seed)
    ores = oracle_round(rnd)
    calls, pre, dec, links = dev_tables(rnd)
    gp, gd, gc = fused(ctx, rnd.model, calls, pre, dec, links)
    ndiff = assert_search_matches(rnd.model, rnd.calls["L_in"], rnd.calls["L_out"], rnd.pre, rnd.dec, rnd.links,
                                  ores, gp, gd, gc)
    assert ndiff <= max(2, len(gp) // 100)        # near-ties are rare


@pytest.mark.parametrize("name,seed", [("tiny", 1), ("mid", 1)])
def test_materialised_tensor_select_and_fused_agree(ctx, name, seed):
    import torch
    rnd = synth.make_round(name, seed, near_capacity=True)
    ores = oracle_round(rnd, want_cost=True, want_feas=True)
    calls, pre, dec, links = dev_tables(rnd)
    C, P, D = rnd.calls["n"], rnd.pre["n"], rnd.dec["n"]
    cost = torch.empty(C * P * D, dtype=torch.float32, device="cuda:0")
    feas = torch.empty(C * D, dtype=torch.uint8, device="cuda:0")
    ctx.hx_score_placements(rnd.model, calls, pre, dec, links, cost=cost, feas=feas)
    ctx.hx_stream_status()
    gcost = cost.cpu().numpy().reshape(C, P, D)
    assert_costs_close(gcost, ores.cost, "cost tensor")
    assert np.array_equal(feas.cpu().numpy().reshape(C, D), ores.feas)      # integer mask: exact
    assert 0.01 < 1 - ores.feas.mean() < 0.5
    # select on the tensor = first minimum of the tensor = what the fused search returns, bit for bit
    bp = torch.empty(C, dtype=torch.int32, device="cuda:0"); bd = torch.empty_like(bp)
    bc = torch.empty(C, dtype=torch.float32, device="cuda:0")
    ctx.hx_select(C, P, D, cost, bp, bd, bc)
    ctx.hx_stream_status()
    flat = gcost.reshape(C, -1)
    am = flat.argmin(axis=1)
    none = np.isinf(flat.min(axis=1))
    assert np.array_equal(bp.cpu().numpy(), np.where(none, -1, am // D))
    assert np.array_equal(bd.cpu().numpy(), np.where(none, -1, am % D))
    assert np.array_equal(bc.cpu().numpy(), flat.min(axis=1))
    fp, fd, fc = fused(ctx, rnd.model, calls, pre, dec, links)
    assert np.array_equal(fp, bp.cpu().numpy()) and np.array_equal(fd, bd.cpu().numpy())
    assert np.array_equal(fc, bc.cpu().numpy())
    # infeasible pairs are never chosen
    ok = fd >= 0
    assert ores.feas[np.nonzero(ok)[0], fd[ok]].all()


SHAPES = [  # C, P, D, T: ragged tails, every lane/slot variant, the limits
    (1, 1, 1, 1), (3, 1, 9, 2), (5, 7, 1, 3), (17, 63, 65, 8), (9, 65, 8, 5), (6, 129, 31, 4),
    (5, 200, 257, 7), (4, 257, 300, 8), (3, 520, 77, 8), (2, 1024, 1024, 8), (70, 300, 70, 3),
]


@pytest.mark.parametrize("C,P,D,T", SHAPES)
def test_fused_search_ragged_shapes(ctx, C, P, D, T):
    rng = np.random.default_rng(1000 + C + P + D)
    types, pre, dec, links = random_pool(rng, P, D, T)
    L, O = synth.gen_lengths(rng, C)
    if C > 2:
        L[1] = 400000                     # fits nowhere: no feasible pair
    model = synth.MODEL
    ores = o.score(model, L, O, pre, dec, links)
    pre["n"], dec["n"] = P, D
    from paper_2605_16637_amd import binding
    calls = binding.to_device(dict(n=C, L_in=L, L_out=O))
    dp, dd, dl = binding.to_device(pre), binding.to_device(dec), binding.to_device(links)
    gp, gd, gc = fused(ctx, model, calls, dp, dd, dl)
    assert_search_matches(model, L, O, pre, dec, links, ores, gp, gd, gc)
    if C > 2:
        assert (gp[1], gd[1]) == (-1, -1) and np.isinf(gc[1])


def test_ties_resolve_to_lowest_flat_index(ctx):
    # homogeneous idle pool: all P*D candidates tie -> (0, 0); then knock out
    # the low indices one at a time
    from paper_2605_16637_amd import binding
    model = synth.MODEL
    P, D = 70, 19
    pre = dict(n=P, flops=np.full(P, 4e14, np.float32), hbm_bw=np.full(P, 2e12, np.float32),
               backlog_tok=np.zeros(P, np.int32), type=np.zeros(P, np.int32))
    dec = dict(n=D, flops=np.full(D, 4e14, np.float32), hbm_bw=np.full(D, 2e12, np.float32),
               used_tok=np.zeros(D, np.int32), cap_tok=np.full(D, 10**6, np.int32), batch=np.zeros(D, np.int32),
               qd_tok=np.zeros(D, np.int32), type=np.zeros(D, np.int32))
    links = dict(n_types=1, bw=np.array([[2.5e10]], np.float32), latency=None)
    L = np.array([64, 1500, 32768], np.int32); O = np.array([16, 300, 4096], np.int32)
    calls = binding.to_device(dict(n=3, L_in=L, L_out=O))
    gp, gd, gc = fused(ctx, model, calls, binding.to_device(pre), binding.to_device(dec), binding.to_device(links))
    assert (gp == 0).all() and (gd == 0).all()
    pre["backlog_tok"][:5] = 9000          # prefill 0..4 slower
    dec["used_tok"][:3] = 999999           # decode 0..2 full
    gp, gd, gc = fused(ctx, model, calls, binding.to_device(pre), binding.to_device(dec), binding.to_device(links))
    ores = o.score(model, L, O, pre, dec, links)
    assert (gp == 5).all() and (gd == 3).all()
    assert np.array_equal(gp, ores.best_p) and np.array_equal(gd, ores.best_d)


def test_projected_ratio(ctx):
    rnd = synth.make_round("mid", 3)
    d = rnd.dag
    cost = o.node_cost(rnd.model, d.L_in, d.L_out, rnd.types, rnd.links).astype(np.float32)
    rem, tail, level, hor = o.critical_path(d.succ_row_ptr, d.succ_col, cost.astype(np.float64), d.wf_ptr)
    ores = oracle_round(rnd)
    want = o.urgency(rnd.calls["elapsed"], ores.best_cost, rnd.calls["node"], rnd.calls["wf"], tail, hor)
    calls, pre, dec, links = dev_tables(rnd)
    gp, gd, gc, gr = fused(ctx, rnd.model, calls, pre, dec, links, tail=dev(tail.astype(np.float32)),
                           horizon=dev(hor.astype(np.float32)), want_ratio=True)
    assert_costs_close(gr, want, "ratio")
    assert (tail[rnd.calls["node"]] > 0).any()       # the downstream-tail term is exercised
    # Eq. (2) recomputed from the GPU's own outputs
    eq2 = (rnd.calls["elapsed"].astype(np.float64) + gc + tail[rnd.calls["node"]]) / hor[rnd.calls["wf"]]
    assert np.allclose(gr, eq2, rtol=1e-6)


def test_ratio_of_a_workflow_without_horizon_and_of_a_bad_index(ctx):
    # Eq. (2) divides by the horizon: a horizon of 0 gives +inf whatever the numerator (the oracle's reading), an
    # index outside the arrays gives NaN and is reported -- through hx_score_placements and through hx_urgency
    import torch
    from paper_2605_16637_amd import binding
    rnd = synth.make_round("tiny", 2)
    n = rnd.calls["n"]
    c = {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in rnd.calls.items()}
    c["node"][:] = np.arange(n) % 5; c["wf"][:] = np.arange(n) % 3
    c["elapsed"][1] = 0.0
    tail = np.array([0.0, 1.0, 2.0, 0.5, 0.0], np.float32); hor = np.array([8.0, 0.0, 3.0], np.float32)
    ores = oracle_round(rnd)
    want = o.urgency(c["elapsed"], ores.best_cost, c["node"], c["wf"], tail, hor)
    assert np.isposinf(want[1::3]).all() and np.isfinite(want[0::3]).all()
    calls = binding.to_device(c)
    _, pre, dec, links = dev_tables(rnd)
    gp, gd, gc, gr = fused(ctx, rnd.model, calls, pre, dec, links, tail=dev(tail), horizon=dev(hor), want_ratio=True)
    assert_costs_close(gr, want, "ratio")
    r2 = torch.empty(n, device="cuda:0")
    ctx.hx_urgency(calls, dev(gc), dev(tail), dev(hor), r2)
    ctx.hx_stream_status()
    assert np.array_equal(r2.cpu().numpy(), gr)
    c["wf"][4] = 3; c["node"][7] = -1
    calls = binding.to_device(c)
    ctx.hx_urgency(calls, dev(gc), dev(tail), dev(hor), r2)
    with pytest.raises(binding.HxError) as e:
        ctx.hx_stream_status()
    assert e.value.code == -6
    got = r2.cpu().numpy()
    bad = np.zeros(n, bool); bad[[4, 7]] = True
    assert np.isnan(got[bad]).all() and np.array_equal(got[~bad], gr[~bad])


def test_large_sweep_every_call_by_enumeration(ctx):
    # the full 16384 x 256 x 256 round in the launch configuration the benchmark
    # times: the oracle enumerates all 256 x 256 pairs of every one of the 16384 calls
    rnd = synth.make_round("large", 1)
    calls, pre, dec, links = dev_tables(rnd)
    gp, gd, gc = fused(ctx, rnd.model, calls, pre, dec, links)
    L, O = rnd.calls["L_in"], rnd.calls["L_out"]
    ores = o.score(rnd.model, L, O, rnd.pre, rnd.dec, rnd.links)
    n_diff = assert_search_matches(rnd.model, L, O, rnd.pre, rnd.dec, rnd.links, ores, gp, gd, gc)
    assert n_diff <= rnd.calls["n"] // 200                      # fp32 near-ties are rare
    need = L.astype(np.int64) + O
    free = rnd.dec["cap_tok"].astype(np.int64) - rnd.dec["used_tok"]
    infeasible = (need[:, None] > free[None, :]).mean()
    assert 0.09 < infeasible < 0.11                              # one (call, decode) pair in ten does not fit
    ok = gd >= 0
    assert (need[ok] <= free[gd[ok]]).all()                     # infeasible never chosen
    assert np.array_equal(~ok, need > free.max())               # "none" exactly when nothing fits
    assert (gc[ok] > 0).all() and np.isinf(gc[~ok]).all()
    assert ((gp[ok] >= 0) & (gp[ok] < rnd.pre["n"])).all()


@pytest.mark.parametrize("name", ["large", "stream"])
def test_full_size_against_the_class_collapsed_search(ctx, name):
    """Every call of the full-size rounds, not a sample.  Transfer time depends on the classes only and
    instances of one class share their rates, so for a fixed decode instance the best prefill instance of a
    class is the one with the shortest queue: the minimum over P x D pairs equals the minimum over
    (classes) x D pairs of a pool that keeps one prefill instance per class.  The oracle enumerates that
    32-times smaller pool for all calls; the GPU enumerates the whole pool."""
    rnd = synth.make_round(name, 1)
    calls, pre, dec, links = dev_tables(rnd)
    gp, gd, gc = fused(ctx, rnd.model, calls, pre, dec, links)
    T = rnd.links["n_types"]
    pt, bl = rnd.pre["type"], rnd.pre["backlog_tok"]
    for t in range(T):      # what the shortcut rests on
        assert np.unique(rnd.pre["flops"][pt == t]).size == 1 and np.unique(rnd.pre["hbm_bw"][pt == t]).size == 1
    keep = np.array([np.nonzero(pt == t)[0][np.argmin(bl[pt == t])] for t in range(T)])      # lowest index among equal queues
    small = {k: (np.asarray(v)[keep] if k != "n" else T) for k, v in rnd.pre.items()}
    L, O = rnd.calls["L_in"], rnd.calls["L_out"]
    ores = o.score(rnd.model, L, O, small, rnd.dec, rnd.links)
    assert_costs_close(gc, ores.best_cost, "best cost, all calls")
    none = ores.best_p < 0
    assert np.array_equal(gp < 0, none) and np.array_equal(gd < 0, none)
    # the pair itself: many pairs share the minimum when the decode instance's availability dominates, and the
    # lowest flat index among them need not be the shortest queue of its class -- so every call's GPU pair is
    # priced by the oracle on the full pool and must reach the collapsed search's minimum
    for c in np.nonzero(~none)[0]:
        alt = o.score_one(rnd.model, L[c], O[c], gp[c], gd[c], rnd.pre, rnd.dec, rnd.links)
        assert alt <= ores.best_cost[c] * (1 + REL), c


def test_empty_inputs(ctx):
    import torch
    from paper_2605_16637_amd import binding
    rnd = synth.make_round("tiny", 1)
    calls, pre, dec, links = dev_tables(rnd)
    empty = dict(calls, n=0)
    bp = torch.full((4,), 5, dtype=torch.int32, device="cuda:0"); bd = bp.clone(); bc = torch.zeros(4, device="cuda:0")
    ctx.hx_score_placements(rnd.model, empty, pre, dec, links, best_p=bp, best_d=bd, best_cost=bc)
    ctx.hx_stream_status()
    assert (bp.cpu().numpy() == 5).all()                          # nothing written
    nopool = dict(dec, n=0)
    gp, gd, gc = fused(ctx, rnd.model, calls, pre, nopool, links)
    assert (gp == -1).all() and (gd == -1).all() and np.isinf(gc).all()


def test_errors_are_reported_not_faulted(ctx):
    import torch
    from paper_2605_16637_amd import binding
    rnd = synth.make_round("tiny", 1)
    calls, pre, dec, links = dev_tables(rnd)
    n = rnd.calls["n"]
    bp = torch.empty(n, dtype=torch.int32, device="cuda:0"); bd = torch.empty_like(bp)
    bc = torch.empty(n, dtype=torch.float32, device="cuda:0")
    with pytest.raises(binding.HxError) as e:                    # no output requested
        ctx.hx_score_placements(rnd.model, calls, pre, dec, links)
    assert e.value.code == -1
    with pytest.raises(binding.HxError) as e:                    # too many classes
        ctx.hx_score_placements(rnd.model, calls, pre, dec, dict(links, n_types=9, bw=torch.ones(81, device="cuda:0")),
                                best_p=bp, best_d=bd, best_cost=bc)
    assert e.value.code == -2
    bad = dict(pre, type=torch.full((rnd.pre["n"],), 5, dtype=torch.int32, device="cuda:0"))
    ctx.hx_score_placements(rnd.model, calls, bad, dec, links, best_p=bp, best_d=bd, best_cost=bc)
    with pytest.raises(binding.HxError) as e:                    # class index out of range, seen on the device
        ctx.hx_stream_status()
    assert e.value.code == -6
    ctx.hx_stream_status()                                        # sticky status was cleared


@pytest.mark.parametrize("C,P,D,T", [(7, 65, 9, 3), (3, 5, 130, 8), (11, 33, 33, 1)])
def test_materialised_tensor_ragged_and_select_with_ratio(ctx, C, P, D, T):
    import torch
    from paper_2605_16637_amd import binding
    rng = np.random.default_rng(2000 + P + D)
    types, pre, dec, links = random_pool(rng, P, D, T)
    L, O = synth.gen_lengths(rng, C)
    L[0], O[0] = 0, 0                       # degenerate lengths: no prefill work, nothing to decode
    if C > 3:
        L[2], O[2] = 0, 77
        L[3], O[3] = 500, 0
    model = synth.MODEL
    ores = o.score(model, L, O, pre, dec, links, want_cost=True, want_feas=True)
    pre["n"], dec["n"] = P, D
    n_nodes, n_wf = 40, 6
    node = rng.integers(0, n_nodes, C).astype(np.int32); wf = rng.integers(0, n_wf, C).astype(np.int32)
    elapsed = rng.uniform(0, 9, C).astype(np.float32)
    tail = rng.uniform(0, 5, n_nodes).astype(np.float32); hor = rng.uniform(1, 50, n_wf).astype(np.float32)
    calls = binding.to_device(dict(n=C, L_in=L, L_out=O, node=node, wf=wf, elapsed=elapsed))
    dp, dd, dl = binding.to_device(pre), binding.to_device(dec), binding.to_device(links)
    cost = torch.empty(C * P * D, dtype=torch.float32, device="cuda:0")
    feas = torch.empty(C * D, dtype=torch.uint8, device="cuda:0")
    i32 = dict(dtype=torch.int32, device="cuda:0")
    fp, fd = torch.empty(C, **i32), torch.empty(C, **i32)
    fc, fr = torch.empty(C, device="cuda:0"), torch.empty(C, device="cuda:0")
    # tensor, mask and fused outputs from one call
    ctx.hx_score_placements(model, calls, dp, dd, dl, tail=dev(tail), horizon=dev(hor), cost=cost, feas=feas,
                            best_p=fp, best_d=fd, best_cost=fc, ratio=fr)
    ctx.hx_stream_status()
    gcost = cost.cpu().numpy().reshape(C, P, D)
    assert_costs_close(gcost, ores.cost, "cost tensor")
    assert np.array_equal(feas.cpu().numpy().reshape(C, D), ores.feas)
    assert_search_matches(model, L, O, pre, dec, links, ores, fp.cpu().numpy(), fd.cpu().numpy(), fc.cpu().numpy())
    sp, sd = torch.empty(C, **i32), torch.empty(C, **i32)
    sc, sr = torch.empty(C, device="cuda:0"), torch.empty(C, device="cuda:0")
    ctx.hx_select(C, P, D, cost, sp, sd, sc, calls=calls, tail=dev(tail), horizon=dev(hor), ratio=sr)
    ctx.hx_stream_status()
    for a, b in ((sp, fp), (sd, fd), (sc, fc), (sr, fr)):            # select == fused, bit for bit
        assert np.array_equal(a.cpu().numpy(), b.cpu().numpy(), equal_nan=True)
    want = o.urgency(elapsed, ores.best_cost, node, wf, tail, hor)
    assert_costs_close(sr.cpu().numpy(), want, "ratio")
    # a node index beyond the tail array is reported, not read
    bad = dict(calls, node=dev(np.full(C, n_nodes, np.int32)))
    ctx.hx_select(C, P, D, cost, sp, sd, sc, calls=bad, tail=dev(tail), horizon=dev(hor), ratio=sr)
    with pytest.raises(binding.HxError) as e:
        ctx.hx_stream_status()
    assert e.value.code == -6


def test_urgency_entry_point_equals_the_fused_epilogue(ctx):
    """Eq. (2) folded in afterwards (hx_urgency) is the ratio hx_score_placements writes, bit for bit."""
    import torch
    rnd = synth.make_round("mid", 4)
    calls, pre, dec, links = dev_tables(rnd)
    d = rnd.dag
    cost = o.node_cost(rnd.model, d.L_in, d.L_out, rnd.types, rnd.links)
    rem, tail, level, hor = o.critical_path(d.succ_row_ptr, d.succ_col, cost, d.wf_ptr)
    t_tail, t_hor = dev(tail.astype(np.float32)), dev(hor.astype(np.float32))
    gp, gd, gc, gr = fused(ctx, rnd.model, calls, pre, dec, links, tail=t_tail, horizon=t_hor, want_ratio=True)
    ratio = torch.full((rnd.calls["n"],), -3.0, device="cuda:0")
    ctx.hx_urgency(calls, dev(gc), t_tail, t_hor, ratio)
    ctx.hx_stream_status()
    assert np.array_equal(ratio.cpu().numpy(), gr)
    want = o.urgency(rnd.calls["elapsed"], gc.astype(np.float64), rnd.calls["node"], rnd.calls["wf"],
                     tail.astype(np.float32).astype(np.float64), hor.astype(np.float32).astype(np.float64))
    assert_costs_close(ratio.cpu().numpy(), want, "ratio")
    # an index outside the arrays is reported, not followed
    from paper_2605_16637_amd import binding
    bad = dict(calls); bad["node"] = dev(np.full(rnd.calls["n"], 10**8, np.int32))
    ctx.hx_urgency(bad, dev(gc), t_tail, t_hor, ratio)
    with pytest.raises(binding.HxError) as e:
        ctx.hx_stream_status()
    assert e.value.code == -6


def test_debug_validation_counts_bad_elements(ctx):
    # the scoring calls check sizes and pointers only; the debug entry point counts out-of-range elements per category
    from paper_2605_16637_amd import binding
    rnd = synth.make_round("mid", 2)
    calls, pre, dec, links = dev_tables(rnd)
    ok = ctx.hx_validate_round(calls, pre, dec, links, n_nodes=rnd.dag.n_nodes, n_wf=rnd.dag.n_wf)
    assert set(ok) == set(binding.Context.VALIDATE_FIELDS) and not any(ok.values())
    c = {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in rnd.calls.items()}
    p = {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in rnd.pre.items()}
    d = {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in rnd.dec.items()}
    l = {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in rnd.links.items()}
    c["L_in"][[3, 9]] = -1; c["L_out"][5] = -7; c["node"][0] = rnd.dag.n_nodes; c["wf"][[1, 2, 4000]] = -1
    c["elapsed"][[10, 11, 12]] = [np.nan, np.inf, -1.0]
    p["flops"][1] = 0.0; p["hbm_bw"][2] = np.nan; p["backlog_tok"][[7, 8]] = -5; p["type"][63] = 4
    d["flops"][0] = -1e12; d["cap_tok"][3] = -1; d["qd_tok"][3] = -1; d["batch"][9] = -2; d["type"][[5, 6]] = [-1, 99]
    l["bw"] = np.array(l["bw"], np.float32).copy(); l["bw"].reshape(-1)[5] = np.inf
    with pytest.raises(binding.HxError) as e:
        ctx.hx_validate_round(binding.to_device(c), binding.to_device(p), binding.to_device(d), binding.to_device(l),
                              n_nodes=rnd.dag.n_nodes, n_wf=rnd.dag.n_wf)
    assert e.value.code == -1 and "L_in" in str(e.value)
    assert e.value.report == dict(L_in=2, L_out=1, node=1, wf=3, elapsed=3, prefill_rate=2, prefill_backlog=2, prefill_type=1,
                                  decode_rate=1, decode_state=2, decode_type=2, link=1)
    # an empty round and an empty pool are fine
    none = dict(calls, n=0)
    assert not any(ctx.hx_validate_round(none, dict(pre, n=0), dict(dec, n=0), links).values())
