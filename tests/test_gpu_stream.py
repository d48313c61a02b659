"""GPU parity of whole scheduling rounds, and of rounds replayed from a HIP graph.

Streaming: every round reveals new calls (hx_node_cost -> hx_dag_append), scores
them against the current pool snapshot (hx_score_placements with the projected
ratio) and commits the chosen placements (hx_commit).  The oracle runs the same
rounds on its own state; it adopts the GPU's pair for a call only after checking
that the oracle's cost of that pair is within tolerance of the oracle's best."""
import numpy as np
import pytest

from oracle import hx_oracle as o
from paper_2605_16637_amd import synth
from gpu_helpers import REL, assert_costs_close, assert_search_matches, dev, dev_tables
from test_gpu_dag import fetch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    from paper_2605_16637_amd import binding
    c = binding.Context(0)
    yield c
    c.close()


@pytest.mark.parametrize("seed,n_live,rounds,P,D", [(1, 300, 25, 64, 64), (2, 60, 40, 20, 33)])
def test_streaming_rounds(ctx, seed, n_live, rounds, P, D):
    import torch
    from paper_2605_16637_amd import binding
    model = synth.MODEL
    gen = synth.StreamGen(seed, n_live, final_lo=6, final_hi=20)
    rng = np.random.default_rng(100 + seed)
    L0, O0 = synth.gen_lengths(rng, 4000)
    types, links, pre, dec = synth.gen_pool(rng, P, D, 8, L0, O0, near_capacity=True)
    d_links = binding.to_device(links)
    d_pre, d_dec = binding.to_device(pre), binding.to_device(dec)
    tF, tB = dev(types["flops"]), dev(types["hbm_bw"])
    ctx.hx_dag_reserve(400000, 600000, 100000, 24)
    # oracle-side state
    o_pre = {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in pre.items()}
    o_dec = {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in dec.items()}
    prow = np.zeros(1, np.int32); pcol = np.zeros(0, np.int32)
    cost_all = np.zeros(0, np.float64); wf_all = np.zeros(0, np.int32)
    n_diff = n_calls = 0
    for r in range(rounds):
        b = gen.next_batch()
        n_new, n_wf = b["n_new"], b["n_wf_total"]
        # reveal: node cost of the new calls, append
        g_cost = torch.empty(n_new, device="cuda:0")
        ctx.hx_node_cost(model, dev(b["L_in"]), dev(b["L_out"]), tF, tB, d_links, g_cost)
        ctx.hx_dag_append(dev(b["parent_row_ptr"]), dev(b["parent_col"]), g_cost, dev(b["wf"]))
        g_rem, g_tail, g_level, g_hor, n_nodes = ctx.hx_dag_view(n_wf)
        # the ready calls of the round are the calls just revealed
        elapsed = rng.uniform(0, 30, n_new).astype(np.float32)
        calls = dict(n=n_new, L_in=dev(b["L_in"]), L_out=dev(b["L_out"]), node=dev(b["ids"]), wf=dev(b["wf"]),
                     elapsed=dev(elapsed))
        bp = torch.empty(n_new, dtype=torch.int32, device="cuda:0"); bd = torch.empty_like(bp)
        bc = torch.empty(n_new, device="cuda:0"); ratio = torch.empty(n_new, device="cuda:0")
        ctx.hx_score_placements(model, calls, d_pre, d_dec, d_links, tail=g_tail, horizon=g_hor,
                                best_p=bp, best_d=bd, best_cost=bc, ratio=ratio)
        # drains sized to what the round adds, so the pool stays in its regime
        Ls, Os = int(b["L_in"].sum()), int(b["L_out"].sum())
        dp = np.full(P, Ls // P, np.int32); dq = np.full(D, Os // D, np.int32); rl = np.full(D, (Ls + Os) // D, np.int32)
        ctx.hx_commit(calls, bp, bd, d_pre["backlog_tok"], d_dec["used_tok"], d_dec["batch"], d_dec["qd_tok"],
                      dev(dp), dev(dq), dev(rl))
        ctx.hx_stream_status()

        # the same round on the oracle's own state
        o_cost = o.node_cost(model, b["L_in"], b["L_out"], types, links)
        prow = np.concatenate([prow, prow[-1] + b["parent_row_ptr"][1:]]).astype(np.int32)
        pcol = np.concatenate([pcol, b["parent_col"]]); cost_all = np.concatenate([cost_all, o_cost])
        wf_all = np.concatenate([wf_all, b["wf"]])
        rem, tail, level, hor = o.critical_path_by_parents(prow, pcol, cost_all, wf_all, n_wf, round_f32=False)
        assert n_nodes == cost_all.size
        assert np.array_equal(fetch(g_level), level)
        assert_costs_close(fetch(g_rem), rem, "rem"); assert_costs_close(fetch(g_hor), hor, "horizon")
        ores = o.score(model, b["L_in"], b["L_out"], o_pre, o_dec, links)
        gp, gd, gc = bp.cpu().numpy(), bd.cpu().numpy(), bc.cpu().numpy()
        n_diff += assert_search_matches(model, b["L_in"], b["L_out"], o_pre, o_dec, links, ores, gp, gd, gc)
        n_calls += n_new
        want_ratio = o.urgency(elapsed, ores.best_cost, b["ids"], b["wf"], tail, hor)
        assert_costs_close(ratio.cpu().numpy(), want_ratio, "ratio")
        # commit on the oracle's state with the (validated) pairs; integer state must agree exactly
        bl, us, ba, qd, rc = o.commit(b["L_in"], b["L_out"], gp, gd, o_pre["backlog_tok"], o_dec["used_tok"],
                                      o_dec["batch"], o_dec["qd_tok"], dp, dq, rl)
        assert rc == 0
        o_pre["backlog_tok"], o_dec["used_tok"], o_dec["batch"], o_dec["qd_tok"] = bl, us, ba, qd
        assert np.array_equal(d_pre["backlog_tok"].cpu().numpy(), bl)
        assert np.array_equal(d_dec["used_tok"].cpu().numpy(), us)
        assert np.array_equal(d_dec["batch"].cpu().numpy(), ba)
        assert np.array_equal(d_dec["qd_tok"].cpu().numpy(), qd)
    assert n_diff <= max(3, n_calls // 200)
    assert (ores.best_p < 0).mean() < 0.9       # the pool did not drift into "nothing fits"


def test_round_replayed_from_a_hip_graph(ctx):
    # the benchmark replays a captured round; every replay must equal the eager
    # result, with eager work and synchronisation between replays
    import torch
    rnd = synth.make_round("mid", 5)
    d = rnd.dag
    calls, pre, dec, links = dev_tables(rnd)
    from paper_2605_16637_amd import binding
    tF, tB = dev(rnd.types["flops"]), dev(rnd.types["hbm_bw"])
    L_in, L_out = dev(d.L_in), dev(d.L_out)
    rp, col, wp = dev(d.succ_row_ptr), dev(d.succ_col), dev(d.wf_ptr)
    f32 = dict(dtype=torch.float32, device="cuda:0"); i32 = dict(dtype=torch.int32, device="cuda:0")
    cost = torch.empty(d.n_nodes, **f32); rem = torch.empty(d.n_nodes, **f32); tail = torch.empty(d.n_nodes, **f32)
    level = torch.empty(d.n_nodes, **i32); hor = torch.empty(d.n_wf, **f32)
    n = rnd.calls["n"]
    bp = torch.empty(n, **i32); bd = torch.empty(n, **i32); bc = torch.empty(n, **f32); ratio = torch.empty(n, **f32)
    state0 = [pre["backlog_tok"].clone(), dec["used_tok"].clone(), dec["batch"].clone(), dec["qd_tok"].clone()]
    drain_p = torch.full((rnd.pre["n"],), 70000, **i32); drain_q = torch.full((rnd.dec["n"],), 15000, **i32)
    release = torch.full((rnd.dec["n"],), 90000, **i32)

    def reset():
        for t, s in zip((pre["backlog_tok"], dec["used_tok"], dec["batch"], dec["qd_tok"]), state0):
            t.copy_(s)
        for t in (cost, rem, tail, hor, bc, ratio):
            t.fill_(-1.0)
        for t in (level, bp, bd):
            t.fill_(-1)

    def one_round():
        ctx.hx_node_cost(rnd.model, L_in, L_out, tF, tB, links, cost)
        ctx.hx_critical_path(rp, col, cost, wp, rem, tail, level, hor)
        ctx.hx_score_placements(rnd.model, calls, pre, dec, links, tail=tail, horizon=hor,
                                best_p=bp, best_d=bd, best_cost=bc, ratio=ratio)
        ctx.hx_commit(calls, bp, bd, pre["backlog_tok"], dec["used_tok"], dec["batch"], dec["qd_tok"],
                      drain_p, drain_q, release)

    def snapshot():
        torch.cuda.synchronize()
        return [t.cpu().numpy().copy() for t in (cost, rem, tail, level, hor, bp, bd, bc, ratio,
                                                 pre["backlog_tok"], dec["used_tok"], dec["batch"], dec["qd_tok"])]

    reset(); one_round(); one_round()                 # two eager rounds: the second sees the committed state
    want = snapshot()
    ctx.hx_stream_status()
    g = torch.cuda.CUDAGraph()
    reset()
    with torch.cuda.graph(g):
        one_round()
    for rep in range(3):
        reset()
        torch.cuda.synchronize()
        g.replay(); g.replay()
        got = snapshot()
        for a, b in zip(got, want):
            assert np.array_equal(a, b), f"replay {rep} differs from the eager rounds"
        ctx.hx_stream_status()
        # eager work of the program between replays
        one_round()
        torch.cuda.synchronize()
    # the same round as one hx_round call (two launches: the reveal in the search's, the ratio in the commit's), captured
    graph_args = dict(succ_row_ptr=rp, succ_col_idx=col, wf_ptr=wp, L_in=L_in, L_out=L_out,
                      node_cost=cost, rem=rem, tail=tail, level=level, horizon=hor)

    def one_call():
        ctx.hx_round(rnd.model, calls, pre, dec, links, bp, bd, bc, ratio=ratio, type_flops=tF, type_hbm_bw=tB,
                     drain_prefill=drain_p, drain_decode_q=drain_q, release_tok=release, graph=graph_args)

    reset(); one_call()                              # loads what the capture must not load for the first time
    g2 = torch.cuda.CUDAGraph()
    reset()
    with torch.cuda.graph(g2):
        one_call()
    for rep in range(3):
        reset()
        torch.cuda.synchronize()
        g2.replay(); g2.replay()
        for a, b in zip(snapshot(), want):
            assert np.array_equal(a, b), f"replay {rep} of the one-call round differs from the eager rounds"
        ctx.hx_stream_status()
        one_round()
        torch.cuda.synchronize()


def test_prepared_calls_equal_the_calls_they_were_prepared_from(ctx):
    # binding.Context.prepare: the same library calls with their arguments marshalled once; several rounds in a
    # row (the second sees the state the first committed), against the same rounds made call by call
    import torch
    rnd = synth.make_round("tiny", 7)
    d = rnd.dag
    calls, pre, dec, links = dev_tables(rnd)
    tF, tB = dev(rnd.types["flops"]), dev(rnd.types["hbm_bw"])
    L_in, L_out = dev(d.L_in), dev(d.L_out)
    rp, col, wp = dev(d.succ_row_ptr), dev(d.succ_col), dev(d.wf_ptr)
    f32 = dict(dtype=torch.float32, device="cuda:0"); i32 = dict(dtype=torch.int32, device="cuda:0")
    cost = torch.empty(d.n_nodes, **f32); rem = torch.empty(d.n_nodes, **f32); tail = torch.empty(d.n_nodes, **f32)
    level = torch.empty(d.n_nodes, **i32); hor = torch.empty(d.n_wf, **f32)
    n = rnd.calls["n"]
    bp = torch.empty(n, **i32); bd = torch.empty(n, **i32); bc = torch.empty(n, **f32); ratio = torch.empty(n, **f32)
    state = (pre["backlog_tok"], dec["used_tok"], dec["batch"], dec["qd_tok"])
    state0 = [t.clone() for t in state]
    drain = torch.full((rnd.pre["n"],), 3000, **i32), torch.full((rnd.dec["n"],), 500, **i32), torch.full((rnd.dec["n"],), 4000, **i32)

    def one_round():
        ctx.hx_horizons(rnd.model, rp, col, L_in, L_out, tF, tB, links, wp, cost, rem, tail, level, hor)
        ctx.hx_score_placements(rnd.model, calls, pre, dec, links, tail=tail, horizon=hor,
                                best_p=bp, best_d=bd, best_cost=bc, ratio=ratio)
        ctx.hx_commit(calls, bp, bd, *state, *drain)

    def reset():
        for t, s0 in zip(state, state0):
            t.copy_(s0)
        for t in (cost, rem, tail, hor, bc, ratio):
            t.fill_(-1.0)

    def snapshot():
        torch.cuda.synchronize()
        return [t.cpu().numpy().copy() for t in (cost, rem, tail, level, hor, bp, bd, bc, ratio, *state)]

    reset(); one_round(); one_round(); one_round()
    want = snapshot()
    ctx.hx_stream_status()
    reset()
    torch.cuda.synchronize()
    before = snapshot()
    prepared = ctx.prepare(one_round)
    assert prepared.n_calls == 3
    for a, b in zip(snapshot(), before):
        assert np.array_equal(a, b)                      # preparing calls nothing
    prepared(); prepared(); prepared()
    for a, b in zip(snapshot(), want):
        assert np.array_equal(a, b)
    ctx.hx_stream_status()


@pytest.mark.parametrize("P,D,n_live,rounds,cap", [
    (48, 40, 150, 6, 200000),           # a small search: one prefill instance per lane
    (512, 512, 20000, 3, 700000),       # the streaming configuration's shape: the search fills the chip, four per lane
    (100, 300, 3000, 3, 300000),        # two per lane, ragged
])
def test_round_in_one_call_equals_its_four_calls(ctx, P, D, n_live, rounds, cap):
    # hx_round = hx_node_cost -> hx_dag_append -> hx_score_placements (fused, with the ratio) -> hx_commit, enqueued by
    # one library call (in fewer launches: the cost in the append's first kernel, the walks in the search's launch, the
    # ratio in the commit's): a few streaming rounds made both ways on two contexts' graphs and two copies of the pool,
    # bit for bit
    import torch
    from paper_2605_16637_amd import binding
    model = synth.MODEL
    rng = np.random.default_rng(5)
    L0, O0 = synth.gen_lengths(rng, 4000)
    types, links, pre, dec = synth.gen_pool(rng, P, D, 8, L0, O0, near_capacity=True)
    d_links = binding.to_device(links)
    tF, tB = dev(types["flops"]), dev(types["hbm_bw"])
    other = binding.Context(0)
    try:
        pools = [(binding.to_device(pre), binding.to_device(dec)) for _ in range(2)]
        for c in (ctx, other):
            c.hx_dag_reserve(cap, cap * 3 // 2, cap // 4 + n_live, 24)
        gens = [synth.StreamGen(9, n_live, final_lo=6, final_hi=20) for _ in range(2)]
        i32 = dict(dtype=torch.int32, device="cuda:0")
        for r in range(rounds):
            outs = []
            for which, (c, gen, (d_pre, d_dec)) in enumerate(zip((ctx, other), gens, pools)):
                b = gen.next_batch()
                n_new, n_wf = b["n_new"], b["n_wf_total"]
                el = np.random.default_rng(100 + r).uniform(0, 30, n_new).astype(np.float32)
                calls = dict(n=n_new, L_in=dev(b["L_in"]), L_out=dev(b["L_out"]), node=dev(b["ids"]), wf=dev(b["wf"]), elapsed=dev(el))
                bp, bd = torch.empty(n_new, **i32), torch.empty(n_new, **i32)
                bc, ratio = torch.empty(n_new, device="cuda:0"), torch.empty(n_new, device="cuda:0")
                cost = torch.empty(n_new, device="cuda:0")
                dr = [dev(np.full(P, 900, np.int32)), dev(np.full(D, 300, np.int32)), dev(np.full(D, 1500, np.int32))]
                if which == 0:
                    c.hx_round(model, calls, d_pre, d_dec, d_links, bp, bd, bc, ratio=ratio, n_wf=n_wf,
                               parent_row_ptr=dev(b["parent_row_ptr"]), parent_col_idx=dev(b["parent_col"]),
                               new_L_in=calls["L_in"], new_L_out=calls["L_out"], new_wf=calls["wf"], new_cost=cost,
                               type_flops=tF, type_hbm_bw=tB, drain_prefill=dr[0], drain_decode_q=dr[1], release_tok=dr[2])
                else:
                    c.hx_node_cost(model, calls["L_in"], calls["L_out"], tF, tB, d_links, cost)
                    c.hx_dag_append(dev(b["parent_row_ptr"]), dev(b["parent_col"]), cost, calls["wf"])
                    _, g_tail, _, g_hor, _ = c.hx_dag_view(n_wf)
                    c.hx_score_placements(model, calls, d_pre, d_dec, d_links, tail=g_tail, horizon=g_hor,
                                          best_p=bp, best_d=bd, best_cost=bc, ratio=ratio)
                    c.hx_commit(calls, bp, bd, d_pre["backlog_tok"], d_dec["used_tok"], d_dec["batch"], d_dec["qd_tok"], *dr)
                c.hx_stream_status()
                g_rem, g_tail, g_level, g_hor, n_nodes = c.hx_dag_view(n_wf)
                outs.append([x.cpu().numpy() for x in (cost, bp, bd, bc, ratio, d_pre["backlog_tok"], d_dec["used_tok"],
                                                       d_dec["batch"], d_dec["qd_tok"])] + [fetch(g_rem), fetch(g_level), fetch(g_hor)])
            for a, b2 in zip(*outs):
                assert np.array_equal(a, b2), f"round {r}"
            assert (outs[0][1] >= 0).any()
        # a round that reveals nothing and one without calls
        d_pre, d_dec = pools[0]
        empty = dict(n=0, L_in=dev(np.zeros(1, np.int32)), L_out=dev(np.zeros(1, np.int32)))
        before = d_dec["used_tok"].clone()
        ctx.hx_round(model, empty, d_pre, d_dec, d_links, torch.empty(1, **i32), torch.empty(1, **i32), torch.empty(1, device="cuda:0"))
        ctx.hx_stream_status()
        assert torch.equal(before, d_dec["used_tok"])
    finally:
        other.close()


def _round_buffers(torch, binding, rnd, seed):
    """Device copies of one synthetic round: inputs, the outputs of the reveal and of the search, drains."""
    d = rnd.dag
    f32 = dict(dtype=torch.float32, device="cuda:0")
    i32 = dict(dtype=torch.int32, device="cuda:0")
    n, P, D = rnd.calls["n"], rnd.pre["n"], rnd.dec["n"]
    rng = np.random.default_rng(seed)
    return dict(
        calls=binding.to_device(rnd.calls), pre=binding.to_device(rnd.pre), dec=binding.to_device(rnd.dec),
        graph=dict(succ_row_ptr=dev(d.succ_row_ptr), succ_col_idx=dev(d.succ_col), wf_ptr=dev(d.wf_ptr),
                   L_in=dev(d.L_in), L_out=dev(d.L_out),
                   node_cost=torch.empty(d.n_nodes, **f32), rem=torch.empty(d.n_nodes, **f32),
                   tail=torch.empty(d.n_nodes, **f32), level=torch.empty(d.n_nodes, **i32), horizon=torch.empty(d.n_wf, **f32)),
        bp=torch.empty(n, **i32), bd=torch.empty(n, **i32), bc=torch.empty(n, **f32), ratio=torch.empty(n, **f32),
        drains=[dev(rng.integers(0, 4000, P).astype(np.int32)), dev(rng.integers(0, 1500, D).astype(np.int32)),
                dev(rng.integers(0, 6000, D).astype(np.int32))])


def _round_state(b):
    g = b["graph"]
    return [x.cpu().numpy() for x in (g["node_cost"], g["rem"], g["tail"], g["level"], g["horizon"], b["bp"], b["bd"], b["bc"],
                                      b["ratio"], b["pre"]["backlog_tok"], b["dec"]["used_tok"], b["dec"]["batch"], b["dec"]["qd_tok"])]


@pytest.mark.parametrize("name,override", [
    ("tiny", {}),
    ("mid", {}),                                           # one prefill instance per lane
    ("mid", dict(C=3000, P=100, D=70, T=3)),               # two per lane, ragged
    ("mid", dict(C=9000, P=300, D=260, T=8)),              # four per lane, several calls per wavefront
    ("mid", dict(C=700, P=5, D=600, T=2)),
    # workflows of up to 600 nodes: more than the reveal's workgroups stage at a time (several runs per workgroup,
    # single workflows walked in global memory), wide fan-out
    ("mid", dict(n_wf=300, size_lo=4, size_hi=600, fanout_max=6, depth_max=40, C=2000)),
])
def test_round_with_its_whole_graph_equals_its_three_calls(ctx, name, override):
    # hx_round with the round's whole graph = hx_horizons -> hx_score_placements (fused, ratio) -> hx_commit:
    # three consecutive rounds on two copies of the pool, everything bit for bit; then a plain hx_commit on both
    import torch
    from paper_2605_16637_amd import binding
    rnd = synth.make_round(name, 3, **override)
    links = binding.to_device(rnd.links)
    tF, tB = dev(rnd.types["flops"]), dev(rnd.types["hbm_bw"])
    a, b = _round_buffers(torch, binding, rnd, 7), _round_buffers(torch, binding, rnd, 7)
    for r in range(3):
        g = a["graph"]
        ctx.hx_horizons(rnd.model, g["succ_row_ptr"], g["succ_col_idx"], g["L_in"], g["L_out"], tF, tB, links, g["wf_ptr"],
                        g["node_cost"], g["rem"], g["tail"], g["level"], g["horizon"])
        ctx.hx_score_placements(rnd.model, a["calls"], a["pre"], a["dec"], links, tail=g["tail"], horizon=g["horizon"],
                                best_p=a["bp"], best_d=a["bd"], best_cost=a["bc"], ratio=a["ratio"])
        ctx.hx_commit(a["calls"], a["bp"], a["bd"], a["pre"]["backlog_tok"], a["dec"]["used_tok"], a["dec"]["batch"],
                      a["dec"]["qd_tok"], *a["drains"])
        ctx.hx_round(rnd.model, b["calls"], b["pre"], b["dec"], links, b["bp"], b["bd"], b["bc"], ratio=b["ratio"],
                     type_flops=tF, type_hbm_bw=tB, drain_prefill=b["drains"][0], drain_decode_q=b["drains"][1],
                     release_tok=b["drains"][2], graph=b["graph"])
        ctx.hx_stream_status()
        for x, y in zip(_round_state(a), _round_state(b)):
            assert np.array_equal(x, y, equal_nan=True), f"round {r}"
        assert (a["bp"] >= 0).any()
    for s in (a, b):
        ctx.hx_commit(s["calls"], s["bp"], s["bd"], s["pre"]["backlog_tok"], s["dec"]["used_tok"], s["dec"]["batch"],
                      s["dec"]["qd_tok"], *s["drains"])
    ctx.hx_stream_status()
    for x, y in zip(_round_state(a), _round_state(b)):
        assert np.array_equal(x, y, equal_nan=True)
    # without the ratio, and with counters at the edge of int32: the same saturation, the same report
    for s in (a, b):
        s["pre"]["backlog_tok"].fill_(2147483000)
    ctx.hx_score_placements(rnd.model, a["calls"], a["pre"], a["dec"], links, best_p=a["bp"], best_d=a["bd"], best_cost=a["bc"])
    ctx.hx_commit(a["calls"], a["bp"], a["bd"], a["pre"]["backlog_tok"], a["dec"]["used_tok"], a["dec"]["batch"],
                  a["dec"]["qd_tok"])
    assert (a["bp"] >= 0).any()
    with pytest.raises(binding.HxError) as e1:
        ctx.hx_stream_status()
    assert e1.value.code == -7     # HX_ERR_OVERFLOW
    ctx.hx_round(rnd.model, b["calls"], b["pre"], b["dec"], links, b["bp"], b["bd"], b["bc"],
                 type_flops=tF, type_hbm_bw=tB, graph=b["graph"])
    with pytest.raises(binding.HxError) as e2:
        ctx.hx_stream_status()
    assert e2.value.code == -7
    for x, y in zip(_round_state(a)[5:8] + _round_state(a)[9:], _round_state(b)[5:8] + _round_state(b)[9:]):
        assert np.array_equal(x, y)


def test_round_takes_one_form_of_reveal(ctx):
    # new nodes for the context's graph, or the round's whole graph: both at once is refused before anything is enqueued
    import torch
    from paper_2605_16637_amd import binding
    rnd = synth.make_round("tiny", 1)
    links = binding.to_device(rnd.links)
    tF, tB = dev(rnd.types["flops"]), dev(rnd.types["hbm_bw"])
    b = _round_buffers(torch, binding, rnd, 1)
    before = [x.clone() for x in (b["pre"]["backlog_tok"], b["dec"]["used_tok"])]
    one = dev(np.zeros(1, np.int32))
    with pytest.raises(binding.HxError) as e:
        ctx.hx_round(rnd.model, b["calls"], b["pre"], b["dec"], links, b["bp"], b["bd"], b["bc"], ratio=b["ratio"],
                     parent_row_ptr=dev(np.zeros(2, np.int32)), parent_col_idx=None, new_L_in=one, new_L_out=one, new_wf=one,
                     new_cost=torch.empty(1, device="cuda:0"), type_flops=tF, type_hbm_bw=tB, graph=b["graph"])
    assert e.value.code == -1      # HX_ERR_INVALID_ARG
    torch.cuda.synchronize()
    assert torch.equal(before[0], b["pre"]["backlog_tok"]) and torch.equal(before[1], b["dec"]["used_tok"])
    ctx.hx_stream_status()
