"""GPU parity of the horizon path (standalone node cost, critical path in its
single-pass and level-synchronous forms, incremental append) and of the
commit step, against the CPU oracle, through the C ABI."""
import numpy as np
import pytest

from oracle import hx_oracle as o
from paper_2605_16637_amd import synth
from gpu_helpers import assert_costs_close, dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    from paper_2605_16637_amd import binding
    c = binding.Context(0)
    yield c
    c.close()


def gpu_cp(ctx, row_ptr, col, cost32, wf_ptr, max_sweeps=0, check=True):
    import torch
    n, n_wf = len(row_ptr) - 1, len(wf_ptr) - 1
    rem = torch.full((n,), -1.0, device="cuda:0"); tail = torch.full((n,), -1.0, device="cuda:0")
    level = torch.full((n,), -1, dtype=torch.int32, device="cuda:0")
    hor = torch.full((n_wf,), -1.0, device="cuda:0")
    ctx.hx_critical_path(dev(np.asarray(row_ptr, np.int32)), dev(np.asarray(col, np.int32)), dev(cost32),
                         dev(np.asarray(wf_ptr, np.int32)), rem, tail, level, hor, max_sweeps=max_sweeps)
    if check:
        ctx.hx_stream_status()
    return rem.cpu().numpy(), tail.cpu().numpy(), level.cpu().numpy(), hor.cpu().numpy()


def assert_cp_bit_exact(got, want):
    rem, tail, level, hor = got
    orem, otail, olevel, ohor = want          # fp64 holders of exact fp32 values
    assert np.array_equal(level, olevel)
    assert np.array_equal(rem, orem.astype(np.float32)) and np.array_equal(rem.astype(np.float64), orem)
    assert np.array_equal(tail.astype(np.float64), otail)
    assert np.array_equal(hor.astype(np.float64), ohor)


@pytest.mark.parametrize("name,seed", [("tiny", 1), ("mid", 1), ("mid", 2)])
def test_node_cost_and_critical_path(ctx, name, seed):
    import torch
    from paper_2605_16637_amd import binding
    rnd = synth.make_round(name, seed)
    d = rnd.dag
    ocost = o.node_cost(rnd.model, d.L_in, d.L_out, rnd.types, rnd.links)
    gcost = torch.empty(d.n_nodes, device="cuda:0")
    ctx.hx_node_cost(rnd.model, dev(d.L_in), dev(d.L_out), dev(rnd.types["flops"]), dev(rnd.types["hbm_bw"]),
                     binding.to_device(rnd.links), gcost)
    ctx.hx_stream_status()
    assert_costs_close(gcost.cpu().numpy(), ocost, "node cost")
    # the pass itself: same fp32 costs into both sides -> identical bits
    cost32 = ocost.astype(np.float32)
    want = o.critical_path(d.succ_row_ptr, d.succ_col, cost32.astype(np.float64), d.wf_ptr, round_f32=True)
    got = gpu_cp(ctx, d.succ_row_ptr, d.succ_col, cost32, d.wf_ptr)
    assert_cp_bit_exact(got, want)
    got = gpu_cp(ctx, d.succ_row_ptr, d.succ_col, cost32, d.wf_ptr, max_sweeps=int(want[2].max()) + 2)
    assert_cp_bit_exact(got, want)
    # and against the fp64 definition, within the fp32 tolerance
    want64 = o.critical_path(d.succ_row_ptr, d.succ_col, ocost, d.wf_ptr, round_f32=False)
    assert_costs_close(got[0], want64[0], "rem"); assert_costs_close(got[3], want64[3], "horizon")
    # whole chain on the GPU: its own node cost into its own pass
    got2 = gpu_cp(ctx, d.succ_row_ptr, d.succ_col, gcost.cpu().numpy(), d.wf_ptr)
    assert np.array_equal(got2[2], want[2])
    assert_costs_close(got2[0], want64[0], "rem, GPU cost"); assert_costs_close(got2[3], want64[3], "horizon, GPU cost")


def test_critical_path_stress_full_size(ctx):
    # 100 000 workflows, 2.0 M nodes, ~3.4 M edges, depth up to 32
    rnd = synth.make_round("cp", 1)
    d = rnd.dag
    assert d.n_wf == 100000 and 1.9e6 < d.n_nodes < 2.1e6
    rng = np.random.default_rng(3)
    cost32 = o.node_cost(rnd.model, d.L_in, d.L_out, rnd.types, rnd.links).astype(np.float32)
    want = o.critical_path(d.succ_row_ptr, d.succ_col, cost32.astype(np.float64), d.wf_ptr, round_f32=True)
    assert 24 <= want[2].max() <= 31
    got = gpu_cp(ctx, d.succ_row_ptr, d.succ_col, cost32, d.wf_ptr)
    assert_cp_bit_exact(got, want)
    got = gpu_cp(ctx, d.succ_row_ptr, d.succ_col, cost32, d.wf_ptr, max_sweeps=int(want[2].max()) + 2)
    assert_cp_bit_exact(got, want)


def test_single_pass_edge_cases(ctx):
    # empty graph, workflows without nodes, one huge workflow (walked outside LDS),
    # more workflows than one block takes
    got = gpu_cp(ctx, [0], [], np.zeros(0, np.float32), [0])
    assert all(x.size == 0 for x in got)
    got = gpu_cp(ctx, [0, 0], [], np.array([2.5], np.float32), [0, 0, 1, 1])
    assert list(got[3]) == [0.0, 2.5, 0.0] and got[0][0] == 2.5 and got[2][0] == 0
    n = 20000                                  # chain longer than the LDS slice
    rng = np.random.default_rng(4)
    cost32 = rng.uniform(0.1, 2.0, n).astype(np.float32)
    row_ptr = np.minimum(np.arange(n + 1), n - 1).astype(np.int32)
    col = np.arange(1, n, dtype=np.int32)
    want = o.critical_path(row_ptr, col, cost32.astype(np.float64), [0, n], round_f32=True)
    assert_cp_bit_exact(gpu_cp(ctx, row_ptr, col, cost32, [0, n]), want)
    assert want[2][0] == n - 1
    dag = synth.gen_dag(rng, 1000, 1, 3, 2, 3)  # 1000 tiny workflows, some of one node
    c32 = rng.uniform(0.1, 2.0, dag.n_nodes).astype(np.float32)
    want = o.critical_path(dag.succ_row_ptr, dag.succ_col, c32.astype(np.float64), dag.wf_ptr, round_f32=True)
    assert_cp_bit_exact(gpu_cp(ctx, dag.succ_row_ptr, dag.succ_col, c32, dag.wf_ptr), want)


def test_sweeps_accept_any_numbering_and_report_cycles(ctx):
    from paper_2605_16637_amd import binding
    rnd = synth.make_round("mid", 4)
    d = rnd.dag
    rng = np.random.default_rng(5)
    cost32 = rng.uniform(0.5, 3.0, d.n_nodes).astype(np.float32)
    perm = rng.permutation(d.n_nodes)
    inv = np.argsort(perm)
    deg = np.diff(d.succ_row_ptr)[inv]
    rp = np.zeros(d.n_nodes + 1, np.int32); rp[1:] = np.cumsum(deg)
    src_old = np.repeat(inv, deg)
    offs = np.arange(int(deg.sum())) - np.repeat(rp[:-1], deg)
    col = perm[d.succ_col[d.succ_row_ptr[src_old] + offs]].astype(np.int32)
    want = o.critical_path(rp, col, cost32[inv].astype(np.float64), [0, d.n_nodes], round_f32=True)
    got = gpu_cp(ctx, rp, col, cost32[inv], [0, d.n_nodes], max_sweeps=int(want[2].max()) + 2)
    assert_cp_bit_exact(got, want)
    # the single pass refuses this numbering instead of returning wrong values silently
    gpu_cp(ctx, rp, col, cost32[inv], [0, d.n_nodes], check=False)
    with pytest.raises(binding.HxError) as e:
        ctx.hx_stream_status()
    assert e.value.code == -3
    # a cycle: no fixed point within the limit
    gpu_cp(ctx, [0, 1, 2, 3], [1, 2, 0], np.ones(3, np.float32), [0, 3], max_sweeps=8, check=False)
    with pytest.raises(binding.HxError) as e:
        ctx.hx_stream_status()
    assert e.value.code == -3
    # too few sweeps for the depth is reported the same way
    gpu_cp(ctx, d.succ_row_ptr, d.succ_col, cost32, d.wf_ptr, max_sweeps=2, check=False)
    with pytest.raises(binding.HxError):
        ctx.hx_stream_status()


@pytest.mark.parametrize("edge,code", [((1, 4), -3),     # into a later workflow that shares the block
                                       ((4, 1), -3),     # backwards, into an earlier workflow
                                       ((2, 2), -3),     # onto itself
                                       ((1, 9), -3),     # past the last node
                                       (None, 0)])
def test_single_pass_reports_edges_that_leave_their_workflow(ctx, edge, code):
    from paper_2605_16637_amd import binding
    # two chains of three nodes, 0-1-2 and 3-4-5, plus one extra edge
    succ = {0: [1], 1: [2], 2: [], 3: [4], 4: [5], 5: []}
    if edge:
        succ[edge[0]] = succ[edge[0]] + [edge[1]]
    row_ptr = np.cumsum([0] + [len(succ[v]) for v in range(6)]).astype(np.int32)
    col = np.array([u for v in range(6) for u in succ[v]], np.int32)
    cost32 = np.arange(1, 7, dtype=np.float32)
    got = gpu_cp(ctx, row_ptr, col, cost32, [0, 3, 6], check=False)
    if code == 0:
        ctx.hx_stream_status()
        assert list(got[0]) == [6.0, 5.0, 3.0, 15.0, 11.0, 6.0] and list(got[3]) == [6.0, 15.0]
        assert list(got[2]) == [2, 1, 0, 2, 1, 0]
    else:
        with pytest.raises(binding.HxError) as e:
            ctx.hx_stream_status()
        assert e.value.code == code
        # the workflow the bad edge does not start in is untouched by it
        other = slice(3, 6) if edge[0] < 3 else slice(0, 3)
        assert list(got[0][other]) == ([15.0, 11.0, 6.0] if edge[0] < 3 else [6.0, 5.0, 3.0])


def _random_forest(rng, sizes, fan_out, p_second=0.5):
    """Workflows of the given sizes, ids parent-first and workflow-contiguous; every node but a workflow's
    first draws one parent (and sometimes a second) among the earlier nodes of its workflow that still
    have fewer than `fan_out` successors."""
    succ, wf_ptr = [], [0]
    for size in sizes:
        base = len(succ)
        succ.extend([] for _ in range(size))
        for i in range(1, size):
            free = [u for u in range(base, base + i) if len(succ[u]) < fan_out]
            for u in set(rng.choice(free, size=min(len(free), 1 + (rng.random() < p_second)), replace=False).tolist()):
                succ[u].append(base + i)
        wf_ptr.append(len(succ))
    row_ptr = np.cumsum([0] + [len(x) for x in succ]).astype(np.int32)
    col = np.array([u for x in succ for u in sorted(x)], np.int32)
    return row_ptr, col, np.array(wf_ptr, np.int32)


@pytest.mark.parametrize("sizes,fan_out,seed", [
    ([40] * 30, 12, 1),                         # nodes with up to 12 successors
    ([3, 900, 5, 700, 1, 650, 20] * 3, 4, 2),   # neighbours that do not fit one block's LDS together
    ([60, 1390, 2, 1400, 1401, 7, 1399], 9, 3), # at and around the most one block stages; wide nodes too
    ([1] * 300 + [2500] + [4] * 100, 3, 4),     # one workflow too large for LDS between small ones
])
def test_single_pass_wide_nodes_and_runs_of_workflows(ctx, sizes, fan_out, seed):
    rng = np.random.default_rng(seed)
    row_ptr, col, wf_ptr = _random_forest(rng, sizes, fan_out)
    assert (np.diff(row_ptr).max() > 4) == (fan_out > 4)
    cost32 = rng.uniform(0.1, 2.0, len(row_ptr) - 1).astype(np.float32)
    want = o.critical_path(row_ptr, col, cost32.astype(np.float64), wf_ptr, round_f32=True)
    assert_cp_bit_exact(gpu_cp(ctx, row_ptr, col, cost32, wf_ptr), want)
    # a wide node with one edge out of its workflow is reported
    wide = int(np.argmax(np.diff(row_ptr)))
    if row_ptr[wide + 1] - row_ptr[wide] > 4 and wf_ptr[1] <= wide:
        col2 = col.copy(); col2[row_ptr[wide + 1] - 1] = 0
        gpu_cp(ctx, row_ptr, col2, cost32, wf_ptr, check=False)
        from paper_2605_16637_amd import binding
        with pytest.raises(binding.HxError) as e:
            ctx.hx_stream_status()
        assert e.value.code == -3


def gpu_horizons(ctx, rnd, row_ptr, col, L_in, L_out, wf_ptr, check=True):
    import torch
    from paper_2605_16637_amd import binding
    n, n_wf = len(row_ptr) - 1, len(wf_ptr) - 1
    f = lambda v: torch.full((n,), v, device="cuda:0")
    cost, rem, tail = f(-1.0), f(-1.0), f(-1.0)
    level = torch.full((n,), -1, dtype=torch.int32, device="cuda:0")
    hor = torch.full((n_wf,), -1.0, device="cuda:0")
    ctx.hx_horizons(rnd.model, dev(np.asarray(row_ptr, np.int32)), dev(np.asarray(col, np.int32)),
                    dev(np.asarray(L_in, np.int32)), dev(np.asarray(L_out, np.int32)),
                    dev(rnd.types["flops"]), dev(rnd.types["hbm_bw"]), binding.to_device(rnd.links),
                    dev(np.asarray(wf_ptr, np.int32)), cost, rem, tail, level, hor)
    if check:
        ctx.hx_stream_status()
    return cost.cpu().numpy(), (rem.cpu().numpy(), tail.cpu().numpy(), level.cpu().numpy(), hor.cpu().numpy())


@pytest.mark.parametrize("name,seed", [("tiny", 1), ("mid", 3), ("large", 1), ("cp", 2)])
def test_horizons_in_one_launch(ctx, name, seed):
    """Node cost and critical path in one launch: the cost within tolerance of the oracle's and bit for
    bit what hx_node_cost gives; the pass bit for bit the oracle's fp32 pass on those costs."""
    import torch
    from paper_2605_16637_amd import binding
    rnd = synth.make_round(name, seed)
    d = rnd.dag
    gcost, got = gpu_horizons(ctx, rnd, d.succ_row_ptr, d.succ_col, d.L_in, d.L_out, d.wf_ptr)
    assert_costs_close(gcost, o.node_cost(rnd.model, d.L_in, d.L_out, rnd.types, rnd.links), "node cost")
    two = torch.empty(d.n_nodes, device="cuda:0")
    ctx.hx_node_cost(rnd.model, dev(d.L_in), dev(d.L_out), dev(rnd.types["flops"]), dev(rnd.types["hbm_bw"]),
                     binding.to_device(rnd.links), two)
    assert np.array_equal(gcost, two.cpu().numpy())
    want = o.critical_path(d.succ_row_ptr, d.succ_col, gcost.astype(np.float64), d.wf_ptr, round_f32=True)
    assert_cp_bit_exact(got, want)


@pytest.mark.parametrize("sizes,fan_out,seed", [
    ([40] * 30, 12, 1), ([3, 900, 5, 700, 1, 650, 20] * 3, 4, 2), ([1] * 300 + [2500] + [4] * 100, 3, 4), ([], 3, 5), ([0, 1, 0], 3, 6)])
def test_horizons_in_one_launch_wide_nodes_and_runs(ctx, sizes, fan_out, seed):
    rng = np.random.default_rng(seed)
    rnd = synth.make_round("tiny", 1)
    row_ptr, col, wf_ptr = _random_forest(rng, sizes, fan_out)
    n = len(row_ptr) - 1
    L_in, L_out = rng.integers(64, 8000, n).astype(np.int32), rng.integers(16, 2000, n).astype(np.int32)
    gcost, got = gpu_horizons(ctx, rnd, row_ptr, col, L_in, L_out, wf_ptr)
    if n == 0:
        assert all(x.size == 0 for x in got[:3]) and list(got[3]) == [0.0] * (len(wf_ptr) - 1)
        return
    assert_costs_close(gcost, o.node_cost(rnd.model, L_in, L_out, rnd.types, rnd.links), "node cost")
    want = o.critical_path(row_ptr, col, gcost.astype(np.float64), wf_ptr, round_f32=True)
    assert_cp_bit_exact(got, want)


def fetch(raw):
    """Copy a borrowed device array of the context to the host (device-to-device copy into a tensor first)."""
    import ctypes
    import torch
    out = torch.empty(raw.numel(), dtype=raw.dtype, device="cuda:0")
    if raw.numel():
        torch.cuda.synchronize()
        hip = ctypes.CDLL("libamdhip64.so")
        rc = hip.hipMemcpy(ctypes.c_void_p(out.data_ptr()), ctypes.c_void_p(raw.addr), ctypes.c_size_t(raw.numel() * 4), 3)
        assert rc == 0
    return out.cpu().numpy()


def view(ctx, n, n_wf):
    rem, tail, level, hor, n_nodes = ctx.hx_dag_view(n_wf)
    assert n_nodes == n
    return fetch(rem), fetch(tail), fetch(level), fetch(hor)


@pytest.mark.parametrize("seed,n_live,rounds", [(1, 40, 12), (2, 700, 8)])
def test_incremental_append_equals_full_recompute(ctx, seed, n_live, rounds):
    gen = synth.StreamGen(seed, n_live, final_lo=4, final_hi=14)
    rng = np.random.default_rng(seed)
    ctx.hx_dag_reserve(200000, 300000, 50000, 16)
    prow = np.zeros(1, np.int32); pcol = np.zeros(0, np.int32)
    cost_all = np.zeros(0, np.float32); wf_all = np.zeros(0, np.int32)
    prev_h = np.zeros(0)
    for r in range(rounds):
        b = gen.next_batch()
        cost32 = rng.uniform(0.2, 4.0, b["n_new"]).astype(np.float32)
        ctx.hx_dag_append(dev(b["parent_row_ptr"]), dev(b["parent_col"]), dev(cost32), dev(b["wf"]))
        ctx.hx_stream_status()
        prow = np.concatenate([prow, prow[-1] + b["parent_row_ptr"][1:]]).astype(np.int32)
        pcol = np.concatenate([pcol, b["parent_col"]]); cost_all = np.concatenate([cost_all, cost32])
        wf_all = np.concatenate([wf_all, b["wf"]])
        n_wf = b["n_wf_total"]
        want = o.critical_path_by_parents(prow, pcol, cost_all.astype(np.float64), wf_all, n_wf, round_f32=True)
        got = view(ctx, cost_all.size, n_wf)
        assert np.array_equal(got[2], want[2])
        assert np.array_equal(got[0].astype(np.float64), want[0]) and np.array_equal(got[1].astype(np.float64), want[1])
        assert np.array_equal(got[3].astype(np.float64), want[3])
        assert (want[3][:prev_h.size] >= prev_h).all()      # horizons only grow under reveal
        prev_h = want[3]
    assert want[2].max() >= 3


def test_observed_costs_replace_estimates(ctx):
    """Sec. 5.1: estimates are replaced by observed latencies when they become known.  Costs of existing nodes
    go up and down; rem, tail and horizons must equal a full recomputation, and appending goes on from there."""
    gen = synth.StreamGen(9, 300, final_lo=5, final_hi=25)
    rng = np.random.default_rng(9)
    ctx.hx_dag_reserve(100000, 150000, 20000, 32)
    prow = np.zeros(1, np.int32); pcol = np.zeros(0, np.int32)
    cost_all = np.zeros(0, np.float32); wf_all = np.zeros(0, np.int32)

    def check(n_wf):
        want = o.critical_path_by_parents(prow, pcol, cost_all.astype(np.float64), wf_all, n_wf, round_f32=True)
        got = view(ctx, cost_all.size, n_wf)
        assert np.array_equal(got[2], want[2])
        for k in (0, 1, 3):
            assert np.array_equal(got[k].astype(np.float64), want[k]), k
        return want

    for r in range(8):
        b = gen.next_batch()
        c32 = rng.uniform(0.2, 4.0, b["n_new"]).astype(np.float32)
        ctx.hx_dag_append(dev(b["parent_row_ptr"]), dev(b["parent_col"]), dev(c32), dev(b["wf"]))
        prow = np.concatenate([prow, prow[-1] + b["parent_row_ptr"][1:]]).astype(np.int32)
        pcol = np.concatenate([pcol, b["parent_col"]]); cost_all = np.concatenate([cost_all, c32]); wf_all = np.concatenate([wf_all, b["wf"]])
        n_wf = b["n_wf_total"]
        if r in (3, 5, 7):
            before = check(n_wf)
            ids = rng.choice(cost_all.size, max(1, cost_all.size // 10), replace=False).astype(np.int32)
            new = (cost_all[ids] * rng.choice([0.0, 0.3, 1.0, 2.5], ids.size)).astype(np.float32)     # down, same, up
            ctx.hx_dag_set_cost(dev(ids), dev(new))
            ctx.hx_stream_status()
            cost_all[ids] = new
            after = check(n_wf)
            assert (after[3] < before[3]).any() and (after[3] > before[3]).any()       # horizons moved both ways
    from paper_2605_16637_amd import binding
    ctx.hx_dag_set_cost(dev(np.array([0, 10**7], np.int32)), dev(np.array([1.0, 1.0], np.float32)))
    with pytest.raises(binding.HxError) as e:
        ctx.hx_stream_status()
    assert e.value.code == -6


def test_append_errors(ctx):
    from paper_2605_16637_amd import binding
    ctx.hx_dag_reserve(8, 8, 2, 4)
    with pytest.raises(binding.HxError) as e:            # beyond the reserved store
        ctx.hx_dag_append(dev(np.zeros(10, np.int32)), dev(np.zeros(0, np.int32)), dev(np.ones(9, np.float32)),
                          dev(np.zeros(9, np.int32)))
    assert e.value.code == -4
    # a parent that is not an earlier node
    ctx.hx_dag_append(dev(np.array([0, 1], np.int32)), dev(np.array([0], np.int32)), dev(np.ones(1, np.float32)),
                      dev(np.zeros(1, np.int32)))
    with pytest.raises(binding.HxError) as e:
        ctx.hx_stream_status()
    assert e.value.code == -3
    # a chain deeper than max_depth is no error: the walks do not go level by level
    ctx.hx_dag_reserve(16, 16, 1, 2)
    ctx.hx_dag_append(dev(np.array([0, 0, 1, 2, 3, 4, 5], np.int32)), dev(np.arange(5, dtype=np.int32)),
                      dev(np.ones(6, np.float32)), dev(np.zeros(6, np.int32)))
    ctx.hx_stream_status()
    rem, tail, level, hor = view(ctx, 6, 1)
    assert list(rem) == [6, 5, 4, 3, 2, 1] and list(level) == [5, 4, 3, 2, 1, 0] and list(hor) == [6]


def chain_and_fan(n_chain, n_fan):
    """A chain 0 <- 1 <- ... and then one node whose parents are the last n_fan chain nodes."""
    rp = np.concatenate([[0], np.arange(n_chain), [n_chain - 1 + n_fan]]).astype(np.int32)       # node 0 has no parent
    col = np.concatenate([np.arange(n_chain - 1), np.arange(n_chain - n_fan, n_chain)]).astype(np.int32)
    return rp, col


def test_append_walks_that_hand_over_to_the_sweeps(ctx):
    """A walk is cut short when more than 16 grown parents wait at once, or after 1024 visited nodes; the rest
    goes level by level.  Both paths must still give the full recomputation, and too few sweeps are reported."""
    from paper_2605_16637_amd import binding
    rng = np.random.default_rng(12)
    for n_chain, n_fan, depth in ((60, 40, 64), (1500, 1, 1500)):
        n = n_chain + 1
        rp, col = chain_and_fan(n_chain, n_fan)
        cost = rng.uniform(0.5, 2.0, n).astype(np.float32)
        ctx.hx_dag_reserve(n + 4, col.size + 4, 1, depth)
        # the chain first, then the node with the many parents
        ctx.hx_dag_append(dev(rp[:n_chain + 1]), dev(col[:n_chain - 1]), dev(cost[:n_chain]), dev(np.zeros(n_chain, np.int32)))
        ctx.hx_stream_status()
        ctx.hx_dag_append(dev(np.array([0, n_fan], np.int32)), dev(col[n_chain - 1:]), dev(cost[n_chain:]), dev(np.zeros(1, np.int32)))
        ctx.hx_stream_status()
        want = o.critical_path_by_parents(rp, col, cost.astype(np.float64), np.zeros(n, np.int32), 1, round_f32=True)
        got = view(ctx, n, 1)
        assert np.array_equal(got[2], want[2])
        for k in (0, 1, 3):
            assert np.array_equal(got[k].astype(np.float64), want[k]), k
    # the 1500-deep chain with room for 3 sweeps only: the cut walk cannot be finished, and says so
    rp, col = chain_and_fan(1500, 1)
    ctx.hx_dag_reserve(1600, 1600, 1, 3)
    ctx.hx_dag_append(dev(rp[:1501]), dev(col[:1499]), dev(np.ones(1500, np.float32)), dev(np.zeros(1500, np.int32)))
    with pytest.raises(binding.HxError) as e:
        ctx.hx_stream_status()
    assert e.value.code == -4


@pytest.mark.parametrize("C", [900, 5000, 200000])      # one launch (small rounds); two launches, few and many workgroups
def test_commit_matches_oracle(ctx, C):
    import torch
    from paper_2605_16637_amd import binding
    rng = np.random.default_rng(6)
    P, D = 37, 53
    L, O = synth.gen_lengths(rng, C)
    bp = rng.integers(-1, P, C).astype(np.int32)
    bd = np.where(bp < 0, -1, rng.integers(0, D, C)).astype(np.int32)
    st = [rng.integers(0, 20000, P).astype(np.int32), rng.integers(0, 300000, D).astype(np.int32),
          rng.integers(0, 200, D).astype(np.int32), rng.integers(0, 20000, D).astype(np.int32)]
    dr = [rng.integers(0, 80 * C, P).astype(np.int32), rng.integers(0, 6 * C, D).astype(np.int32),
          rng.integers(0, 40 * C, D).astype(np.int32)]
    want = o.commit(L, O, bp, bd, *st, *dr)
    assert want[4] == 0
    g = [dev(x.copy()) for x in st]
    calls = binding.to_device(dict(n=C, L_in=L, L_out=O))
    ctx.hx_commit(calls, dev(bp), dev(bd), g[0], g[1], g[2], g[3], dev(dr[0]), dev(dr[1]), dev(dr[2]))
    ctx.hx_stream_status()
    for got, w in zip(g, want[:4]):
        assert np.array_equal(got.cpu().numpy(), w)
    # overflow and a placement outside the pool are reported
    big = binding.to_device(dict(n=2, L_in=np.array([2**30, 2**30], np.int32), L_out=np.array([16, 16], np.int32)))
    g = [dev(np.zeros(1, np.int32)) for _ in range(4)]
    ctx.hx_commit(big, dev(np.zeros(2, np.int32)), dev(np.zeros(2, np.int32)), *g)
    with pytest.raises(binding.HxError) as e:
        ctx.hx_stream_status()
    assert e.value.code == -7
    ctx.hx_commit(big, dev(np.array([3, 0], np.int32)), dev(np.zeros(2, np.int32)), *g)
    with pytest.raises(binding.HxError) as e:
        ctx.hx_stream_status()
    assert e.value.code == -6
