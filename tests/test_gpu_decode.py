"""GPU parity of the decode stage (Sec. 5.4: capacity-feasible start on token-capacity
intervals, instance locks, decode greedy), through the C ABI.

Start times are not arithmetic results: a start is `now` or the end of one of the instance's
intervals, so it is compared bit for bit.  Which of those it is depends on fp32 comparisons of
decode time against gaps of the timeline; where the GPU's start differs from the oracle's, it
must still lie between the oracle's starts for a decode time a shade shorter and a shade longer
(the start is monotone in the decode time), and such cases must be rare."""
import numpy as np
import pytest

from oracle import hx_oracle as o
from paper_2605_16637_amd import synth
from gpu_helpers import REL, assert_costs_close, dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    from paper_2605_16637_amd import binding
    c = binding.Context(0)
    yield c
    c.close()


def dev_iv(iv):
    return dict(stride=int(iv["stride"]), count=dev(np.asarray(iv["count"], np.int32)),
                start=dev(np.asarray(iv["start"], np.float32)), end=dev(np.asarray(iv["end"], np.float32)),
                tok=dev(np.asarray(iv["tok"], np.int32)))


def dev_queue(L, O, node=None, wf=None, elapsed=None):
    import torch
    q = dict(n=len(L), L_in=dev(np.asarray(L, np.int32)), L_out=dev(np.asarray(O, np.int32)))
    if node is not None:
        q.update(node=dev(np.asarray(node, np.int32)), wf=dev(np.asarray(wf, np.int32)), elapsed=dev(np.asarray(elapsed, np.float32)))
    return q


def dev_dec(dec):
    from paper_2605_16637_amd import binding
    D = len(dec["flops"])
    return binding.to_device({**{k: np.asarray(v) for k, v in dec.items() if k != "n"}, "n": D})


def run_score(ctx, model, L, O, lock, dec, iv, node=None, wf=None, elapsed=None, tail=None, hor=None, want_all=True):
    import torch
    Q, D = len(L), len(dec["flops"])
    f32 = dict(dtype=torch.float32, device="cuda:0")
    bd = torch.full((Q,), -9, dtype=torch.int32, device="cuda:0")
    bs, bc = torch.full((Q,), -9.0, **f32), torch.full((Q,), -9.0, **f32)
    ratio = torch.full((Q,), -9.0, **f32) if tail is not None else None
    st = torch.full((Q * D,), -9.0, **f32) if want_all else None
    co = torch.full((Q * D,), -9.0, **f32) if want_all else None
    ctx.hx_decode_score(model, dev_queue(L, O, node, wf, elapsed), None if lock is None else dev(np.asarray(lock, np.int32)),
                        dev_dec(dec), dev_iv(iv), bd, bs, bc,
                        tail=None if tail is None else dev(np.asarray(tail, np.float32)),
                        horizon=None if hor is None else dev(np.asarray(hor, np.float32)), ratio=ratio, start=st, cost=co)
    ctx.hx_stream_status()
    out = dict(best_d=bd.cpu().numpy(), best_start=bs.cpu().numpy(), best_cost=bc.cpu().numpy())
    if ratio is not None:
        out["ratio"] = ratio.cpu().numpy()
    if want_all:
        out["start"] = st.cpu().numpy().reshape(Q, D)
        out["cost"] = co.cpu().numpy().reshape(Q, D)
    return out


def decode_time(model, L, O, dec, d):
    return float(O) * o.term("decode_token_time", model, int(L), int(O), int(dec["batch"][d]), int(dec["used_tok"][d]),
                             float(np.float32(dec["flops"][d])), float(np.float32(dec["hbm_bw"][d])))


def start_is_valid(model, L, O, dec, iv_lists, d, S_gpu):
    """S_gpu lies between the oracle's starts for a slightly shorter and a slightly longer decode time."""
    s, e, k = iv_lists(d)
    T = decode_time(model, L, O, dec, d)
    slack = REL * (T + (S_gpu if np.isfinite(S_gpu) else 0.0))
    lo = o.decode_start(int(L + O), max(T * (1 - REL) - slack, 0.0), int(dec["cap_tok"][d]), s, e, k)
    hi = o.decode_start(int(L + O), T * (1 + REL) + slack, int(dec["cap_tok"][d]), s, e, k)
    return lo <= S_gpu <= hi


def lists_of(iv):
    K = int(iv["stride"])
    st, en, tk, cnt = (np.asarray(iv[x]) for x in ("start", "end", "tok", "count"))
    return lambda d: (st[d * K:d * K + cnt[d]].astype(np.float64), en[d * K:d * K + cnt[d]].astype(np.float64),
                      tk[d * K:d * K + cnt[d]])


def check_score(model, L, O, lock, dec, iv, got, want, pairs=None):
    """got: GPU outputs with the full tensors; want: oracle DecodeScore with tensors.  Returns the number of
    (call, instance) pairs whose start differs from the oracle's (all of them validated)."""
    Q, D = got["start"].shape
    gs, ws = got["start"].astype(np.float64), want.start
    assert np.array_equal(np.isinf(gs), np.isinf(ws)), "pattern of (call, instance) pairs with no start differs"
    fl = iv_lists = lists_of(iv)
    bad = np.argwhere(gs != ws)
    for c, d in bad:
        assert start_is_valid(model, L[c], O[c], dec, fl, d, gs[c, d]), f"start of call {c} on instance {d}: {gs[c, d]} vs {ws[c, d]}"
    same = gs == ws
    fin = np.isfinite(ws) & same
    err = np.abs(got["cost"].astype(np.float64)[fin] - want.cost[fin]) / np.maximum(want.cost[fin], 1e-30)
    assert err.size == 0 or err.max() <= REL, f"cost: max relative error {err.max():.3e}"
    # selection: the GPU's own tensor decides, bit for bit (lowest instance among equal costs)
    gc = got["cost"]
    row_min = gc.min(axis=1) if D else np.full(Q, np.inf, np.float32)
    want_d = np.where(np.isfinite(row_min), gc.argmin(axis=1) if D else 0, -1)
    assert np.array_equal(got["best_d"], want_d)
    assert np.array_equal(got["best_cost"], row_min)
    rows = np.arange(Q)
    assert np.array_equal(got["best_start"], np.where(want_d >= 0, got["start"][rows, np.maximum(want_d, 0)] if D else np.inf, np.inf))
    # and against the oracle: same instance, or an instance whose oracle cost is within the tolerance of the oracle's best
    diff = np.nonzero(got["best_d"] != want.best_d)[0]
    for c in diff:
        d = got["best_d"][c]
        assert d >= 0 and want.best_d[c] >= 0
        alt = got["start"][c, d] + decode_time(model, L[c], O[c], dec, d)
        assert alt <= want.best_cost[c] * (1 + REL) or not same[c].all(), f"call {c}: instance {d} vs {want.best_d[c]}"
    if lock is not None:
        lk = np.asarray(lock)
        assert ((got["best_d"][lk >= 0] == lk[lk >= 0]) | (got["best_d"][lk >= 0] == -1)).all()
    return len(bad)


@pytest.mark.parametrize("Q,D,stride,res,plan,seed", [(48, 4, 16, 10, 3, 1), (300, 7, 40, 20, 8, 2), (1000, 33, 24, 12, 6, 3),
                                                        (513, 64, 64, 40, 10, 4), (2049, 5, 30, 1, 12, 5),
                                                        # the kernel searches a timeline in one of three ways, by its shape:
                                                        # few planned intervals among many resident ones (all cases above),
                                                        # the same with a timeline too long for its table, mostly planned ones
                                                        (600, 6, 400, 340, 30, 6), (400, 3, 511, 508, 3, 7), (700, 5, 160, 20, 110, 8),
                                                        (300, 4, 300, 1, 290, 9),
                                                        # more instances than groups of them, a queue shorter than a workgroup
                                                        (100, 300, 8, 4, 2, 10), (257, 1, 12, 6, 3, 11)])
def test_decode_score_matches_oracle(ctx, Q, D, stride, res, plan, seed):
    r, lock, iv = synth.make_decode_round("decode_tiny", seed, n_wf=max(8, Q // 8), Q=Q, D=D, T=min(4, D), stride=stride,
                                          n_resident=res, n_planned=plan)
    L, O = r.calls["L_in"], r.calls["L_out"]
    rem, tail, level, hor = o.critical_path(r.dag.succ_row_ptr, r.dag.succ_col, np.random.default_rng(seed).uniform(0.5, 6, r.dag.n_nodes),
                                            r.dag.wf_ptr)
    got = run_score(ctx, r.model, L, O, lock, r.dec, iv, r.calls["node"], r.calls["wf"], r.calls["elapsed"], tail, hor)
    want = o.decode_score(r.model, L, O, lock, r.dec, iv, want_all=True)
    n_bad = check_score(r.model, L, O, lock, r.dec, iv, got, want)
    assert n_bad <= max(2, Q * D // 2000)
    fin = np.isfinite(want.start)
    assert (want.start[fin] > 0).any() and ((want.start[fin] == 0).any() or res < 2)
    # Eq. (2) at the decode stage, from the GPU's own best cost
    el = r.calls["elapsed"].astype(np.float64)
    with np.errstate(all="ignore"):
        want_r = (el + got["best_cost"].astype(np.float64) + tail[r.calls["node"]].astype(np.float32)) / hor[r.calls["wf"]].astype(np.float32)
    assert_costs_close(got["ratio"], want_r, "ratio")
    # free calls only, no tensors requested
    got2 = run_score(ctx, r.model, L, O, None, r.dec, iv, want_all=False)
    want2 = o.decode_score(r.model, L, O, None, r.dec, iv)
    same = got2["best_d"] == want2.best_d
    assert same.mean() > 0.99
    assert np.array_equal(got2["best_start"][same].astype(np.float64), want2.best_start[same])
    assert_costs_close(got2["best_cost"][same], want2.best_cost[same], "best cost of free calls")


def test_decode_score_is_the_same_every_time(ctx):
    # no atomics, no dependence on which workgroup runs first: two passes over the same input agree bit for bit,
    # also with another pass of another shape in between (the scratch is reused)
    r, lock, iv = synth.make_decode_round("decode_mid", 5)
    L, O = r.calls["L_in"], r.calls["L_out"]
    first = run_score(ctx, r.model, L, O, lock, r.dec, iv)
    r2, lock2, iv2 = synth.make_decode_round("decode_tiny", 6)
    run_score(ctx, r2.model, r2.calls["L_in"], r2.calls["L_out"], lock2, r2.dec, iv2)
    again = run_score(ctx, r.model, L, O, lock, r.dec, iv)
    for key in first:
        assert np.array_equal(first[key], again[key]), key


def test_decode_score_edge_cases(ctx):
    import torch
    model = synth.MODEL
    dec = dict(flops=np.array([4e14, 1e15], np.float32), hbm_bw=np.array([2e12, 3.3e12], np.float32),
               used_tok=np.array([1000, 5000], np.int32), cap_tok=np.array([10000, 20000], np.int32),
               batch=np.array([1, 3], np.int32), qd_tok=np.zeros(2, np.int32), type=np.zeros(2, np.int32))
    L = np.array([600, 9000, 15000, 30000, 64, 0], np.int32); O = np.array([100, 1000, 1000, 10, 0, 0], np.int32)
    # no intervals at all: everything that fits starts now
    iv0 = dict(stride=0, count=np.zeros(2, np.int32), start=np.zeros(0, np.float32), end=np.zeros(0, np.float32), tok=np.zeros(0, np.int32))
    iv0d = dict(stride=0, count=dev(np.zeros(2, np.int32)), start=None, end=None, tok=None)
    Q = len(L)
    bd = torch.full((Q,), -9, dtype=torch.int32, device="cuda:0"); bs = torch.full((Q,), -9.0, device="cuda:0"); bc = torch.full((Q,), -9.0, device="cuda:0")
    ctx.hx_decode_score(model, dev_queue(L, O), None, dev_dec(dec), iv0d, bd, bs, bc)
    ctx.hx_stream_status()
    want = o.decode_score(model, L, O, None, dec, iv0)
    assert np.array_equal(bd.cpu().numpy(), want.best_d) and list(want.best_d) == [1, 1, 1, -1, 0, 0]   # the faster instance; nowhere; zero-length decodes tie -> lowest
    assert np.array_equal(bs.cpu().numpy().astype(np.float64), want.best_start)
    assert_costs_close(bc.cpu().numpy(), want.best_cost)
    # degenerate entries hold nothing: empty span, zero tokens, span wholly in the past; equal times; a full list of 511
    K = 511
    rng = np.random.default_rng(9)
    st = np.zeros((2, K), np.float32); en = np.zeros((2, K), np.float32); tk = np.zeros((2, K), np.int32)
    st[0, :6] = [3.0, 1.0, -9.0, 2.0, 2.0, -1.0]; en[0, :6] = [3.0, 5.0, -2.0, 4.0, 4.0, 2.0]; tk[0, :6] = [9000, 0, 9000, 4000, 5000, 9500]
    st[1] = rng.uniform(-5, 20, K).astype(np.float32); en[1] = st[1] + rng.uniform(0.1, 10, K).astype(np.float32)
    tk[1] = rng.integers(1, 150, K)
    iv = dict(stride=K, count=np.array([6, K], np.int32), start=st.reshape(-1), end=en.reshape(-1), tok=tk.reshape(-1))
    lock = np.array([-1, 0, 1, -1, 1, 0], np.int32)
    got = run_score(ctx, model, L, O, lock, dec, iv)
    want = o.decode_score(model, L, O, lock, dec, iv, want_all=True)
    assert check_score(model, L, O, lock, dec, iv, got, want) == 0
    assert want.start[0, 0] == 2.0 and want.start[1, 0] == 4.0      # by hand: 9500 held until 2 (700 do not fit), 9000 from 2 to 4 (10000 do not)
    # no instance, empty queue
    none = {k: v[:0] for k, v in dec.items()}
    ivn = dict(stride=4, count=np.zeros(0, np.int32), start=np.zeros(0, np.float32), end=np.zeros(0, np.float32), tok=np.zeros(0, np.int32))
    g = run_score(ctx, model, L, O, None, none, ivn, want_all=False)
    assert (g["best_d"] == -1).all() and np.isinf(g["best_cost"]).all() and np.isinf(g["best_start"]).all()
    ctx.hx_decode_score(model, dev_queue(L[:0], O[:0]), None, dev_dec(dec), dev_iv(iv), None, None, None)


def test_decode_score_errors(ctx):
    from paper_2605_16637_amd import binding
    r, lock, iv = synth.make_decode_round("decode_tiny", 7)
    L, O = r.calls["L_in"].copy(), r.calls["L_out"].copy()
    bad_lock = lock.copy(); bad_lock[5] = 4          # D = 4: out of range
    with pytest.raises(binding.HxError) as e:
        run_score(ctx, r.model, L, O, bad_lock, r.dec, iv)
    assert e.value.code == -6
    good = run_score(ctx, r.model, L, O, lock, r.dec, iv)            # the sticky status was cleared by reading it
    L2 = L.copy(); L2[3] = -5
    with pytest.raises(binding.HxError) as e:
        run_score(ctx, r.model, L2, O, lock, r.dec, iv)
    assert e.value.code == -6
    cnt = iv["count"].copy(); cnt[1] = iv["stride"] + 1
    with pytest.raises(binding.HxError) as e:
        run_score(ctx, r.model, L, O, lock, r.dec, dict(iv, count=cnt))
    assert e.value.code == -6
    with pytest.raises(binding.HxError) as e:
        run_score(ctx, r.model, L, O, lock, r.dec, widen(iv, 4, 512 - iv["stride"]))
    assert e.value.code == -2
    import torch
    Q = len(L)
    out = [torch.empty(Q, dtype=torch.int32, device="cuda:0"), torch.empty(Q, device="cuda:0"), torch.empty(Q, device="cuda:0")]
    with pytest.raises(binding.HxError) as e:                      # no output arrays
        ctx.hx_decode_score(r.model, dev_queue(L, O), None, dev_dec(r.dec), dev_iv(iv), None, None, None)
    assert e.value.code == -1
    with pytest.raises(binding.HxError) as e:                      # a ratio without node, workflow, elapsed, tail, horizon
        ctx.hx_decode_score(r.model, dev_queue(L, O), None, dev_dec(r.dec), dev_iv(iv), *out, ratio=torch.empty(Q, device="cuda:0"))
    assert e.value.code == -1
    big = 1025                                                     # a queue the one-workgroup planner does not take
    with pytest.raises(binding.HxError) as e:
        run_plan(ctx, r.model, np.full(big, 100), np.full(big, 10), None, np.zeros(big, np.int32), np.zeros(big, np.int32),
                 np.zeros(big, np.float32), [0.0], [10.0], r.dec, iv)
    assert e.value.code == -2
    again = run_score(ctx, r.model, L, O, lock, r.dec, iv)
    assert np.array_equal(again["best_d"], good["best_d"]) and np.array_equal(again["cost"], good["cost"])


def test_decode_score_full_size_sampled(ctx):
    """The benchmark's decode-stage configuration (16384 calls x 256 instances, ~118 intervals each):
    sampled (call, instance) pairs against the oracle one by one, the selection against the GPU's own tensor."""
    r, lock, iv = synth.make_decode_round("decode_large", 1)
    L, O = r.calls["L_in"], r.calls["L_out"]
    got = run_score(ctx, r.model, L, O, lock, r.dec, iv)
    Q, D = got["start"].shape
    gc = got["cost"]
    row_min = gc.min(axis=1)
    assert np.array_equal(got["best_d"], np.where(np.isfinite(row_min), gc.argmin(axis=1), -1))
    assert np.array_equal(got["best_cost"], row_min)
    lk = np.asarray(lock)
    legal = (lk[:, None] < 0) | (lk[:, None] == np.arange(D)[None, :])
    assert np.isinf(got["start"][~legal]).all()
    fl = lists_of(iv)
    rng = np.random.default_rng(11)
    cs = np.concatenate([rng.integers(0, Q, 700), np.nonzero(lk >= 0)[0][:300]])
    ds = np.concatenate([rng.integers(0, D, 700), lk[np.nonzero(lk >= 0)[0][:300]]])
    n_bad = waits = 0
    for c, d in zip(cs, ds):
        if not legal[c, d]:
            continue
        s, e, k = fl(d)
        T = decode_time(r.model, L[c], O[c], r.dec, d)
        S = o.decode_start(int(L[c] + O[c]), T, int(r.dec["cap_tok"][d]), s, e, k)
        g = float(got["start"][c, d])
        if g != S:
            n_bad += 1
            assert start_is_valid(r.model, L[c], O[c], r.dec, fl, d, g), (c, d, g, S)
        elif np.isfinite(S):
            waits += S > 0
            assert abs(float(gc[c, d]) - (S + T)) <= REL * (S + T)
    assert n_bad <= 2 and waits > 50


# ---- recomputing greedy ----------------------------------------------------------------

def run_plan(ctx, model, L, O, lock, node, wf, elapsed, tail, hor, dec, iv):
    import torch
    Q = len(L)
    i32 = dict(dtype=torch.int32, device="cuda:0")
    bd, rk = torch.full((Q,), -9, **i32), torch.full((Q,), -9, **i32)
    bs, bc, rt = (torch.full((Q,), -9.0, device="cuda:0") for _ in range(3))
    div = dev_iv(iv)
    ctx.hx_decode_plan_greedy(model, dev_queue(L, O, node, wf, elapsed), None if lock is None else dev(np.asarray(lock, np.int32)),
                              dev_dec(dec), div, dev(np.asarray(tail, np.float32)), dev(np.asarray(hor, np.float32)),
                              bd, bs, bc, rt, rk)
    ctx.hx_stream_status()
    K = int(iv["stride"])
    D = len(dec["flops"])
    return dict(best_d=bd.cpu().numpy(), best_start=bs.cpu().numpy(), best_cost=bc.cpu().numpy(), ratio=rt.cpu().numpy(),
                rank=rk.cpu().numpy(), count=div["count"].cpu().numpy(), start=div["start"].cpu().numpy().reshape(D, K),
                end=div["end"].cpu().numpy().reshape(D, K), tok=div["tok"].cpu().numpy().reshape(D, K))


def widen(iv, D, extra):
    """The same interval lists with room for `extra` more entries per instance."""
    K0 = int(iv["stride"]); K = K0 + extra
    out = dict(stride=K, count=np.asarray(iv["count"], np.int32).copy())
    for key, dt in (("start", np.float32), ("end", np.float32), ("tok", np.int32)):
        a = np.zeros((D, K), dt)
        a[:, :K0] = np.asarray(iv[key]).reshape(D, K0)
        out[key] = a.reshape(-1)
    return out


def check_plan_stepwise(model, L, O, lock, node, wf, elapsed, tail, hor, dec, iv, got):
    """The oracle replays the GPU's order on its own copy of the intervals: at every step the GPU's call must
    be a most urgent one, its instance an earliest-finish one and its start a valid one, up to the fp32
    tolerance; only then is the GPU's interval appended to the oracle's state."""
    Q, D, K = len(L), len(dec["flops"]), int(iv["stride"])
    assert sorted(got["rank"]) == list(range(Q))
    st = {k: np.asarray(iv[k]).copy() for k in ("start", "end", "tok")}
    cnt = np.asarray(iv["count"], np.int32).copy()
    alive = list(range(Q))
    el = np.asarray(elapsed, np.float32).astype(np.float64)
    tl = np.asarray(tail, np.float32).astype(np.float64); hz = np.asarray(hor, np.float32).astype(np.float64)
    lock_a = None if lock is None else np.asarray(lock, np.int32)
    for k in range(Q):
        c = int(np.nonzero(got["rank"] == k)[0][0])
        cur = dict(stride=K, count=cnt, **st)
        # Which interval end a start is hangs on comparisons of start + decode time against other interval times, and a
        # plan makes exact ties of them (a call placed where another one of the same decode time ended).  fp32 and fp64
        # may then resolve a tie differently, and the start jumps.  So the oracle scores the step twice, with every decode
        # time a shade shorter and a shade longer: the GPU's costs lie between the two, and its pick must be at least as
        # urgent as every call's most optimistic score.
        lk = None if lock_a is None else lock_a[alive]
        shift = 2.5e-7 * (1.0 + float(np.max(st["end"], initial=0.0)))
        s = o.decode_score_bracket(model, L[alive], O[alive], lk, dec, cur, t_scale=1 + REL, t_shift=shift)        # pessimistic
        s_lo = o.decode_score_bracket(model, L[alive], O[alive], lk, dec, cur, t_scale=1 - REL, t_shift=-shift)   # optimistic
        with np.errstate(all="ignore"):
            R = (el[alive] + s_lo.best_cost + tl[np.asarray(node)[alive]]) / hz[np.asarray(wf)[alive]]
        i = alive.index(c)
        top = R.max()
        mine = float(got["ratio"][c])
        assert (np.isinf(top) and np.isinf(R[i])) or mine >= top * (1 - 2 * REL), f"step {k}: call {c} ratio {mine} vs {top}"
        d = int(got["best_d"][c])
        if np.isinf(R[i]):
            # nothing feasible, or a workflow without horizon: infinitely urgent either way, lowest index first
            assert np.isinf(got["ratio"][c])
            assert c == min(a for a, r in zip(alive, R) if np.isinf(r))
        if np.isinf(s_lo.best_cost[i]):
            assert d == -1 and np.isinf(got["best_cost"][c]) and np.isinf(got["best_start"][c])
        else:
            assert d >= 0 and (lock_a is None or lock_a[c] < 0 or lock_a[c] == d)
            S = float(got["best_start"][c])
            assert start_is_valid(model, L[c], O[c], dec, lists_of(cur), d, S), f"step {k}: start of call {c} on {d}"
            alt = S + decode_time(model, L[c], O[c], dec, d)
            assert alt <= s.best_cost[i] * (1 + REL), f"step {k}: instance of call {c}"
            assert abs(got["best_cost"][c] - alt) <= REL * alt
            if hz[wf[c]] > 0:
                want_r = (el[c] + alt + tl[node[c]]) / hz[wf[c]]
                assert abs(got["ratio"][c] - want_r) <= REL * want_r
            at = d * K + cnt[d]
            st["start"][at] = got["best_start"][c]; st["end"][at] = got["best_cost"][c]; st["tok"][at] = L[c] + O[c]
            cnt[d] += 1
        alive.remove(c)
    assert np.array_equal(got["count"], cnt)
    for d in range(D):
        n = cnt[d]
        for key in ("start", "end", "tok"):
            assert np.array_equal(got[key][d, :n], st[key].reshape(D, K)[d, :n]), (d, key)


@pytest.mark.parametrize("Q,D,stride,res,plan,lockf,seed", [(3, 2, 4, 2, 1, 0.5, 1), (40, 4, 16, 10, 3, 0.5, 2), (64, 8, 20, 12, 4, 0.0, 3),
                                                              # (80 x 64 with 96 entries each leaves no local memory for the finish of
                                                              # every pair: the planner then rescans the calls of the changed instance)
                                                              (100, 16, 30, 20, 6, 1.0, 4), (80, 64, 16, 10, 3, 0.3, 5),
                                                              # two instances and long chains of appended intervals: exact ties of start + decode time
                                                              (69, 2, 2, 1, 1, 0.3726785374341105, 760292)])
def test_decode_greedy_matches_oracle(ctx, Q, D, stride, res, plan, lockf, seed):
    r, lock, iv = synth.make_decode_round("decode_tiny", 20 + seed, n_wf=max(8, Q // 4), Q=Q, D=D, T=min(4, D), stride=stride,
                                          n_resident=res, n_planned=plan, lock_fraction=lockf)
    L, O = r.calls["L_in"], r.calls["L_out"]
    rng = np.random.default_rng(seed)
    n_nodes, n_wf = Q + 5, 4
    node = rng.permutation(n_nodes)[:Q].astype(np.int32); wf = rng.integers(0, n_wf, Q).astype(np.int32)
    elapsed = rng.uniform(0, 20, Q).astype(np.float32)
    tail = rng.uniform(0, 5, n_nodes).astype(np.float32); hor = rng.uniform(5, 50, n_wf).astype(np.float32)
    big = widen(iv, D, Q)                    # every call may land on one instance; 64 x 96 entries still fit one workgroup
    got = run_plan(ctx, r.model, L, O, lock, node, wf, elapsed, tail, hor, r.dec, big)
    check_plan_stepwise(r.model, L, O, lock, node, wf, elapsed, tail, hor, r.dec, big, got)
    want = o.decode_plan_greedy(r.model, L, O, lock, elapsed, node, wf, tail, hor, r.dec, big)
    if np.array_equal(got["rank"], want.rank) and np.array_equal(got["best_d"], want.best_d):
        assert_costs_close(got["best_cost"], want.best_cost, "plan cost"); assert_costs_close(got["ratio"], want.ratio, "plan ratio")
        assert np.array_equal(got["count"], want.count)
    assert (got["best_start"][got["best_d"] >= 0] > 0).any()


@pytest.mark.parametrize("Q,D,stride,res,plan", [(40, 4, 16, 10, 3), (80, 64, 16, 10, 3)])      # finish of every pair kept; not kept
def test_decode_greedy_with_workflows_without_horizon(ctx, Q, D, stride, res, plan):
    # a workflow whose horizon is 0 makes its calls infinitely urgent: they are planned first, lowest index first, and
    # placed like any other call; their ratio stays +inf when their best instance moves
    r, lock, iv = synth.make_decode_round("decode_tiny", 31, n_wf=max(8, Q // 4), Q=Q, D=D, T=min(4, D), stride=stride,
                                          n_resident=res, n_planned=plan, lock_fraction=0.2)
    L, O = r.calls["L_in"], r.calls["L_out"]
    rng = np.random.default_rng(7)
    n_nodes, n_wf = Q + 5, 4
    node = rng.permutation(n_nodes)[:Q].astype(np.int32); wf = rng.integers(0, n_wf, Q).astype(np.int32)
    elapsed = rng.uniform(0, 20, Q).astype(np.float32)
    tail = rng.uniform(0, 5, n_nodes).astype(np.float32); hor = rng.uniform(5, 50, n_wf).astype(np.float32)
    hor[1] = 0.0
    big = widen(iv, D, Q)
    got = run_plan(ctx, r.model, L, O, lock, node, wf, elapsed, tail, hor, r.dec, big)
    check_plan_stepwise(r.model, L, O, lock, node, wf, elapsed, tail, hor, r.dec, big, got)
    urgent = np.nonzero(wf == 1)[0]
    assert urgent.size > 2 and np.isinf(got["ratio"][urgent]).all()
    assert np.array_equal(np.sort(got["rank"][urgent]), np.arange(urgent.size))            # before every other call
    assert np.array_equal(np.argsort(got["rank"][urgent]), np.arange(urgent.size))           # in index order
    assert (got["best_d"][urgent] >= 0).any()


@pytest.mark.parametrize("Q,D,stride,res,plan", [(40, 4, 16, 10, 3), (80, 64, 16, 10, 3)])      # finish of every pair kept; not kept
def test_decode_greedy_with_calls_that_decode_nothing(ctx, Q, D, stride, res, plan):
    # a call without output tokens finishes when it starts: its interval holds nothing and the instance's timeline
    # stays as it is (the planner then builds the timeline again instead of inserting the interval)
    r, lock, iv = synth.make_decode_round("decode_tiny", 37, n_wf=max(8, Q // 4), Q=Q, D=D, T=min(4, D), stride=stride,
                                          n_resident=res, n_planned=plan, lock_fraction=0.2)
    L, O = r.calls["L_in"].copy(), r.calls["L_out"].copy()
    O[::3] = 0
    rng = np.random.default_rng(11)
    n_nodes, n_wf = Q + 5, 4
    node = rng.permutation(n_nodes)[:Q].astype(np.int32); wf = rng.integers(0, n_wf, Q).astype(np.int32)
    elapsed = rng.uniform(0, 20, Q).astype(np.float32)
    tail = rng.uniform(0, 5, n_nodes).astype(np.float32); hor = rng.uniform(5, 50, n_wf).astype(np.float32)
    big = widen(iv, D, Q)
    got = run_plan(ctx, r.model, L, O, lock, node, wf, elapsed, tail, hor, r.dec, big)
    check_plan_stepwise(r.model, L, O, lock, node, wf, elapsed, tail, hor, r.dec, big, got)
    placed = got["best_d"] >= 0
    assert (placed & (O == 0)).sum() > 3 and (placed & (O > 0)).sum() > 3
    assert np.array_equal(got["best_start"][placed & (O == 0)], got["best_cost"][placed & (O == 0)])


def test_decode_greedy_at_the_benchmarks_size(ctx):
    # the queue bench.py times: 256 calls x 32 instances, 24 resident + 4 planned entries each, lists of 140 entries
    Q, D = 256, 32
    r, lock, iv = synth.make_decode_round("decode_tiny", 2, n_wf=64, Q=Q, D=D, T=4, stride=28, n_resident=24, n_planned=4)
    L, O = r.calls["L_in"], r.calls["L_out"]
    rng = np.random.default_rng(1)
    node = np.arange(Q, dtype=np.int32); wf = (np.arange(Q) % 8).astype(np.int32)
    tail = rng.uniform(0, 5, Q).astype(np.float32); hor = rng.uniform(10, 60, 8).astype(np.float32)
    elapsed = rng.uniform(0, 30, Q).astype(np.float32)
    big = widen(iv, D, 140 - 28)
    got = run_plan(ctx, r.model, L, O, lock, node, wf, elapsed, tail, hor, r.dec, big)
    check_plan_stepwise(r.model, L, O, lock, node, wf, elapsed, tail, hor, r.dec, big, got)
    assert sorted(got["rank"]) == list(range(Q)) and (got["best_d"] >= 0).mean() > 0.9


def test_decode_greedy_hand_worked_and_limits(ctx):
    from paper_2605_16637_amd import binding
    from helpers import ROUND_MODEL
    dec = dict(flops=np.array([1e13], np.float32), hbm_bw=np.array([1e12], np.float32), used_tok=np.zeros(1, np.int32),
               cap_tok=np.array([1500], np.int32), batch=np.zeros(1, np.int32), qd_tok=np.zeros(1, np.int32), type=np.zeros(1, np.int32))
    iv = dict(stride=4, count=np.zeros(1, np.int32), start=np.zeros(4, np.float32), end=np.zeros(4, np.float32), tok=np.zeros(4, np.int32))
    # two equal calls, room for one at a time (worked by hand in the oracle's pin): the urgent one now, the other after it
    g = run_plan(ctx, ROUND_MODEL, np.array([1000, 1000]), np.array([100, 100]), [-1, 0], [0, 1], [0, 0], [1.0, 5.0], [0.0, 0.0], [10.0], dec, iv)
    assert list(g["rank"]) == [1, 0] and list(g["best_d"]) == [0, 0]
    assert g["best_start"][1] == 0.0 and g["best_cost"][1] == pytest.approx(1.0105, rel=REL)
    assert g["best_start"][0] == g["best_cost"][1] and g["best_cost"][0] == pytest.approx(2.021, rel=REL)
    assert g["ratio"][1] == pytest.approx(0.60105, rel=REL) and g["ratio"][0] == pytest.approx(0.3021, rel=REL)
    assert list(g["count"]) == [2]
    # a call that can never fit is ranked first and changes nothing
    g = run_plan(ctx, ROUND_MODEL, np.array([1000, 2000]), np.array([100, 100]), None, [0, 1], [0, 0], [1.0, 1.0], [0.0, 0.0], [10.0], dec, iv)
    assert list(g["rank"]) == [1, 0] and list(g["best_d"]) == [0, -1] and np.isinf(g["best_cost"][1]) and list(g["count"]) == [1]
    # a full list: reported through the status word
    iv1 = dict(stride=1, count=np.zeros(1, np.int32), start=np.zeros(1, np.float32), end=np.zeros(1, np.float32), tok=np.zeros(1, np.int32))
    with pytest.raises(binding.HxError) as e:
        run_plan(ctx, ROUND_MODEL, np.array([100, 100]), np.array([10, 10]), None, [0, 1], [0, 0], [1.0, 1.0], [0.0, 0.0], [10.0], dec, iv1)
    assert e.value.code == -4
    # too much for one workgroup's local memory
    D = 256
    decb = {k: np.repeat(v, D) for k, v in dec.items()}
    ivb = dict(stride=500, count=np.zeros(D, np.int32), start=np.zeros(D * 500, np.float32), end=np.zeros(D * 500, np.float32),
               tok=np.zeros(D * 500, np.int32))
    with pytest.raises(binding.HxError) as e:
        run_plan(ctx, ROUND_MODEL, np.array([100, 100]), np.array([10, 10]), None, [0, 1], [0, 0], [1.0, 1.0], [0.0, 0.0], [10.0], decb, ivb)
    assert e.value.code == -2


def test_decode_pass_and_ordering_replayed_from_a_hip_graph(ctx):
    """After one eager call has sized the library's scratch, the decode pass and the ordering (both paths: all
    pairs and sample sort) are plain kernel launches: captured in a HIP graph, every replay must equal the eager
    result, with eager work and synchronisation between the replays."""
    import torch
    for name, kw in (("decode_mid", {}), ("decode_mid", dict(Q=20000, n_wf=4000))):
        r, lock, iv = synth.make_decode_round(name, 3, **kw)
        L, O = r.calls["L_in"], r.calls["L_out"]
        Q = len(L)
        q = dev_queue(L, O, r.calls["node"], r.calls["wf"], r.calls["elapsed"])
        dd, div, d_lock = dev_dec(r.dec), dev_iv(iv), dev(lock)
        tail = torch.rand(r.dag.n_nodes, device="cuda:0"); hor = torch.rand(r.dag.n_wf, device="cuda:0") * 20 + 5
        i32 = dict(dtype=torch.int32, device="cuda:0")
        bd, rk = torch.empty(Q, **i32), torch.empty(Q, **i32)
        bs, bc, rt = (torch.empty(Q, device="cuda:0") for _ in range(3))
        outs = (bd, bs, bc, rt, rk)

        def one():
            ctx.hx_decode_score(r.model, q, d_lock, dd, div, bd, bs, bc, tail=tail, horizon=hor, ratio=rt)
            ctx.hx_rank(rt, rk)

        def clear():
            for t in outs:
                t.fill_(-1)

        clear(); one(); torch.cuda.synchronize()
        ctx.hx_stream_status()
        want = [t.cpu().numpy().copy() for t in outs]
        order = np.argsort(-want[3].astype(np.float64), kind="stable")
        assert np.array_equal(want[4][order], np.arange(Q))
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            one()
        for rep in range(3):
            clear(); torch.cuda.synchronize()
            g.replay(); torch.cuda.synchronize()
            for a, b in zip(outs, want):
                assert np.array_equal(a.cpu().numpy(), b), f"replay {rep} differs from the eager call"
            ctx.hx_stream_status()
            one(); torch.cuda.synchronize()            # eager work between replays
