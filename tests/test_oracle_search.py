"""Pins of the oracle's enumeration and selection (Sec. 5.3: the pair with the
earliest projected decode finish; Sec. 5.4: infeasible pairs are never legal;
ties go to the lowest flat index p*D + d).  No GPU."""
import numpy as np

from oracle import hx_oracle as o
from paper_2605_16637_amd import synth
from helpers import random_pool


def test_argmin_is_first_minimum_of_the_tensor():
    # the search result equals numpy's first-occurrence argmin over the
    # enumerated tensor, on pools of up to 4 x 4
    rng = np.random.default_rng(21)
    M = synth.MODEL
    for trial in range(30):
        P, D, T = int(rng.integers(1, 5)), int(rng.integers(1, 5)), int(rng.integers(1, 4))
        types, pre, dec, links = random_pool(rng, P, D, T)
        L, O = synth.gen_lengths(rng, 17)
        r = o.score(M, L, O, pre, dec, links, want_cost=True, want_feas=True)
        flat = r.cost.reshape(len(L), -1)
        for c in range(len(L)):
            if np.isinf(flat[c]).all():
                assert (r.best_p[c], r.best_d[c]) == (-1, -1) and np.isinf(r.best_cost[c])
                continue
            i = int(np.argmin(flat[c]))
            assert (r.best_p[c], r.best_d[c]) == (i // D, i % D)
            assert r.best_cost[c] == flat[c, i]
            others = np.delete(flat[c], i)
            assert r.second[c] == (others.min() if others.size else np.inf)
        # hxo_select on the tensor agrees with the fused enumeration
        bp, bd, bc = o.select(r.cost)
        assert np.array_equal(bp, r.best_p) and np.array_equal(bd, r.best_d) and np.array_equal(bc, r.best_cost)


def test_infeasible_pairs_are_never_chosen():
    rng = np.random.default_rng(22)
    rnd = synth.make_round("tiny", seed=3, near_capacity=True)
    r = o.score(rnd.model, rnd.calls["L_in"], rnd.calls["L_out"], rnd.pre, rnd.dec, rnd.links,
                want_cost=True, want_feas=True)
    need = rnd.calls["L_in"].astype(np.int64) + rnd.calls["L_out"]
    free = rnd.dec["cap_tok"].astype(np.int64) - rnd.dec["used_tok"]
    want = (need[:, None] <= free[None, :])
    assert np.array_equal(r.feas.astype(bool), want)
    assert 0.02 < 1.0 - want.mean() < 0.4          # the mask is exercised
    # the mask and the +inf entries of the tensor are the same thing
    assert np.array_equal(np.isinf(r.cost), np.broadcast_to(~want[:, None, :], r.cost.shape))
    ok = r.best_d >= 0
    assert want[np.nonzero(ok)[0], r.best_d[ok]].all()
    assert (~want[~ok]).all()


def test_ties_go_to_lowest_flat_index():
    # homogeneous idle pool: every pair has the same cost
    M = synth.MODEL
    P, D = 3, 4
    pre = dict(flops=[4e14] * P, hbm_bw=[2e12] * P, backlog_tok=[0] * P, type=[0] * P)
    dec = dict(flops=[4e14] * D, hbm_bw=[2e12] * D, used_tok=[0] * D, cap_tok=[10**6] * D,
               batch=[0] * D, qd_tok=[0] * D, type=[0] * D)
    links = dict(n_types=1, bw=np.array([[2.5e10]], np.float32), latency=None)
    r = o.score(M, [64, 1500, 32768], [16, 300, 4096], pre, dec, links, want_cost=True)
    assert (r.cost == r.cost[:, :1, :1]).all()
    assert (r.best_p == 0).all() and (r.best_d == 0).all()
    assert np.array_equal(r.second, r.best_cost)
    # make (0,0) infeasible-free but slower: the next flat index wins
    pre["backlog_tok"] = [5000, 0, 0]
    r = o.score(M, [1500], [300], pre, dec, links)
    assert (r.best_p[0], r.best_d[0]) == (1, 0)
    dec["used_tok"] = [999000, 0, 0, 0]
    r = o.score(M, [1500], [300], pre, dec, links)
    assert (r.best_p[0], r.best_d[0]) == (1, 1)


def test_single_decode_or_single_prefill_reduces_to_1d():
    # a call locked to one decode instance (Sec. 5.4) searches prefill only
    rng = np.random.default_rng(23)
    M = synth.MODEL
    types, pre, dec, links = random_pool(rng, 4, 4, 2)
    dec["cap_tok"] = np.full(4, 10**6, np.int32)
    L, O = synth.gen_lengths(rng, 25)
    full = o.score(M, L, O, pre, dec, links, want_cost=True)
    for d in range(4):
        one = {k: np.asarray(v)[d:d + 1] for k, v in dec.items()}
        r = o.score(M, L, O, pre, one, links, want_cost=True)
        assert np.array_equal(r.cost[:, :, 0], full.cost[:, :, d])
        assert np.array_equal(r.best_p, full.cost[:, :, d].argmin(axis=1))
    for p in range(4):
        one = {k: np.asarray(v)[p:p + 1] for k, v in pre.items()}
        r = o.score(M, L, O, one, dec, links, want_cost=True)
        assert np.array_equal(r.cost[:, 0, :], full.cost[:, p, :])
        assert np.array_equal(r.best_d, full.cost[:, p, :].argmin(axis=1))


def test_threads_do_not_change_results():
    rnd = synth.make_round("tiny", seed=2)
    a = o.score(rnd.model, rnd.calls["L_in"], rnd.calls["L_out"], rnd.pre, rnd.dec, rnd.links, nthreads=1)
    b = o.score(rnd.model, rnd.calls["L_in"], rnd.calls["L_out"], rnd.pre, rnd.dec, rnd.links, nthreads=4)
    assert np.array_equal(a.best_p, b.best_p) and np.array_equal(a.best_cost, b.best_cost)


def test_bad_type_index_is_rejected():
    import pytest
    rnd = synth.make_round("tiny", seed=2)
    bad = dict(rnd.pre, type=np.array([0, 1, 2, 0], np.int32))
    with pytest.raises(ValueError):
        o.score(rnd.model, rnd.calls["L_in"], rnd.calls["L_out"], bad, rnd.dec, rnd.links)
