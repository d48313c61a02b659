"""The seeded input generators (host logic): same seed -> same round, and the rounds have the structure the
workloads are meant to have (ids parent-first and workflow-contiguous, depth and fan-out caps, about one
(call, decode instance) pair in ten infeasible on the near-capacity pools, well-formed interval lists)."""
import numpy as np
import pytest

from paper_2605_16637_amd import synth


def same(a, b):
    if isinstance(a, dict):
        return a.keys() == b.keys() and all(same(a[k], b[k]) for k in a)
    if isinstance(a, np.ndarray):
        return a.dtype == b.dtype and np.array_equal(a, b)
    return a == b


@pytest.mark.parametrize("name", ["tiny", "mid"])
def test_rounds_are_reproducible(name):
    a, b, c = synth.make_round(name, 3), synth.make_round(name, 3), synth.make_round(name, 4)
    for x in ("calls", "pre", "dec", "links", "types"):
        assert same(getattr(a, x), getattr(b, x))
    assert np.array_equal(a.dag.succ_col, b.dag.succ_col) and np.array_equal(a.dag.L_in, b.dag.L_in)
    assert not np.array_equal(a.calls["L_in"], c.calls["L_in"])


@pytest.mark.parametrize("name,depth_cap,fan_cap", [("tiny", 5, 3), ("mid", 12, 4)])
def test_dag_structure(name, depth_cap, fan_cap):
    d = synth.make_round(name, 1).dag
    n = d.n_nodes
    assert d.wf_ptr[0] == 0 and d.wf_ptr[-1] == n and (np.diff(d.wf_ptr) > 0).all()
    assert np.array_equal(d.wf_of_node, np.repeat(np.arange(d.n_wf), np.diff(d.wf_ptr)))
    src = np.repeat(np.arange(n), np.diff(d.succ_row_ptr))
    assert (d.succ_col > src).all()                                   # parent-first numbering
    assert np.array_equal(d.wf_of_node[src], d.wf_of_node[d.succ_col])  # edges stay inside a workflow
    assert np.diff(d.succ_row_ptr).max() <= fan_cap
    child = np.repeat(np.arange(n), np.diff(d.parent_row_ptr))
    assert sorted(zip(d.parent_col.tolist(), child.tolist())) == sorted(zip(src.tolist(), d.succ_col.tolist()))
    depth = np.zeros(n, np.int64)
    for v in range(n):                                                # ids are topological
        ps = d.parent_col[d.parent_row_ptr[v]:d.parent_row_ptr[v + 1]]
        if ps.size:
            depth[v] = depth[ps].max() + 1
    assert depth.max() < depth_cap
    assert d.L_in.min() >= 64 and d.L_in.max() <= 32768 and d.L_out.min() >= 16 and d.L_out.max() <= 4096


def test_near_capacity_pool_and_calls():
    r = synth.make_round("large", 1)
    need = r.calls["L_in"].astype(np.int64) + r.calls["L_out"]
    free = r.dec["cap_tok"].astype(np.int64) - r.dec["used_tok"]
    assert 0.09 < (need[:, None] > free[None, :]).mean() < 0.11     # free = a U(0.8, 1) quantile of demand: 0.10 expected
    assert (r.dec["used_tok"] >= 0).all() and (r.dec["used_tok"] <= r.dec["cap_tok"]).all()
    assert np.array_equal(r.pre["type"], np.arange(r.pre["n"]) % 8)
    for t in range(8):
        assert np.unique(r.pre["flops"][r.pre["type"] == t]).size == 1
    out_deg = np.diff(r.dag.succ_row_ptr)[r.calls["node"]]
    assert 0.6 < (out_deg == 0).mean() < 0.9                          # mostly leaves of the revealed graph
    assert np.array_equal(r.calls["wf"], r.dag.wf_of_node[r.calls["node"]])
    assert np.array_equal(r.links["bw"], r.links["bw"].T)             # slower NIC of the two classes


def test_stream_batches():
    g = synth.StreamGen(5, 200, final_lo=6, final_hi=12)
    seen = 0
    sizes = {}
    for _ in range(12):
        b = g.next_batch()
        n = b["n_new"]
        assert np.array_equal(b["ids"], np.arange(seen, seen + n))
        rp, col = b["parent_row_ptr"], b["parent_col"]
        assert rp[0] == 0 and rp[-1] == col.size and (np.diff(rp) >= 0).all() and np.diff(rp).max() <= 2
        child = np.repeat(b["ids"], np.diff(rp))
        assert (col < child).all() and (col >= 0).all()
        for w in b["wf"]:
            sizes[int(w)] = sizes.get(int(w), 0) + 1
        seen += n
    assert max(sizes.values()) <= 12 and b["n_wf_total"] == max(sizes) + 1


def test_decode_round_intervals():
    r, lock, iv = synth.make_decode_round("decode_mid", 2)
    D, K = r.dec["n"], iv["stride"]
    cnt = iv["count"]
    assert cnt.shape == (D,) and (cnt >= 1).all() and (cnt <= K).all()
    st, en, tk = (iv[k].reshape(D, K) for k in ("start", "end", "tok"))
    live = np.arange(K)[None, :] < cnt[:, None]
    assert (en[live] > st[live]).all() and (tk[live] >= 0).all()
    occ0 = np.where(live & (st <= 0) & (en > 0), tk, 0).sum(axis=1)
    assert (occ0 <= r.dec["cap_tok"]).all() and (occ0 > 0.5 * r.dec["cap_tok"]).all()       # near capacity now
    assert (st[live] > 0).any()                                        # some planned entries start later
    assert ((lock >= -1) & (lock < D)).all() and 0.3 < (lock >= 0).mean() < 0.7
    a = synth.make_decode_round("decode_mid", 2)
    assert np.array_equal(a[1], lock) and same(a[2], iv)
