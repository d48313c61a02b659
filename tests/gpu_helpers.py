"""Helpers of the GPU parity tests: move a synthetic round to the device, call
the library through its binding, and compare with the oracle."""
import numpy as np

from oracle import hx_oracle as o

REL = 1e-5     # fp32 costs against the fp64 oracle


def dev(x):
    import torch
    if x is None:
        return None
    return torch.from_numpy(np.ascontiguousarray(x)).to("cuda:0")


def dev_tables(rnd):
    from paper_2605_16637_amd import binding
    calls = binding.to_device(rnd.calls)
    pre = binding.to_device(rnd.pre)
    dec = binding.to_device(rnd.dec)
    links = binding.to_device(rnd.links)
    return calls, pre, dec, links


def fused(ctx, model, calls, pre, dec, links, tail=None, horizon=None, want_ratio=False):
    import torch
    n = int(calls["n"])
    bp = torch.full((n,), -7, dtype=torch.int32, device="cuda:0")
    bd = torch.full((n,), -7, dtype=torch.int32, device="cuda:0")
    bc = torch.full((n,), -7.0, dtype=torch.float32, device="cuda:0")
    ratio = torch.full((n,), -7.0, dtype=torch.float32, device="cuda:0") if want_ratio else None
    ctx.hx_score_placements(model, calls, pre, dec, links, tail=tail, horizon=horizon,
                            best_p=bp, best_d=bd, best_cost=bc, ratio=ratio)
    ctx.hx_stream_status()
    out = [bp.cpu().numpy(), bd.cpu().numpy(), bc.cpu().numpy()]
    if want_ratio:
        out.append(ratio.cpu().numpy())
    return out


def assert_costs_close(gpu, ref, what="cost"):
    gpu = np.asarray(gpu, np.float64)
    ref = np.asarray(ref, np.float64)
    assert gpu.shape == ref.shape
    assert np.array_equal(np.isinf(gpu), np.isinf(ref)), f"{what}: infeasible pattern differs"
    assert not np.isnan(gpu).any(), f"{what}: NaN"
    fin = np.isfinite(ref)
    err = np.abs(gpu[fin] - ref[fin]) / np.maximum(np.abs(ref[fin]), 1e-30)
    assert err.size == 0 or err.max() <= REL, f"{what}: max relative error {err.max():.3e}"
    return float(err.max()) if err.size else 0.0


def assert_search_matches(rnd_model, L_in, L_out, pre, dec, links, ores, gp, gd, gc, rows=None):
    """Selected indices equal the oracle's, except where the oracle's cost of
    the GPU's pair is within REL of the oracle's best (a near-tie in fp32);
    best costs within REL; 'no feasible pair' agrees exactly.  `rows` maps the
    compared entries to call indices when only a sample is checked."""
    rows = np.arange(len(gp)) if rows is None else rows
    assert_costs_close(gc, ores.best_cost, "best_cost")
    none_o = ores.best_p < 0
    assert np.array_equal(gp < 0, none_o) and np.array_equal(gd < 0, none_o)
    diff = np.nonzero((gp != ores.best_p) | (gd != ores.best_d))[0]
    for i in diff:
        c = rows[i]
        alt = o.score_one(rnd_model, L_in[c], L_out[c], gp[i], gd[i], pre, dec, links)
        assert np.isfinite(alt) and alt <= ores.best_cost[i] * (1 + REL), \
            f"call {c}: GPU chose ({gp[i]},{gd[i]}) cost {alt}, oracle ({ores.best_p[i]},{ores.best_d[i]}) cost {ores.best_cost[i]}"
    return len(diff)
