"""hx_commit_static, the commit for callers that cannot allocate, against hx_commit
through the C ABI: integer state bit for bit, on two calls in a row (the second
on a smaller round and a smaller pool, so whatever the first left in the
library's static array would show), status word included.  In a fresh process
the first call below is also the first use of the library on the device (no
context exists yet), which exercises the on-demand look-up of the array."""
import numpy as np
import pytest

from paper_2605_16637_amd import synth

pytestmark = pytest.mark.gpu


def _round(rng, C, P, D):
    L, O = synth.gen_lengths(rng, C)
    bp = rng.integers(-1, P, C).astype(np.int32)
    bd = np.where(bp < 0, -1, rng.integers(0, D, C)).astype(np.int32)
    st = [rng.integers(0, 20000, P).astype(np.int32), rng.integers(0, 300000, D).astype(np.int32),
          rng.integers(0, 200, D).astype(np.int32), rng.integers(0, 20000, D).astype(np.int32)]
    dr = [rng.integers(0, 80 * max(C, 1), P).astype(np.int32), rng.integers(0, 6 * max(C, 1), D).astype(np.int32),
          rng.integers(0, 40 * max(C, 1), D).astype(np.int32)]
    return L, O, bp, bd, st, dr


def test_commit_static_equals_commit_on_two_calls_in_a_row():
    import torch
    from paper_2605_16637_amd import binding
    dev = lambda x: torch.from_numpy(np.ascontiguousarray(x)).to("cuda:0")
    rng = np.random.default_rng(16)
    cases = [_round(rng, 40000, 700, 1024), _round(rng, 3000, 37, 53), _round(rng, 0, 5, 3)]
    # static entry point first: three calls in a row on one stream, shrinking inputs
    status = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    got = []
    for L, O, bp, bd, st, dr in cases:
        g = [dev(x.copy()) for x in st]
        calls = binding.to_device(dict(n=len(L), L_in=L, L_out=O))
        binding.hx_commit_static(calls, dev(bp), dev(bd), g[0], g[1], g[2], g[3], dev(dr[0]), dev(dr[1]), dev(dr[2]),
                                 status=status)
        got.append(g)
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    ctx = binding.Context(0)
    for (L, O, bp, bd, st, dr), g in zip(cases, got):
        w = [dev(x.copy()) for x in st]
        calls = binding.to_device(dict(n=len(L), L_in=L, L_out=O))
        ctx.hx_commit(calls, dev(bp), dev(bd), w[0], w[1], w[2], w[3], dev(dr[0]), dev(dr[1]), dev(dr[2]))
        ctx.hx_stream_status()
        for a, b in zip(g, w):
            assert torch.equal(a, b)
    # conditions only the GPU sees land in the caller's status word, and nowhere when there is none
    big = binding.to_device(dict(n=2, L_in=np.array([2**30, 2**30], np.int32), L_out=np.array([16, 16], np.int32)))
    g = [dev(np.zeros(1, np.int32)) for _ in range(4)]
    binding.hx_commit_static(big, dev(np.zeros(2, np.int32)), dev(np.zeros(2, np.int32)), *g, status=status)
    torch.cuda.synchronize()
    assert int(status.item()) == -7 and int(g[0].item()) == 2**31 - 1
    status.zero_()
    binding.hx_commit_static(big, dev(np.array([3, 0], np.int32)), dev(np.zeros(2, np.int32)), *g, status=status)
    torch.cuda.synchronize()
    assert int(status.item()) == -6
    binding.hx_commit_static(big, dev(np.array([3, 0], np.int32)), dev(np.zeros(2, np.int32)), *g, status=None)
    # a round after the faulty ones is unaffected
    L, O, bp, bd, st, dr = cases[1]
    g = [dev(x.copy()) for x in st]
    calls = binding.to_device(dict(n=len(L), L_in=L, L_out=O))
    binding.hx_commit_static(calls, dev(bp), dev(bd), g[0], g[1], g[2], g[3], dev(dr[0]), dev(dr[1]), dev(dr[2]))
    torch.cuda.synchronize()
    for a, b in zip(g, got[1]):
        assert torch.equal(a, b)
    ctx.close()


def test_commit_static_rejects_what_its_scratch_cannot_hold():
    import torch
    from paper_2605_16637_amd import binding
    dev = lambda x: torch.from_numpy(np.ascontiguousarray(x)).to("cuda:0")
    z = lambda n: dev(np.zeros(n, np.int32))
    calls = binding.to_device(dict(n=1, L_in=np.ones(1, np.int32), L_out=np.ones(1, np.int32)))
    with pytest.raises(binding.HxError) as e:
        binding.hx_commit_static(calls, z(1), z(1), z(1025), z(4), z(4), z(4))
    assert e.value.code == -2 and "1024" in str(e.value)
    with pytest.raises(binding.HxError) as e:
        binding.hx_commit_static(calls, z(1), z(1), z(4), z(1025), z(1025), z(1025))
    assert e.value.code == -2
