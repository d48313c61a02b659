"""Pins of the oracle's commit-and-drain step (the simulated-state update of
Algorithm 1, applied once per round).  The paper gives no numbers for it; these are
hand-worked integers and order-independence.  No GPU."""
import numpy as np

from oracle import hx_oracle as o


def test_hand_worked_commit():
    L = [100, 200, 300, 400]
    O = [10, 20, 30, 40]
    bp = [0, 1, -1, 0]
    bd = [1, 1, -1, 0]
    # prefill 0 gets 100 + 400, prefill 1 gets 200; the unplaced call adds nothing
    # decode 0: qd += 40, used += 440; decode 1: qd += 30, used += 110 + 220
    bl, us, ba, qd, rc = o.commit(L, O, bp, bd, [1000, 50], [5000, 4000], [3, 2], [7, 9],
                                  drain_prefill=[600, 1000], drain_decode_q=[10, 100], release_tok=[1000, 280],
                                  tokens_per_seq=2048, max_batch=256)
    assert rc == 0
    assert list(bl) == [1000 + 500 - 600, 0]                 # 50 + 200 - 1000 clamps at 0
    assert list(qd) == [7 + 40 - 10, 0]                      # 9 + 30 - 100 clamps at 0
    assert list(us) == [5000 + 440 - 1000, 4000 + 330 - 280]
    assert list(ba) == [3, 2]                                # ceil(4440/2048) = 3, ceil(4050/2048) = 2
    # batch clips at max_batch and is 0 for an empty instance
    *_, ba, _, rc = o.commit([], [], [], [], [0], [10**6, 0], [0, 0], [0, 0], [0], [0, 0], [0, 0], 2048, 256)
    assert list(ba) == [256, 0]


def test_commit_is_order_independent():
    rng = np.random.default_rng(41)
    C, P, D = 500, 5, 7
    L = rng.integers(64, 32768, C); O = rng.integers(16, 4096, C)
    bp = rng.integers(-1, P, C); bd = np.where(bp < 0, -1, rng.integers(0, D, C))
    args = ([100] * P, [1000] * D, [1] * D, [50] * D, [3000] * P, [700] * D, [9000] * D)
    a = o.commit(L, O, bp, bd, *args)
    perm = rng.permutation(C)
    b = o.commit(L[perm], O[perm], bp[perm], bd[perm], *args)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)
    # totals: every placed call is counted exactly once
    bl0 = np.array([100] * P) + np.bincount(bp[bp >= 0], weights=L[bp >= 0], minlength=P).astype(np.int64)
    assert np.array_equal(a[0], np.maximum(bl0 - 3000, 0))


def test_commit_overflow_is_an_error():
    *_, rc = o.commit([2**30, 2**30], [16, 16], [0, 0], [0, 0], [0], [0], [0], [0], [0], [0], [0])
    assert rc == -4
