"""Pins of the oracle's mean pooling (the second pooling mode of Section 2.1.1) against
things other than itself: torch's embedding_bag(mode='mean') in fp64, autograd for the
gradient each row receives, a closed form and a hand-computed case.  CPU only."""
import math

import numpy as np
import pytest
import torch

from oracle import Oracle
from test_oracle_pins import RNG, make_tables, random_batch


def torch_mean_forward(W, idx, off, B):
    outs = []
    for t in range(len(W)):
        lo, hi = off[t * B], off[(t + 1) * B]
        outs.append(torch.nn.functional.embedding_bag(torch.from_numpy(idx[lo:hi]), torch.from_numpy(W[t].astype(np.float64)),
                                                      torch.from_numpy(off[t * B:(t + 1) * B] - lo), mode="mean"))
    return torch.cat(outs, dim=1).numpy()


@pytest.mark.parametrize("slots", [0, 64])
@pytest.mark.parametrize("dt", [np.float32, np.float16])
def test_mean_forward_matches_embedding_bag(slots, dt):
    rows, dims = [1000, 333], [8, 16]
    W, M = make_tables(rows, dims, [dt] * 2, seed=3)
    W0 = [w.copy() for w in W]
    o = Oracle(W, M, [slots] * 2, ways=8, pooling="mean")
    B = 29
    idx, off = random_batch(rows, B, 6, seed=10)
    assert (np.diff(off) == 0).any()  # empty bags are part of the case
    o.prefetch(idx, off)
    np.testing.assert_array_equal(o.forward(), torch_mean_forward(W0, idx, off, B).astype(np.float32))


def test_mean_hand_example():
    # one table, 3 rows, dim 2; bags {0,2,2}, {}, {1}
    W = [np.array([[1.0, 2.0], [10.0, 20.0], [100.0, 200.0]], dtype=np.float32)]
    M = [np.zeros(3, dtype=np.float32)]
    o = Oracle(W, M, [2], ways=2, pooling="mean")
    o.prefetch(np.array([0, 2, 2, 1]), np.array([0, 3, 3, 4]))
    assert o.forward().tolist() == [[67.0, 134.0], [0.0, 0.0], [10.0, 20.0]]


def test_mean_gradient_matches_autograd():
    rows, dims, B, lr, eps = [40, 25], [4, 8], 12, 0.01, 1e-8
    W, M = make_tables(rows, dims, [np.float32] * 2, seed=9, std=1.0)
    W0 = [w.copy() for w in W]
    idx, off = random_batch(rows, B, 5, seed=11)
    go = RNG(12).standard_normal((B, sum(dims))).astype(np.float32)
    o = Oracle(W, M, [8, 0], ways=4, pooling="mean")
    o.prefetch(idx, off)
    o.forward()
    o.backward_update(go, lr, eps)
    o.flush()
    col = 0
    for t in range(2):
        p = torch.from_numpy(W0[t].astype(np.float64)).requires_grad_()
        lo, hi = off[t * B], off[(t + 1) * B]
        out = torch.nn.functional.embedding_bag(torch.from_numpy(idx[lo:hi]), p,
                                                torch.from_numpy(off[t * B:(t + 1) * B] - lo), mode="mean")
        (out * torch.from_numpy(go[:, col:col + dims[t]].astype(np.float64))).sum().backward()
        g = p.grad.numpy()
        m = (g * g).mean(axis=1)
        np.testing.assert_allclose(M[t], m, rtol=1e-6, atol=1e-12)
        np.testing.assert_allclose(W[t], W0[t] - lr * g / (np.sqrt(m)[:, None] + eps), rtol=1e-6, atol=1e-9)
        col += dims[t]


def test_mean_first_update_closed_form():
    # bag 0 = {3, 3, 5} (3 lookups), bag 1 = {3}: row 3 receives 2/3 go[0] + go[1], row 5 receives 1/3 go[0]
    D, lr, eps = 8, 0.1, 1e-2
    W, M = make_tables([10], [D], [np.float32], seed=7, std=1.0)
    W0 = W[0].copy()
    o = Oracle(W, M, [0], ways=4, pooling="mean")
    go = RNG(8).standard_normal((2, D)).astype(np.float32)
    o.prefetch(np.array([3, 3, 5, 3]), np.array([0, 3, 4]))
    o.forward()
    o.backward_update(go, lr, eps)
    for r, g in ((3, 2.0 / 3.0 * go[0].astype(np.float64) + go[1]), (5, go[0].astype(np.float64) / 3.0)):
        np.testing.assert_allclose(W[0][r], W0[r] - lr * g / (np.linalg.norm(g) / math.sqrt(D) + eps), rtol=1e-6)
        np.testing.assert_allclose(M[0][r], (g * g).mean(), rtol=1e-6)


def test_bags_of_one_lookup_pool_alike():
    # with one lookup per bag mean and sum are the same operator
    rows, dims, B = [200], [8], 16
    res = {}
    for mode in ("sum", "mean"):
        W, M = make_tables(rows, dims, [np.float16], seed=4)
        o = Oracle(W, M, [32], ways=4, pooling=mode)
        g = RNG(1)
        for k in range(5):
            idx = g.integers(0, rows[0], size=B)
            o.prefetch(idx, np.arange(B + 1))
            out = o.forward()
            o.backward_update(RNG(k).standard_normal((B, 8)).astype(np.float32), 0.05, 1e-8)
        o.flush()
        res[mode] = (out, W[0].copy(), M[0].copy())
    for a, b in zip(res["sum"], res["mean"]):
        assert np.array_equal(a, b)


def test_pooling_is_fixed_before_the_first_batch():
    from oracle import lib
    W, M = make_tables([10], [4], [np.float32])
    o = Oracle(W, M, [4], ways=2)
    assert lib().orc_set_pooling(o.h, 3) != 0
    o.prefetch(np.array([1]), np.array([0, 1]))
    assert lib().orc_set_pooling(o.h, 1) != 0
