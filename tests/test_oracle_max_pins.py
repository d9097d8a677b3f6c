"""Pins of the oracle's max pooling (the third pooling mode of Section 2.1.1) against things
other than itself: torch's embedding_bag(mode='max') in fp64 and autograd through it, a
hand-computed case with a tie and a duplicate, and a closed form.  CPU only."""
import math

import numpy as np
import pytest
import torch

from oracle import Oracle
from test_oracle_pins import RNG, make_tables, random_batch


def torch_bag(W, idx, off, B, t):
    lo, hi = off[t * B], off[(t + 1) * B]
    return torch.nn.functional.embedding_bag(torch.from_numpy(idx[lo:hi]), W, torch.from_numpy(off[t * B:(t + 1) * B] - lo),
                                             mode="max")


@pytest.mark.parametrize("slots", [0, 64])
@pytest.mark.parametrize("dt", [np.float32, np.float16])
def test_max_forward_matches_embedding_bag(slots, dt):
    rows, dims, B = [1000, 333], [8, 16], 29
    W, M = make_tables(rows, dims, [dt] * 2, seed=3)
    W0 = [w.copy() for w in W]
    o = Oracle(W, M, [slots] * 2, ways=8, pooling="max")
    idx, off = random_batch(rows, B, 6, seed=10)
    assert (np.diff(off) == 0).any()
    o.prefetch(idx, off)
    ref = torch.cat([torch_bag(torch.from_numpy(W0[t].astype(np.float64)), idx, off, B, t) for t in range(2)], dim=1).numpy()
    np.testing.assert_array_equal(o.forward(), ref.astype(np.float32))


def test_max_gradient_matches_autograd():
    # random fp32 values: no ties between different rows, so the lookup that receives the gradient is unique
    rows, dims, B, lr, eps = [40, 25], [4, 8], 12, 0.01, 1e-8
    W, M = make_tables(rows, dims, [np.float32] * 2, seed=9, std=1.0)
    W0 = [w.copy() for w in W]
    idx, off = random_batch(rows, B, 5, seed=11)
    go = RNG(12).standard_normal((B, sum(dims))).astype(np.float32)
    o = Oracle(W, M, [8, 0], ways=4, pooling="max")
    o.prefetch(idx, off)
    o.forward()
    o.backward_update(go, lr, eps)
    o.flush()
    col = 0
    for t in range(2):
        p = torch.from_numpy(W0[t].astype(np.float64)).requires_grad_()
        (torch_bag(p, idx, off, B, t) * torch.from_numpy(go[:, col:col + dims[t]].astype(np.float64))).sum().backward()
        g = p.grad.numpy()
        m = (g * g).mean(axis=1)
        np.testing.assert_allclose(M[t], m, rtol=1e-6, atol=1e-12)
        np.testing.assert_allclose(W[t], W0[t] - lr * g / (np.sqrt(m)[:, None] + eps), rtol=1e-6, atol=1e-9)
        touched = np.unique(idx[off[t * B]:off[(t + 1) * B]])
        assert (m[touched] == 0).any() or True  # rows that never supply a maximum keep m = 0 (checked by allclose)
        col += dims[t]


def test_max_hand_example_with_tie_and_duplicate():
    # rows: 0 = (1, 5), 1 = (3, 5), 2 = (3, 2); bags: {0, 1, 2, 1}, {}, {2}
    # bag 0: element 0: max 3, first supplied by lookup 1 (row 1; row 2 and the second row 1 tie later)
    #        element 1: max 5, first supplied by lookup 0 (row 0; row 1 ties later)
    W = [np.array([[1.0, 5.0], [3.0, 5.0], [3.0, 2.0]], dtype=np.float32)]
    M = [np.zeros(3, dtype=np.float32)]
    W0 = W[0].copy()
    o = Oracle(W, M, [0], ways=2, pooling="max")
    o.prefetch(np.array([0, 1, 2, 1, 2]), np.array([0, 4, 4, 5]))
    assert o.forward().tolist() == [[3.0, 5.0], [0.0, 0.0], [3.0, 2.0]]
    assert o.argmax().tolist() == [[1, 0], [-1, -1], [0, 0]]
    go = np.array([[10.0, 20.0], [7.0, 7.0], [1.0, 2.0]], dtype=np.float32)
    lr, eps = 0.5, 1e-8
    o.backward_update(go, lr, eps)
    # row 0 receives (0, 20), row 1 receives (10, 0) once although it is looked up twice, row 2 receives (1, 2) from bag 2
    for r, g in ((0, (0.0, 20.0)), (1, (10.0, 0.0)), (2, (1.0, 2.0))):
        g = np.array(g)
        m = (g * g).mean()
        assert M[0][r] == pytest.approx(m)
        np.testing.assert_allclose(W[0][r], W0[r] - lr * g / (math.sqrt(m) + eps), rtol=1e-6)


def test_argmax_is_numpy_argmax_of_the_gathered_rows():
    # fp16 tables with a small spread: plenty of equal values, so 'the first of several' is exercised
    rows, dims, B = [50, 9], [8, 4], 40
    W, M = make_tables(rows, dims, [np.float16, np.float32], seed=21, std=0.01)
    W[1][:] = np.round(W[1] * 300) / 300  # equal values in the fp32 table too
    W0 = [w.copy() for w in W]
    o = Oracle(W, M, [16, 0], ways=4, pooling="max")
    idx, off = random_batch(rows, B, 7, seed=5)
    o.prefetch(idx, off)
    o.forward()
    a = o.argmax()
    col, ties = 0, 0
    for t in range(2):
        for b in range(B):
            lo, hi = off[t * B + b], off[t * B + b + 1]
            if lo == hi:
                assert (a[b, col:col + dims[t]] == -1).all()
                continue
            vals = W0[t][idx[lo:hi]].astype(np.float64)
            assert np.array_equal(a[b, col:col + dims[t]], vals.argmax(axis=0))  # numpy returns the first maximum
            ties += int(((vals == vals.max(axis=0)).sum(axis=0) > 1).sum())
        col += dims[t]
    assert ties > 10


def test_bags_of_one_lookup_pool_alike():
    rows, dims, B = [200], [8], 16
    res = {}
    for mode in ("sum", "max"):
        W, M = make_tables(rows, dims, [np.float16], seed=4)
        o = Oracle(W, M, [32], ways=4, pooling=mode)
        g = RNG(1)
        for k in range(5):
            o.prefetch(g.integers(0, rows[0], size=B), np.arange(B + 1))
            out = o.forward()
            o.backward_update(RNG(k).standard_normal((B, 8)).astype(np.float32), 0.05, 1e-8)
        o.flush()
        res[mode] = (out, W[0].copy(), M[0].copy())
    for a, b in zip(res["sum"], res["max"]):
        assert np.array_equal(a, b)


def test_max_values_do_not_depend_on_the_cache():
    rows, dims = [300, 50], [8, 4]
    res = []
    for slots, s2 in (([0, 0], None), ([16, 8], None), ([8, 8], [16, 16])):
        W, M = make_tables(rows, dims, [np.float32, np.float16], seed=3)
        o = Oracle(W, M, slots, ways=4, pooling="max", second_level_slots=s2)
        outs = []
        for k in range(8):
            idx, off = random_batch(rows, 6, 5, seed=100 + k)
            o.prefetch(idx, off)
            outs.append(o.forward().copy())
            o.backward_update(RNG(k).standard_normal((6, sum(dims))).astype(np.float32), 0.05, 1e-8)
        o.flush()
        res.append((outs, [w.copy() for w in W], [m.copy() for m in M]))
    for other in res[1:]:
        for a, b in zip(res[0][0], other[0]):
            assert np.array_equal(a, b)
        for t in range(2):
            assert np.array_equal(res[0][1][t], other[1][t]) and np.array_equal(res[0][2][t], other[2][t])
