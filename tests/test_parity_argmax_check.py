"""The check that the GPU parity tests apply to 'who supplied each maximum' (parity_util.compare_argmax),
exercised on the CPU with choices planted by hand: the oracle's own choice passes with no flips, a row
whose value lies within the bar of the maximum is accepted and counted, a clearly smaller row, a
position outside the bag, the later of two lookups of one row and a pooled value that is not the chosen
row's are all refused."""
import numpy as np
import pytest

from oracle import Oracle
from paper_2305_01515_amd import synth
from parity_util import compare_argmax


def setup():
    # one fp16 table, dim 8; bag 0 = rows (0, 1, 2, 1), bag 1 empty, bag 2 = row 2
    W = [np.zeros((4, 8), dtype=np.float16)]
    W[0][0] = 0.5
    W[0][1] = 0.5 + 2 ** -11  # one fp16 ulp above row 0: inside the bar of 2e-3
    W[0][2] = 0.25
    M = [np.zeros(4, dtype=np.float32)]
    tab = synth.TableCfg(4, 8, synth.FP16, None, "fixed", 1, cache_slots=0)
    cfg = synth.WorkloadCfg("hand", [tab], batch=3, ways=2, steps=1, seed=1, init_std=0.05, lr=0.05)
    o = Oracle(W, M, [0], ways=2, pooling="max")
    idx, off = np.array([0, 1, 2, 1, 2]), np.array([0, 4, 4, 5])
    o.prefetch(idx, off)
    out = o.forward()
    return cfg, o, idx, off, out


def test_own_choice_has_no_flips():
    cfg, o, idx, off, out = setup()
    a = o.argmax()
    assert a[0].tolist() == [1] * 8 and a[1].tolist() == [-1] * 8
    assert compare_argmax(cfg, o, idx, off, a.copy(), out.copy(), "hand") == 0


def test_near_tie_is_accepted_and_counted():
    cfg, o, idx, off, out = setup()
    a, g = o.argmax().copy(), out.copy()
    a[0, 3] = 0  # row 0 instead of row 1: one ulp below
    g[0, 3] = 0.5
    assert compare_argmax(cfg, o, idx, off, a, g, "hand") == 1
    assert g[0, 3] == out[0, 3]  # the checked element is patched for the comparison of the pooled output


@pytest.mark.parametrize("pos,value,what", [(2, 0.25, "larger by more than the bar"), (3, 0.5 + 2 ** -11, "looked up twice"),
                                            (4, 0.5, "not in the bag"), (0, 0.47, "not that of the row")])
def test_wrong_choices_are_refused(pos, value, what):
    cfg, o, idx, off, out = setup()
    a, g = o.argmax().copy(), out.copy()
    a[0, 5], g[0, 5] = pos, value
    with pytest.raises(AssertionError, match=what):
        compare_argmax(cfg, o, idx, off, a, g, "hand")
