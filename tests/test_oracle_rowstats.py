"""Pins for the oracle's row statistics (paper Eq. 1 and Eq. 5)."""
import math

import numpy as np
import pytest
import scipy.special
import scipy.stats

from oracle import fly_oracle as O


def test_uniform_row_has_unit_entropy():
    for V in (2, 16, 8192, 128256):
        st = O.row_statistics(np.full(V, 3.25))
        assert abs(st["H"] - math.log(V)) < 1e-9
        assert abs(st["h"] - 1.0) < 1e-12
        assert abs(st["p_top1"] - 1.0 / V) < 1e-15
        assert st["argmax"] == 0            # every entry ties: lowest index
        assert st["margin"] == 0.0


def test_one_hot_row_has_zero_entropy():
    l = np.zeros(8192)
    l[4711] = 1e4
    st = O.row_statistics(l)
    assert st["argmax"] == 4711
    assert st["h"] == 0.0 and st["H"] == 0.0
    assert st["p_top1"] == 1.0
    assert st["margin"] == 1e4


def test_two_token_row_is_binary_entropy():
    for a, b in ((0.3, -1.2), (2.0, 2.5), (-4.0, 4.0)):
        st = O.row_statistics(np.array([a, b]))
        p = 1.0 / (1.0 + math.exp(b - a))      # sigmoid(a - b)
        Hb = -(p * math.log(p) + (1 - p) * math.log(1 - p))
        assert abs(st["H"] - Hb) < 1e-12
        assert abs(st["h"] - Hb / math.log(2)) < 1e-12
        assert abs(st["p_top1"] - max(p, 1 - p)) < 1e-12
        assert st["argmax"] == (0 if a >= b else 1)


def test_shift_invariance_and_zero_scale():
    rng = np.random.default_rng(0)
    l = rng.normal(size=1000) * 3
    a, b = O.row_statistics(l), O.row_statistics(l + 123.456)
    assert a["argmax"] == b["argmax"]
    assert abs(a["H"] - b["H"]) < 1e-9 and abs(a["p_top1"] - b["p_top1"]) < 1e-12
    assert abs((b["lse"] - a["lse"]) - 123.456) < 1e-9
    z = O.row_statistics(l * 0.0)
    assert abs(z["h"] - 1.0) < 1e-12


def test_against_scipy_and_bruteforce():
    rng = np.random.default_rng(1)
    for V in (3, 7, 16, 513):
        for scale in (0.1, 1.0, 8.0):
            l = rng.normal(size=V) * scale
            st = O.row_statistics(l)
            assert abs(st["lse"] - scipy.special.logsumexp(l)) < 1e-10
            p = scipy.special.softmax(l)
            assert abs(st["H"] - scipy.stats.entropy(p)) < 1e-10
            assert abs(st["h"] - scipy.stats.entropy(p, base=V)) < 1e-10
            assert abs(st["p_top1"] - p.max()) < 1e-12
            # pure-python literal of Eq. 5
            Z = sum(math.exp(x) for x in l)
            H = -sum((math.exp(x) / Z) * math.log(math.exp(x) / Z) for x in l)
            assert abs(st["H"] - H) < 1e-10
            srt = sorted(l)
            assert abs(st["margin"] - (srt[-1] - srt[-2])) < 1e-15
            assert 0.0 <= st["h"] <= 1.0


@pytest.mark.parametrize("idx", [0, 15, 16, 255, 256, 8191])
def test_planted_argmax_and_ties(idx):
    l = np.linspace(-1, 1, 8192)
    l[idx] = 5.0
    assert O.row_statistics(l)["argmax"] == idx
    # an exact tie later in the row does not move the argmax
    if idx < 8191:
        l[8191] = 5.0
        st = O.row_statistics(l)
        assert st["argmax"] == idx and st["margin"] == 0.0


def test_minus_infinity_entries_contribute_nothing():
    l = np.array([0.0, -np.inf, 0.0, -np.inf])
    st = O.row_statistics(l)
    assert abs(st["H"] - math.log(2)) < 1e-12
    assert abs(st["h"] - 0.5) < 1e-12       # V counts all four columns


def test_block_and_decision_statistics():
    import torch
    rng = np.random.default_rng(2)
    L = rng.normal(size=(5, 64))
    blk = O.block_statistics(L)
    for i in range(5):
        r = O.row_statistics(L[i])
        assert blk["argmax"][i] == r["argmax"] and blk["h"][i] == r["h"]
    # decision in float32: two logits that differ only beyond float32 tie there,
    # and the lowest index wins
    L[0, 10] = 9.0
    L[0, 3] = 9.0 + 1e-12
    L[0, 3], L[0, 10] = L[0, 10], L[0, 3]   # larger value now at the higher index
    dec = O.decision_statistics(torch.from_numpy(L))
    assert O.row_statistics(L[0])["argmax"] == 10
    assert dec["argmax"][0] == 3
