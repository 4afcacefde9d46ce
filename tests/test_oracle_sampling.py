"""Pins for the oracle's draw of the target's token at temperature > 0 (no GPU).

The paper states its rule with the argmax (Eqs. 1-2) and reports temperature-1
results without giving the rule; drawing y_i from softmax(l_i / T) and using
it in Eq. 2 is this build's reading.  What is pinned here is the draw itself:
the counter-based generator against its published known-answer vectors, the
uniform mapping against its range, the Gumbel-max construction against the
softmax probabilities it must reproduce (chi-square over many draws) and the
limits in which the draw is certain.
"""
import os

import numpy as np
import pytest
from scipy import stats

import synth
from oracle import fly_oracle as O
from tests.helpers import draft_chain, oracle_model, oracle_verify

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def test_philox_known_answers():
    rows = [l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        w = [int(x, 16) for x in r]
        out = O.philox4x32_10(np.array([w[0:4]], dtype=np.uint32), (w[4], w[5]))
        assert [int(x) for x in out[0]] == w[6:10]


def test_philox_is_a_bijection_of_the_counter_on_a_sample():
    # distinct counters, same key -> distinct blocks (the round function is invertible)
    ctr = np.zeros((4096, 4), dtype=np.uint32)
    ctr[:, 0] = np.arange(4096)
    out = O.philox4x32_10(ctr, (5, 6))
    assert len({tuple(int(x) for x in r) for r in out}) == 4096


def test_sample_bits_layout():
    # word v % 4 of block (v // 4, m, offset lo, offset hi) under key (seed lo, seed hi)
    seed, offset = (0x11223344 << 32) | 0x55667788, (0x0A0B0C0D << 32) | 0x01020304
    bits = O.sample_bits(3, 10, seed, offset)
    for m in range(3):
        for v in range(10):
            blk = O.philox4x32_10(np.array([[v // 4, m, 0x01020304, 0x0A0B0C0D]], dtype=np.uint32),
                                  (0x55667788, 0x11223344))
            assert int(bits[m, v]) == int(blk[0, v % 4])


def test_a_subset_of_rows_draws_what_the_whole_call_draws():
    rng = np.random.default_rng(5)
    logits = rng.normal(size=(40, 64))
    whole = O.sample_rows(logits, 21, 8)
    rows = [3, 17, 39]
    part = O.sample_rows(logits[rows], 21, 8, rows=rows)
    assert np.array_equal(part["token"], whole["token"][rows])
    assert np.allclose(part["margin"], whole["margin"][rows])


def test_uniform_is_strictly_inside_the_unit_interval_and_exact_in_float32():
    edge = np.array([0, 1, 511, 512, 2**32 - 1, 2**31], dtype=np.uint32)
    u = O.uniform_open01(edge)
    assert u.min() == 2.0 ** -24 and u.max() == 1.0 - 2.0 ** -24
    assert np.array_equal(u.astype(np.float32).astype(np.float64), u)
    bits = O.sample_bits(64, 4096, 7, 1)
    u = O.uniform_open01(bits)
    assert stats.kstest(u.ravel(), "uniform").pvalue > 1e-3


def test_gumbel_moments():
    g = O.gumbel_noise(O.sample_bits(128, 8192, 3, 9))
    assert abs(g.mean() - np.euler_gamma) < 5e-3
    assert abs(g.var() - np.pi ** 2 / 6) < 2e-2
    assert stats.kstest(g.ravel()[:200000], "gumbel_r").pvalue > 1e-3


@pytest.mark.parametrize("seed,offset", [(1, 0), (2 ** 40 + 17, 2 ** 33 + 5)])
def test_draws_follow_the_softmax(seed, offset):
    rng = np.random.default_rng(11)
    V, N = 12, 60000
    logits = rng.normal(size=V) * 1.5
    logits[3] = -np.inf                      # a token of probability zero is never drawn
    p = np.exp(logits - logits.max())
    p /= p.sum()
    drawn = O.sample_rows(np.tile(logits, (N, 1)), seed, offset)["token"]
    counts = np.bincount(drawn, minlength=V)
    assert counts[3] == 0
    keep = p > 0
    assert stats.chisquare(counts[keep], p[keep] * N).pvalue > 1e-3


def test_a_planted_mistake_in_the_noise_fails_the_chi_square():
    # exponential instead of Gumbel noise: the draws no longer follow the softmax
    rng = np.random.default_rng(12)
    V, N = 12, 60000
    logits = rng.normal(size=V) * 1.5
    p = np.exp(logits - logits.max())
    p /= p.sum()
    u = O.uniform_open01(O.sample_bits(N, V, 1, 0))
    wrong = np.argmax(logits[None, :] - np.log(u), axis=1)
    assert stats.chisquare(np.bincount(wrong, minlength=V), p * N).pvalue < 1e-6


def test_offsets_and_rows_give_independent_draws():
    logits = np.zeros((2000, 16))
    a = O.sample_rows(logits, 5, 0)["token"]
    b = O.sample_rows(logits, 5, 1)["token"]
    again = O.sample_rows(logits, 5, 0)["token"]
    assert np.array_equal(a, again)
    assert 0.02 < np.mean(a == b) < 0.12          # 1/16 by chance
    assert 0.02 < np.mean(a[1:] == a[:-1]) < 0.12
    table = np.zeros((16, 16))
    np.add.at(table, (a, b), 1)
    assert stats.chi2_contingency(table).pvalue > 1e-3


def test_certain_limits():
    rng = np.random.default_rng(13)
    logits = rng.normal(size=(50, 300))
    cold = O.sample_rows(logits * 1e4, 9, 2)    # temperature -> 0: the argmax
    assert np.array_equal(cold["token"], np.argmax(logits, axis=1))
    one_hot = np.full((5, 40), -np.inf)
    one_hot[np.arange(5), [0, 7, 39, 20, 1]] = 0.0
    assert list(O.sample_rows(one_hot, 9, 2)["token"]) == [0, 7, 39, 20, 1]
    # the margin is that of the perturbed logits
    l = np.zeros((1, 4))
    r = O.sample_rows(l, 1, 1)
    z = np.sort(O.gumbel_noise(O.sample_bits(1, 4, 1, 1))[0])
    assert abs(r["margin"][0] - (z[-1] - z[-2])) < 1e-6


def test_verify_block_with_drawn_tokens_applies_the_rule_to_them():
    cfg = synth.CONFIGS["c1_tiny"]
    model = oracle_model(cfg)
    tokens = draft_chain(cfg, model)
    B, R = tokens.shape
    K = R - 1
    out = oracle_verify(cfg, model, tokens, W=1, return_logits=True, sample=(77, 3))
    again = O.sample_rows(out["logits"].reshape(B * R, -1), 77, 3)["token"].reshape(B, R)
    assert np.array_equal(out["sampled"], again)
    acc = O.accept_block(tokens[:, 1:], out["sampled"], out["h"], cfg.theta, 1)
    assert np.array_equal(acc["accept_len"], out["accept_len"])
    assert np.array_equal(acc["next_token"], out["next_token"])
    # strict verification keeps the drafts up to the first one that differs from the drawn token
    strict = oracle_verify(cfg, model, tokens, theta=2.0, W=0, sample=(77, 3))
    for b in range(B):
        diff = np.append(tokens[b, 1:] != strict["sampled"][b, :K], True)
        assert strict["accept_len"][b] == int(np.argmax(diff))
        assert strict["next_token"][b] == strict["sampled"][b, strict["accept_len"][b]]
