"""Pins for the oracle's acceptance rule (paper Sec. 2.2, Eqs. 2-11, Alg. 1).

The rule has no printed worked example (the overview figure is an image), so
it is pinned by what the text fixes: the limit statements of the ablation
section, the boundary rule, hand-worked cases, structural invariants of the
equations, and exhaustive agreement of three independently written forms.
"""
import itertools
import random

import numpy as np
import pytest

from oracle import fly_oracle as O


def run_all_forms(delta, h, theta, W):
    """Evaluate the three forms; assert they agree; return s."""
    K = len(delta)
    target = list(range(100, 100 + K + 1))
    draft = [target[i] if delta[i] else 7 for i in range(K)]
    s_gate, s_defer, s_eq = O.accept_equations(delta, h, theta, W)
    s_alg, emitted = O.accept_algorithm(draft, target, h, theta, W)
    s_pred = O.accept_predicate(delta, h, theta, W)
    assert s_eq == s_alg == s_pred, (delta, h, theta, W, s_eq, s_alg, s_pred)
    # Emitted tokens: kept drafts (mismatching ones stay the draft's token),
    # then the target's token at s (Alg. 1, both reject branches and accept-all).
    assert len(emitted) == s_alg
    assert emitted[:-1] == draft[: s_alg - 1]
    assert emitted[-1] == target[s_alg - 1]
    # Strict at j forces DeferDecide(j) = Reject (first conjunct of Eq. 9).
    assert s_defer <= s_gate
    return s_eq


HI, LO = 0.9, 0.1  # entropies above / below theta = 0.3


def test_match_indicator_and_standard():
    assert O.match_indicator([5, 6, 7], [5, 9, 7, 1]) == [1, 0, 1]
    assert O.s_standard([1, 1, 1]) == 4      # all match -> K+1 (Eq. 3)
    assert O.s_standard([1, 0, 1]) == 2      # first mismatch index
    assert O.s_standard([0, 0, 0]) == 1


def test_hand_cases_paper_defaults():
    K, W, th = 15, 6, 0.3  # the paper's 70B setting
    ones = [1] * K

    # no mismatch: everything plus the bonus token
    assert run_all_forms(ones, [HI] * K, th, W) == K + 1

    # single high-entropy mismatch at j with a clean window: kept iff j + W <= K
    for j in range(1, K + 1):
        d = ones.copy(); d[j - 1] = 0
        expect = K + 1 if j + W <= K else j
        assert run_all_forms(d, [HI] * K, th, W) == expect, j

    # the same mismatch at low entropy is always rejected at j
    for j in range(1, K + 1):
        d = ones.copy(); d[j - 1] = 0
        h = [HI] * K; h[j - 1] = LO
        assert run_all_forms(d, h, th, W) == j

    # second mismatch on the last slot of the window (j + W): reject at j
    d = ones.copy(); d[1] = 0; d[1 + W] = 0        # j = 2, j + W = 8
    assert run_all_forms(d, [HI] * K, th, W) == 2
    # second mismatch one past the window (j + W + 1 = 9): first one is kept and
    # the outcome depends on the second alone (9 + 6 = 15 <= 15 -> kept too)
    d = ones.copy(); d[1] = 0; d[2 + W] = 0
    assert run_all_forms(d, [HI] * K, th, W) == K + 1
    # ... unless the second is low-entropy
    h = [HI] * K; h[2 + W] = LO
    assert run_all_forms(d, h, th, W) == 9
    # mismatch right after j (i = j + 1) also counts
    d = ones.copy(); d[1] = 0; d[2] = 0
    assert run_all_forms(d, [HI] * K, th, W) == 2


def test_gate_equality_defers():
    # h == theta is Defer, not Strict (Eq. 6 uses h < theta for Strict)
    K, W = 8, 2
    d = [1] * K; d[0] = 0
    assert run_all_forms(d, [0.3] * K, 0.3, W) == K + 1
    assert run_all_forms(d, [0.29999] * K, 0.3, W) == 1


def test_boundary_rule():
    # j + W > K rejects even a high-entropy mismatch with nothing after it
    K, W = 8, 6
    for j in range(1, K + 1):
        d = [1] * K; d[j - 1] = 0
        s = run_all_forms(d, [HI] * K, 0.3, W)
        assert s == (K + 1 if j <= K - W else j)
    # K = 4 with W = 6 can never defer: FLy equals exact-match decoding
    for bits in itertools.product([0, 1], repeat=4):
        assert run_all_forms(list(bits), [HI] * 4, 0.3, 6) == O.s_standard(bits)


@pytest.mark.parametrize("K", [1, 2, 3, 5, 7])
def test_limits_exhaustive(K):
    """theta above every entropy -> exact-match decoding; theta=0 and W=0 ->
    everything accepted; W >= K -> exact-match decoding (ablation section and
    the boundary rule)."""
    for bits in itertools.product([0, 1], repeat=K):
        delta = list(bits)
        for gates in itertools.product([LO, HI], repeat=K):
            h = list(gates)
            std = O.s_standard(delta)
            for W in range(0, K + 2):
                s = run_all_forms(delta, h, 0.3, W)
                assert s >= std
                assert run_all_forms(delta, h, 2.0, W) == std     # gate rejects all
                if W >= K:
                    assert s == std                                # window never fits
            assert run_all_forms(delta, h, 0.0, 0) == K + 1       # defer all, accept all
            # W = 0 with the gate on: only strict mismatches reject
            strict = [j for j in range(1, K + 1) if delta[j - 1] == 0 and h[j - 1] < 0.3]
            assert run_all_forms(delta, h, 0.3, 0) == (min(strict) if strict else K + 1)


def test_theta_one_is_standard_when_h_below_one():
    # "theta = 1 rejects all mismatches": true whenever h < 1
    rng = random.Random(0)
    for _ in range(300):
        K = rng.randint(1, 20)
        delta = [rng.random() < 0.7 for _ in range(K)]
        delta = [int(x) for x in delta]
        h = [rng.random() * 0.999 for _ in range(K)]
        assert run_all_forms(delta, h, 1.0, rng.randint(0, 8)) == O.s_standard(delta)


def test_monotone_in_theta_and_window():
    rng = random.Random(1)
    for _ in range(400):
        K = rng.randint(1, 24)
        delta = [int(rng.random() < 0.75) for _ in range(K)]
        h = [rng.random() for _ in range(K)]
        thetas = [0.0, 0.2, 0.3, 0.5, 0.8, 1.1]
        for W in (0, 1, 3, 6):
            vals = [run_all_forms(delta, h, t, W) for t in thetas]
            assert all(a >= b for a, b in zip(vals, vals[1:])), (delta, h, W, vals)
        for t in (0.0, 0.3, 0.7):
            vals = [run_all_forms(delta, h, t, W) for W in range(0, K + 2)]
            assert all(a >= b for a, b in zip(vals, vals[1:])), (delta, h, t, vals)


def _brute_force_s(delta, gate_defer, W):
    """Independent restatement used only here: simulate 'provisional accept,
    watch the next W tokens, retroactively reject' token by token."""
    K = len(delta)
    for j in range(1, K + 1):
        if delta[j - 1]:
            continue
        if not gate_defer[j - 1]:
            return j
        # watch the following W draft positions; all must exist and all must match
        ok = True
        for step in range(1, W + 1):
            pos = j + step
            if pos > K or not delta[pos - 1]:
                ok = False
                break
        if not ok:
            return j
    return K + 1


@pytest.mark.parametrize("K", [1, 2, 4, 6, 8])
def test_exhaustive_against_simulation(K):
    Ws = range(0, K + 2) if K <= 6 else (0, 1, 2, 3, 6, 8)
    for bits in itertools.product([0, 1], repeat=K):
        delta = list(bits)
        for gates in itertools.product([0, 1], repeat=K):
            # gate bits at matching positions are irrelevant: skip duplicates
            if any(g and d for g, d in zip(gates, delta)):
                continue
            h = [HI if g else LO for g in gates]
            for W in Ws:
                assert run_all_forms(delta, h, 0.3, W) == _brute_force_s(delta, gates, W)


def test_two_accepted_mismatches():
    # K = 15, W = 6: mismatches at 1 and 8 are both kept (8 + 6 <= 15)
    K, W = 15, 6
    d = [1] * K; d[0] = 0; d[7] = 0
    assert run_all_forms(d, [HI] * K, 0.3, W) == K + 1
    blk = O.accept_block(np.array([[7 if not x else 100 + i for i, x in enumerate(d)]]),
                         np.array([list(range(100, 100 + K + 1))]),
                         np.full((1, K + 1), HI), 0.3, W)
    assert blk["accept_len"][0] == K and blk["n_loose"][0] == 2
    assert blk["next_token"][0] == 100 + K and blk["s"][0] == K + 1


def test_accept_block_convention():
    # reject at j=3: two drafts kept, correction token is the target's y_3
    draft = np.array([[10, 11, 99, 13]])
    target = np.array([[10, 11, 12, 13, 14]])
    h = np.array([[HI, HI, LO, HI, HI]])
    out = O.accept_block(draft, target, h, 0.3, 1)
    assert out["s"][0] == 3 and out["accept_len"][0] == 2
    assert out["next_token"][0] == 12 and out["n_loose"][0] == 0
    # float32 comparison at the gate: h is compared after rounding to float32
    h = np.array([[HI, HI, np.float64(np.float32(0.3)), HI, HI]])
    out = O.accept_block(draft, target, h, 0.3, 1)
    assert out["s"][0] == 5 and out["n_loose"][0] == 1


def test_expected_standard_length_of_workload():
    """With the gate shut, drafts that match independently with probability p
    give E[s] = (1 - p^(K+1)) / (1 - p)."""
    rng = np.random.default_rng(3)
    for p, K, expect in ((0.6, 4, 2.3056), (0.7, 8, 3.1988), (0.75, 16, 3.9699)):
        closed = (1 - p ** (K + 1)) / (1 - p)
        assert abs(closed - expect) < 1e-3
        n = 20000
        delta = (rng.random((n, K)) < p).astype(int)
        s = np.array([O.accept_predicate(list(r), [0.0] * K, 2.0, 6) for r in delta])
        assert abs(s.mean() - closed) < 0.05
