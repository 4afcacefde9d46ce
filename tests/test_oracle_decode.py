"""Pins for the oracle's prompt-lookup drafter and decode loop (no GPU).

The drafter's rule is this build's reading of Sec. 2.3 (the paper gives no
parameters), so it is pinned against an independently written search and
against what the rule must do on periodic sequences.  The loop (Algorithm 1
with the cache rolled forward) is pinned by the property of greedy speculative
decoding that a strict verifier reproduces the target's own greedy output
whatever the drafter proposes, and by recomputing the cache from scratch.
"""
import numpy as np
import pytest
import torch

import synth
from oracle import fly_oracle as O
from tests.helpers import oracle_model


def brute_force_pld(y, n_max, K):
    """Score every end position by the length of the common suffix with the
    whole sequence (capped), take the best score, latest position."""
    L = len(y)
    best = (0, -1)
    for e in range(1, L):
        n = 0
        while n < min(n_max, e) and y[e - 1 - n] == y[L - 1 - n]:
            n += 1
        if n > 0 and (n, e) > best:
            best = (n, e)
    n, e = best
    if n == 0:
        return [y[-1]] * K, 0
    out = []
    for i in range(K):
        src = e + i
        out.append(y[src] if src < L else out[src - L])
    return out, n


def test_pld_matches_independent_search():
    rng = np.random.default_rng(5)
    for _ in range(3000):
        L = int(rng.integers(1, 40))
        y = rng.integers(0, int(rng.integers(2, 6)), size=L).tolist()
        n_max, K = int(rng.integers(1, 6)), int(rng.integers(1, 9))
        assert O.pld_propose(y, n_max, K) == brute_force_pld(y, n_max, K), (y, n_max, K)


@pytest.mark.parametrize("period,n_max", [(1, 1), (2, 3), (3, 3), (5, 2), (7, 4)])
def test_pld_continues_a_periodic_sequence(period, n_max):
    base = list(range(100, 100 + period))          # distinct tokens: one occurrence per period
    for L in range(period + 1, 4 * period + 3):
        y = [base[i % period] for i in range(L)]
        drafts, n = O.pld_propose(y, n_max, 9)
        assert drafts == [base[(L + i) % period] for i in range(9)]
        assert n == min(n_max, L - period) if period > 1 else n == min(n_max, L - 1)


def test_pld_edge_cases():
    assert O.pld_propose([4], 3, 5) == ([4] * 5, 0)                      # nothing earlier
    assert O.pld_propose([1, 2, 3, 4], 3, 3) == ([4, 4, 4], 0)           # no token repeats
    assert O.pld_propose([7, 7], 2, 4) == ([7, 7, 7, 7], 1)              # copy runs into itself
    # the longer n-gram wins over a later but shorter match
    y = [1, 2, 3, 9, 3, 8, 1, 2, 3]
    assert O.pld_propose(y, 3, 2) == ([9, 3], 3)
    assert O.pld_propose(y, 1, 2) == ([8, 1], 1)                         # latest occurrence of "3"
    # among equal lengths the latest occurrence
    assert O.pld_propose([5, 6, 1, 5, 6, 2, 5, 6], 2, 1) == ([2], 2)


CFG = synth.CONFIGS["c1_tiny"]


def model_args(cfg):
    return dict(n_q_heads=cfg.n_q_heads, n_kv_heads=cfg.n_kv_heads, head_dim=cfg.head_dim,
                rope_theta=cfg.rope_theta, eps=cfg.rms_eps, storage=cfg.dtype)


def greedy_continuation(model, cfg, y0, kv0, steps):
    """The target's own greedy decoding, one token per forward pass."""
    y = list(y0)
    kv = [(k.clone(), v.clone()) for k, v in kv0]
    for _ in range(steps):
        out = O.verify_block(np.asarray([[y[-1], 0]]), model["embed"], model["layers"], model["g_final"],
                             model["w_lm"], [(k[None], v[None]) for k, v in kv], None, theta=0.3, W=0,
                             **model_args(cfg))
        y.append(int(out["argmax"][0, 0]))
        kv = [(torch.cat([k, nk[:1]]), torch.cat([v, nv[:1]])) for (k, v), (nk, nv) in zip(kv, out["new_kv"][0])]
    return y


@pytest.fixture(scope="module")
def tiny():
    cfg = CFG.replace(kv_len=24)
    model = oracle_model(cfg)
    kv0 = [(k[0], v[0]) for k, v in model["kv_prefix"]]
    y0 = synth.hash_tokens(11, 77, 9, cfg.vocab).tolist()
    return cfg, model, kv0, y0


def scripted_drafter(reference, wrong_every):
    """Proposes the reference continuation with every `wrong_every`-th position
    (counted over the whole sequence) replaced by another token."""
    def drafter(y, K):
        out = []
        for i in range(K):
            pos = len(y) + i
            tok = reference[pos] if pos < len(reference) else 0
            if pos % wrong_every == 0:
                tok = (tok + 1) % 8192
            out.append(tok)
        return out, -1
    return drafter


def test_strict_loop_reproduces_greedy_decoding(tiny):
    cfg, model, kv0, y0 = tiny
    K, rounds = 4, 4
    ref = greedy_continuation(model, cfg, y0, kv0, rounds * (K + 1))
    res = O.decode_rounds(y0, kv0, model["embed"], model["layers"], model["g_final"], model["w_lm"], None,
                          rounds=rounds, K=K, n_max=3, theta=2.0, W=6, drafter=scripted_drafter(ref, 4),
                          **model_args(cfg))
    assert res["y"] == ref[:len(res["y"])]
    assert len(res["y"]) == len(y0) + sum(res["s"])
    assert max(res["s"]) > 1 and min(res["s"]) < K + 1          # both kept drafts and rejections occurred
    assert res["n_loose"] == [0] * rounds
    assert res["tau"] == sum(res["s"]) / rounds
    # prompt lookup as the drafter: same property
    res2 = O.decode_rounds(y0, kv0, model["embed"], model["layers"], model["g_final"], model["w_lm"], None,
                           rounds=rounds, K=K, n_max=3, theta=2.0, W=6, **model_args(cfg))
    assert res2["y"] == ref[:len(res2["y"])]


def test_loose_loop_bookkeeping_and_cache(tiny):
    cfg, model, kv0, y0 = tiny
    K, rounds = 6, 3
    ref = greedy_continuation(model, cfg, y0, kv0, rounds * (K + 1))
    # theta = 0: every mismatch is deferred; W = 1: kept when the next draft matches
    res = O.decode_rounds(y0, kv0, model["embed"], model["layers"], model["g_final"], model["w_lm"], None,
                          rounds=rounds, K=K, n_max=3, theta=0.0, W=1, drafter=scripted_drafter(ref, 5),
                          **model_args(cfg))
    y = res["y"]
    assert len(y) == len(y0) + sum(res["s"])
    assert sum(res["n_loose"]) > 0 and y != ref[:len(y)]        # a differing draft was kept
    for (k, v), (k0, _) in zip(res["kv"], kv0):
        assert k.shape[0] == v.shape[0] == k0.shape[0] + sum(res["s"]) == k0.shape[0] + len(y) - len(y0)
    # the cache equals the one a single pass over the kept tokens builds
    block = np.asarray([y[len(y0) - 1:]])
    once = O.verify_block(block, model["embed"], model["layers"], model["g_final"], model["w_lm"],
                          [(k[None], v[None]) for k, v in kv0], None, theta=0.3, W=0, **model_args(cfg))
    n_new = len(y) - len(y0)
    for (k, v), (k0, _), (nk, nv) in zip(res["kv"], kv0, once["new_kv"][0]):
        L0 = k0.shape[0]
        assert torch.allclose(k[L0:], nk[:n_new], rtol=0, atol=1e-6)
        assert torch.allclose(v[L0:], nv[:n_new], rtol=0, atol=1e-6)


# ---------------------------------------------------------------------------
# Drafting with a model (Algorithm 1 step 1 with a draft model M_D)
# ---------------------------------------------------------------------------
DRAFTER = synth.CONFIGS["c1_tiny"].replace(name="tiny_drafter", n_layers=1, d=128, n_q_heads=2, n_kv_heads=1,
                                           ffn=256, seed=77, logit_gain=20.0)


def incremental_greedy(model, cfg, y, K, first_pos):
    """The same K tokens by carrying the cache: one token per pass through
    decoder_layer, appending its k, v rows (an independent route: causality
    makes it equal to the full passes)."""
    num = O.Numerics(cfg.dtype)
    kv = [(k[0, :first_pos].clone(), v[0, :first_pos].clone()) for k, v in model["kv_prefix"]]
    logits = None
    toks = [int(t) for t in y[first_pos:]]
    out = []
    feed = list(toks)
    while len(out) < K:
        for t in feed:
            x = model["embed"][torch.tensor([t])].clone()
            for li, w in enumerate(model["layers"]):
                x, k_new, v_new = O.decoder_layer(x, w, kv[li][0], kv[li][1], cfg.n_q_heads, cfg.n_kv_heads,
                                                  cfg.head_dim, cfg.rope_theta, cfg.rms_eps, num)
                kv[li] = (torch.cat([kv[li][0], k_new]), torch.cat([kv[li][1], v_new]))
            xn = num.act(O.rmsnorm(x, model["g_final"], cfg.rms_eps))
            logits = O.lm_head_logits(xn, model["w_lm"], None)
        nxt = int(O.decision_statistics(logits)["argmax"][0])
        out.append(nxt)
        feed = [nxt]
    return out


def test_loop_with_drawn_tokens(tiny):
    """The loop at temperature > 0 (the drawn token takes the argmax's place, a reading of ours):
    every round is the verification step with that round's draw on the state the rounds before
    left; at a temperature near zero it is the greedy loop; and with the gate always strict every
    emitted token is one the target drew."""
    cfg, model, kv0, y0 = tiny
    K, rounds = 4, 4
    args = (model["embed"], model["layers"], model["g_final"], model["w_lm"])
    hot = torch.full((K + 1,), 40.0)            # a gain on the tiny model's logits: a usable entropy range
    res = O.decode_rounds(y0, kv0, *args, hot, rounds=rounds, K=K, n_max=3, theta=2.0, W=0,
                          sample=(11, 100), sample_row0=2 * (K + 1), **model_args(cfg))
    y, kv = list(y0), [(k.clone(), v.clone()) for k, v in kv0]
    drew_other = 0
    for r in range(rounds):
        drafts = res["rounds"][r]["drafts"]
        out = O.verify_block(np.asarray([[y[-1]] + drafts]), *args, [(k[None], v[None]) for k, v in kv], hot,
                             theta=2.0, W=0, sample=(11, 100 + r), sample_row0=2 * (K + 1), **model_args(cfg))
        assert np.array_equal(out["sampled"][0], res["rounds"][r]["sampled"])
        s = int(out["accept_len"][0]) + 1
        assert s == res["s"][r]
        emitted = drafts[:s - 1] + [int(out["next_token"][0])]
        assert emitted == [int(t) for t in out["sampled"][0][:s]]     # strict: only drawn tokens are emitted
        drew_other += int((out["sampled"][0] != out["argmax"][0]).sum())
        y += emitted
        kv = [(torch.cat([k, nk[:s]]), torch.cat([v, nv[:s]])) for (k, v), (nk, nv) in zip(kv, out["new_kv"][0])]
    assert y == res["y"] and drew_other > 0
    other = O.decode_rounds(y0, kv0, *args, hot, rounds=rounds, K=K, n_max=3, theta=2.0, W=0,
                            sample=(11, 101), sample_row0=2 * (K + 1), **model_args(cfg))
    assert other["y"] != res["y"]                                       # the offset selects the draw
    cold = torch.full((K + 1,), 1e6)
    greedy = O.decode_rounds(y0, kv0, *args, cold, rounds=rounds, K=K, n_max=3, theta=0.3, W=1, **model_args(cfg))
    drawn = O.decode_rounds(y0, kv0, *args, cold, rounds=rounds, K=K, n_max=3, theta=0.3, W=1,
                            sample=(11, 100), **model_args(cfg))
    assert drawn["y"] == greedy["y"] and drawn["s"] == greedy["s"]


def test_model_drafter_equals_incremental_decoding():
    cfg = DRAFTER.replace(batch=1, kv_len=12)
    model = oracle_model(cfg)
    rng = np.random.default_rng(3)
    for first_pos, n_after in ((11, 2), (12, 1), (9, 4)):
        y = rng.integers(0, cfg.vocab, size=first_pos + n_after).tolist()
        prefix = [(k[0], v[0]) for k, v in model["kv_prefix"]]
        got = O.model_draft_greedy(y, 5, model["embed"], model["layers"], model["g_final"], model["w_lm"], prefix,
                                   first_pos, n_q_heads=cfg.n_q_heads, n_kv_heads=cfg.n_kv_heads,
                                   head_dim=cfg.head_dim, rope_theta=cfg.rope_theta, eps=cfg.rms_eps,
                                   storage=cfg.dtype)
        assert got == incremental_greedy(model, cfg, y, 5, first_pos), (first_pos, n_after)


def test_model_drafted_strict_loop_is_lossless():
    """Whatever model drafts, a strict verifier (theta above every entropy) emits
    the target's own greedy continuation (the lossless limit the paper starts from)."""
    tcfg = synth.CONFIGS["c1_tiny"].replace(batch=1, kv_len=10, logit_gain=12.0)
    dcfg = DRAFTER.replace(batch=1, kv_len=10, vocab=tcfg.vocab)
    tm, dm = oracle_model(tcfg), oracle_model(dcfg)
    y0 = np.random.default_rng(9).integers(0, tcfg.vocab, size=11).tolist()
    dprefix = [(k[0], v[0]) for k, v in dm["kv_prefix"]]

    def drafter(y, K):
        return O.model_draft_greedy(y, K, dm["embed"], dm["layers"], dm["g_final"], dm["w_lm"], dprefix,
                                    dcfg.kv_len - 1, n_q_heads=dcfg.n_q_heads, n_kv_heads=dcfg.n_kv_heads,
                                    head_dim=dcfg.head_dim, rope_theta=dcfg.rope_theta, eps=dcfg.rms_eps,
                                    storage=dcfg.dtype), 0

    common = dict(n_q_heads=tcfg.n_q_heads, n_kv_heads=tcfg.n_kv_heads, head_dim=tcfg.head_dim,
                  rope_theta=tcfg.rope_theta, eps=tcfg.rms_eps, storage=tcfg.dtype)
    kv0 = [(k[0], v[0]) for k, v in tm["kv_prefix"]]
    strict = O.decode_rounds(y0, kv0, tm["embed"], tm["layers"], tm["g_final"], tm["w_lm"], None, rounds=3, K=4,
                             n_max=3, theta=2.0, W=0, drafter=drafter, **common)
    # the target's own greedy decoding: K = 1 rounds whose single draft is always wrong or right -- s tokens kept
    # either way are the target's argmax chain
    plain = O.decode_rounds(y0, kv0, tm["embed"], tm["layers"], tm["g_final"], tm["w_lm"], None,
                            rounds=len(strict["y"]) - len(y0), K=1, n_max=1, theta=2.0, W=0, **common)
    assert strict["y"] == plain["y"][:len(strict["y"])]
    assert all(1 <= s <= 5 for s in strict["s"])
