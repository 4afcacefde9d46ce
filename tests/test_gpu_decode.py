"""HIP path vs oracle: prompt-lookup drafting (bit-exact) and the multi-round
decode loop of Algorithm 1 with the cache rolled forward, through the C ABI."""
import numpy as np
import pytest
import torch

import synth
from oracle import fly_oracle as O
from tests.gpu_harness import GpuWorkload
from tests.helpers import oracle_model

pytestmark = pytest.mark.gpu

C1 = synth.CONFIGS["c1_tiny"]
B16_SMALL = synth.CONFIGS["c2_8b"].replace(
    name="bf16_small", n_layers=2, d=256, n_q_heads=4, n_kv_heads=2, ffn=512, vocab=2048,
    batch=2, K=4, kv_len=150, weight_std=0.05)


def test_pld_draft_bit_exact():
    from paper_2511_22972_amd import binding as fb
    rng = np.random.default_rng(3)
    cap = 700
    rows = []
    for b in range(96):
        L = int(rng.integers(1, cap + 1))
        alphabet = int(rng.choice([2, 3, 5, 50, 8192]))
        rows.append(rng.integers(0, alphabet, size=L).tolist())
    rows.append([9])                                                  # nothing earlier
    rows.append([1, 2, 3, 4])                                         # no repeat
    rows.append([7, 7])                                               # copy runs into itself
    rows.append([5 + (i % 3) for i in range(cap)])                    # periodic, full row
    rows.append(list(range(300)) + list(range(17)))                   # long-ago occurrence
    B = len(rows)
    ctx = torch.zeros(B, cap, dtype=torch.int32)
    for b, r in enumerate(rows):
        ctx[b, :len(r)] = torch.tensor(r, dtype=torch.int32)
    ctx_len = torch.tensor([len(r) for r in rows], dtype=torch.int32)
    ctx_d, len_d = ctx.cuda(), ctx_len.cuda()
    for K, n_max in ((1, 1), (4, 3), (8, 2), (16, 5), (63, 64)):
        tokens = torch.full((B, K + 1), -1, dtype=torch.int32, device="cuda")
        ngram = torch.full((B,), -1, dtype=torch.int32, device="cuda")
        fb.fly_pld_draft(ctx_d, len_d, K, n_max, tokens, ngram)
        torch.cuda.synchronize()
        got_t, got_n = tokens.cpu().numpy(), ngram.cpu().numpy()
        for b, r in enumerate(rows):
            drafts, n = O.pld_propose(r, n_max, K)
            assert got_t[b, 0] == r[-1]
            assert got_t[b, 1:].tolist() == drafts, (b, K, n_max)
            assert got_n[b] == n
        assert (got_n > 0).sum() > B // 2 and (got_n == 0).sum() > 0


def run_gpu_loop(cfg, prompts, rounds, K, theta, W, n_max, row_scale=None, sample=None):
    fb = __import__("paper_2511_22972_amd.binding", fromlist=["x"])
    lens = [len(p) - 1 for p in prompts]
    cap = (max(lens) + rounds * (K + 1) + K + 1 + 63) // 64 * 64
    wl = GpuWorkload(cfg.replace(K=K), kv_lens=lens, capacity=cap)
    seq = fb.Sequences(wl.kv, max(len(p) for p in prompts) + rounds * (K + 1) + 3, rounds)
    seq.set_sequences(prompts)
    ws = fb.alloc_workspace(fb.fly_decode_workspace_bytes(wl.desc, cfg.batch, K, max(lens) + rounds * (K + 1)))
    if sample is None:
        fb.fly_decode_rounds(wl.model, wl.kv, seq, row_scale, K, theta, W, n_max, rounds, ws)
    else:
        fb.fly_decode_rounds_sampled(wl.model, wl.kv, seq, row_scale, K, theta, W, n_max, rounds, sample[0],
                                     sample[1], ws)
    torch.cuda.synchronize()
    return wl, seq


def oracle_loop(cfg, model, prompts, rounds, K, theta, W, n_max, row_scale=None, sample=None):
    res = []
    for b, p in enumerate(prompts):
        L = len(p) - 1
        kv0 = [(k[b, :L], v[b, :L]) for k, v in model["kv_prefix"]]
        rs = None if row_scale is None else row_scale.reshape(len(prompts), K + 1)[b]
        res.append(O.decode_rounds(p, kv0, model["embed"], model["layers"], model["g_final"], model["w_lm"],
                                   rs, rounds=rounds, K=K, n_max=n_max, theta=theta, W=W, sample=sample,
                                   sample_row0=b * (K + 1),
                                   n_q_heads=cfg.n_q_heads, n_kv_heads=cfg.n_kv_heads, head_dim=cfg.head_dim,
                                   rope_theta=cfg.rope_theta, eps=cfg.rms_eps, storage=cfg.dtype))
    return res


def unambiguous_rounds(res, theta, tol=1e-3):
    """Rounds of one sequence before the first whose decisions hinge on a near tie
    (top-2 margin or entropy-minus-threshold below tol at a draft position or at
    the emitted token)."""
    for r, info in enumerate(res["rounds"]):
        s = res["s"][r]
        margin = info["sample_margin"] if "sample_margin" in info else info["margin"]
        amb = (margin[:s] < tol) | (np.abs(info["h"][:s] - theta) < tol)
        if amb.any():
            return r
    return len(res["rounds"])


def make_prompts(cfg, lens, seed, period=None):
    """Token rows of the given lengths; with `period` the row repeats a random
    block, so that the drafter finds occurrences from the first round on."""
    rows = []
    for b, n in enumerate(lens):
        t = synth.hash_tokens(seed, 900 + b, n, cfg.vocab).tolist()
        if period:
            t = [t[i % period] for i in range(n)]
        rows.append(t)
    return rows


def check_loop(cfg, prompts, rounds, K, theta, W, n_max, kv_tol, row_scale=None, sample=None):
    model = oracle_model(cfg)
    rs_dev = None if row_scale is None else row_scale.to("cuda", torch.float32).contiguous()
    wl, seq = run_gpu_loop(cfg, prompts, rounds, K, theta, W, n_max, row_scale=rs_dev, sample=sample)
    ora = oracle_loop(cfg, model, prompts, rounds, K, theta, W, n_max, row_scale=row_scale, sample=sample)
    trace = seq.accept_trace.cpu().numpy()
    ngram = seq.ngram_trace.cpu().numpy()
    ctx = seq.ctx.cpu().numpy()
    ctx_len = seq.ctx_len.cpu().numpy()
    kv_len = wl.kv.kv_len.cpu().numpy()
    total = seq.accepted_total.cpu().numpy()
    done = seq.rounds_done.cpu().numpy()
    loose = seq.loose_total.cpu().numpy()
    compared_rounds, kept_drafts, loose_kept = 0, 0, 0
    for b, res in enumerate(ora):
        good = unambiguous_rounds(res, theta)
        compared_rounds += good
        assert trace[:good, b].tolist() == res["s"][:good], (b, trace[:, b], res["s"])
        assert ngram[:good, b].tolist() == [r["ngram"] for r in res["rounds"][:good]]
        n_tok = len(prompts[b]) + sum(res["s"][:good])
        assert ctx[b, :n_tok].tolist() == res["y"][:n_tok], b
        kept_drafts += sum(s - 1 for s in res["s"][:good])
        loose_kept += sum(res["n_loose"][:good])
        # the device's own bookkeeping is consistent whatever happened
        assert ctx_len[b] == len(prompts[b]) + trace[:, b].sum() == kv_len[b] + 1
        assert total[b] == trace[:, b].sum() and done[b] == rounds
        if good == rounds:
            assert loose[b] == sum(res["n_loose"])
            # the cache rows written over the rounds equal the oracle's
            L0, L1 = len(prompts[b]) - 1, len(res["y"]) - 1
            for l, (k_ref, v_ref) in enumerate(res["kv"]):
                k_gpu = wl.kv.k[l][b, :, L0:L1, :].permute(1, 0, 2).float().cpu().double()
                v_gpu = wl.kv.v[l][b, :, :, L0:L1].permute(2, 0, 1).float().cpu().double()
                assert (k_gpu - k_ref[L0:L1]).abs().max().item() <= kv_tol, (b, l)
                assert (v_gpu - v_ref[L0:L1]).abs().max().item() <= kv_tol, (b, l)
    print("rounds compared", compared_rounds, "of", rounds * len(prompts), "kept drafts", kept_drafts,
          "loose", loose_kept, "tau", [r["tau"] for r in ora])
    return compared_rounds, kept_drafts, loose_kept


def test_decode_rounds_fp32_tiny_strict_and_loose():
    cfg = C1.replace(batch=3, kv_len=40)
    prompts = make_prompts(cfg, [41, 23, 34], seed=21, period=5)
    rounds = 8
    compared, kept, _ = check_loop(cfg, prompts, rounds, K=4, theta=2.0, W=6, n_max=3, kv_tol=2e-4)
    assert compared >= rounds * 2 and kept > 0
    # every mismatch deferred, window of one: differing drafts are kept
    compared, kept, loose = check_loop(cfg, prompts, rounds, K=6, theta=0.0, W=1, n_max=3, kv_tol=2e-4)
    assert compared >= rounds * 2 and kept > 0


def test_decode_rounds_bf16_small():
    cfg = B16_SMALL.replace(batch=2, kv_len=100)
    prompts = make_prompts(cfg, [101, 60], seed=22, period=7)
    compared, kept, _ = check_loop(cfg, prompts, 6, K=4, theta=0.3, W=2, n_max=3, kv_tol=4e-2)
    assert compared >= 6
    # a prompt and a loose setting under which this random-weight model keeps drafts
    prompts = make_prompts(cfg, [101, 60], seed=24, period=2)
    compared, kept, loose = check_loop(cfg, prompts, 10, K=4, theta=0.0, W=1, n_max=3, kv_tol=4e-2)
    assert compared >= 10 and kept > 0 and loose > 0


def test_decode_rounds_sampled():
    """The loop with drawn target tokens (temperature > 0): tokens, s per round and the cache against
    the oracle's loop with the same draws (row b (K+1) + i of round r's offset), until a round that
    hinges on a near tie of the perturbed logits."""
    cfg = C1.replace(batch=3, kv_len=40)
    prompts = make_prompts(cfg, [41, 23, 34], seed=25, period=5)
    K, rounds = 4, 8
    rs = torch.full((cfg.batch * (K + 1),), 40.0)   # a gain that spreads this tiny model's rows over the entropy range
    compared, kept, _ = check_loop(cfg, prompts, rounds, K=K, theta=2.0, W=6, n_max=3, kv_tol=2e-4, row_scale=rs,
                                   sample=(5, 1000))
    assert compared >= rounds * 2
    compared, kept, loose = check_loop(cfg, prompts, rounds, K=K, theta=0.0, W=1, n_max=3, kv_tol=2e-4,
                                       row_scale=rs, sample=((9 << 32) | 5, (1 << 33) | 7))
    assert compared >= rounds * 2 and kept > 0
    # another offset, another continuation
    wl_a, seq_a = run_gpu_loop(cfg, prompts, 4, K, 2.0, 6, 3, row_scale=rs.cuda(), sample=(5, 1000))
    wl_b, seq_b = run_gpu_loop(cfg, prompts, 4, K, 2.0, 6, 3, row_scale=rs.cuda(), sample=(5, 2000))
    assert not torch.equal(seq_a.ctx, seq_b.ctx)
    bf = B16_SMALL.replace(batch=2, kv_len=100)
    prompts = make_prompts(bf, [101, 60], seed=26, period=7)
    rs = torch.full((bf.batch * (K + 1),), 6.0)
    compared, _, _ = check_loop(bf, prompts, 6, K=K, theta=0.3, W=2, n_max=3, kv_tol=4e-2, row_scale=rs,
                                sample=(3, 50))
    assert compared >= 4


def test_decode_rounds_limits():
    from paper_2511_22972_amd import binding as fb
    cfg = C1.replace(batch=2, kv_len=20)
    prompts = make_prompts(cfg, [21, 12], seed=23)
    wl, seq = run_gpu_loop(cfg, prompts, 0, 4, 0.3, 6, 3)        # zero rounds: nothing changes
    assert seq.ctx_len.cpu().tolist() == [21, 12] and seq.rounds_done.cpu().tolist() == [0, 0]
    ws = fb.alloc_workspace(fb.fly_decode_workspace_bytes(wl.desc, 2, 4, 20 + 1000))
    with pytest.raises(fb.FlyError) as e:                        # the rows cannot hold that many rounds
        fb.fly_decode_rounds(wl.model, wl.kv, seq, None, 4, 0.3, 6, 3, 200, ws)
    assert e.value.status == -10


# ---------------------------------------------------------------------------
# Drafting with a draft model; the loop with the model as drafter
# ---------------------------------------------------------------------------
DRAFT_F32 = C1.replace(name="tiny_drafter", n_layers=1, d=128, n_q_heads=2, n_kv_heads=1, ffn=256, seed=77)
DRAFT_B16 = B16_SMALL.replace(name="bf16_drafter", n_layers=1, d=128, n_q_heads=2, n_kv_heads=1, ffn=256, seed=78)


def oracle_drafts(dcfg, dmodel, b, y, K, first_pos):
    prefix = [(k[b], v[b]) for k, v in dmodel["kv_prefix"]]
    return O.model_draft_greedy(y, K, dmodel["embed"], dmodel["layers"], dmodel["g_final"], dmodel["w_lm"], prefix,
                                first_pos, n_q_heads=dcfg.n_q_heads, n_kv_heads=dcfg.n_kv_heads,
                                head_dim=dcfg.head_dim, rope_theta=dcfg.rope_theta, eps=dcfg.rms_eps,
                                storage=dcfg.dtype, return_margins=True)


@pytest.mark.parametrize("dcfg,K", [(DRAFT_F32, 5), (DRAFT_B16, 4), (DRAFT_B16, 1)])
def test_model_draft_matches_oracle(dcfg, K):
    """fly_model_draft: K chained forward passes of the draft model give the oracle's greedy tokens
    (up to the first draft that hinges on a near tie), for ragged sequence lengths."""
    from paper_2511_22972_amd import binding as fb
    lens = [37, 2, 19, 64]                                    # tokens per sequence (>= 2)
    dcfg = dcfg.replace(batch=len(lens), kv_len=70, K=K)
    wl = GpuWorkload(dcfg, kv_lens=[n - 1 for n in lens], capacity=128)
    prompts = make_prompts(dcfg, lens, seed=31)
    ctx = torch.zeros(len(lens), 80, dtype=torch.int32)
    for b, r in enumerate(prompts):
        ctx[b, :len(r)] = torch.tensor(r, dtype=torch.int32)
    ctx_d = ctx.cuda()
    len_d = torch.tensor(lens, dtype=torch.int32).cuda()
    tokens = torch.full((len(lens), K + 1), -1, dtype=torch.int32, device="cuda")
    ws = fb.alloc_workspace(fb.fly_model_draft_workspace_bytes(wl.desc, len(lens), K, max(lens)))
    fb.fly_model_draft(wl.model, wl.kv, ctx_d, len_d, max(lens), K, tokens, ws)
    torch.cuda.synchronize()
    got = tokens.cpu().numpy()
    dmodel = oracle_model(dcfg)
    compared = 0
    for b, y in enumerate(prompts):
        drafts, margins = oracle_drafts(dcfg, dmodel, b, y, K, len(y) - 2)
        assert got[b, 0] == y[-1]
        for i in range(K):
            if margins[i] < 1e-3:
                break
            assert got[b, 1 + i] == drafts[i], (b, i, got[b], drafts)
            compared += 1
    assert compared >= len(lens) * K - 2
    # a second call on the same state rewrites the same rows: same tokens
    tokens2 = torch.full_like(tokens, -1)
    fb.fly_model_draft(wl.model, wl.kv, ctx_d, len_d, max(lens), K, tokens2, ws)
    torch.cuda.synchronize()
    assert torch.equal(tokens, tokens2)


def run_model_loop(tcfg, dcfg, prompts, rounds, K, theta, W):
    from paper_2511_22972_amd import binding as fb
    lens = [len(p) - 1 for p in prompts]
    cap = (max(lens) + rounds * (K + 1) + 2 * K + 2 + 63) // 64 * 64
    twl = GpuWorkload(tcfg.replace(K=K), kv_lens=lens, capacity=cap)
    dwl = GpuWorkload(dcfg.replace(K=K), kv_lens=lens, capacity=cap)
    seq = fb.Sequences(twl.kv, max(len(p) for p in prompts) + rounds * (K + 1) + 3, rounds)
    seq.set_sequences(prompts)
    ws = fb.alloc_workspace(fb.fly_decode_model_workspace_bytes(twl.desc, dwl.desc, tcfg.batch, K,
                                                                max(lens) + rounds * (K + 1)))
    fb.fly_decode_rounds_model(twl.model, twl.kv, dwl.model, dwl.kv, seq, None, K, theta, W, rounds, ws)
    torch.cuda.synchronize()
    return twl, dwl, seq


def check_model_loop(tcfg, dcfg, prompts, rounds, K, theta, W):
    tmodel, dmodel = oracle_model(tcfg), oracle_model(dcfg)
    twl, dwl, seq = run_model_loop(tcfg, dcfg, prompts, rounds, K, theta, W)
    trace = seq.accept_trace.cpu().numpy()
    ctx = seq.ctx.cpu().numpy()
    compared, kept = 0, 0
    for b, p in enumerate(prompts):
        L = len(p) - 1

        def drafter(y, k, b=b, first=len(p) - 2):
            drafts, margins = oracle_drafts(dcfg, dmodel, b, y, k, first)
            return drafts, min(margins)                       # the tag slot carries the drafter's smallest margin

        kv0 = [(k[b, :L], v[b, :L]) for k, v in tmodel["kv_prefix"]]
        res = O.decode_rounds(p, kv0, tmodel["embed"], tmodel["layers"], tmodel["g_final"], tmodel["w_lm"], None,
                              rounds=rounds, K=K, n_max=1, theta=theta, W=W, drafter=drafter,
                              n_q_heads=tcfg.n_q_heads, n_kv_heads=tcfg.n_kv_heads, head_dim=tcfg.head_dim,
                              rope_theta=tcfg.rope_theta, eps=tcfg.rms_eps, storage=tcfg.dtype)
        good = unambiguous_rounds(res, theta)
        for r, info in enumerate(res["rounds"][:good]):
            if info["ngram"] < 1e-3:                          # a draft hinged on a near tie
                good = r
                break
        assert trace[:good, b].tolist() == res["s"][:good], (b, trace[:, b], res["s"])
        n_tok = len(p) + sum(res["s"][:good])
        assert ctx[b, :n_tok].tolist() == res["y"][:n_tok], b
        compared += good
        kept += sum(s - 1 for s in res["s"][:good])
        assert seq.ctx_len.cpu()[b] == len(p) + trace[:, b].sum() == twl.kv.kv_len.cpu()[b] + 1
    print("model-drafted rounds compared", compared, "of", rounds * len(prompts), "kept drafts", kept)
    return compared, kept


def test_decode_rounds_model_fp32():
    tcfg = C1.replace(batch=3, kv_len=40)
    dcfg = DRAFT_F32.replace(batch=3, kv_len=40, vocab=tcfg.vocab)
    prompts = make_prompts(tcfg, [41, 23, 34], seed=41)
    # (this tiny model's rows are almost uniform: a few rounds hinge on near ties and end the comparison)
    compared, _ = check_model_loop(tcfg, dcfg, prompts, 5, K=4, theta=2.0, W=6)
    assert compared >= 8
    # every mismatch deferred and no window: all K drafts of this unrelated drafter are kept
    compared, kept = check_model_loop(tcfg, dcfg, prompts, 5, K=5, theta=0.0, W=0)
    assert compared >= 8 and kept == 5 * compared


def test_decode_rounds_model_self_drafting_bf16():
    """The target as its own drafter: apart from the one cache row the drafter recomputes from
    the token (the target's synthetic prefix row differs), the drafts are the target's own
    choices, so most rounds keep all K drafts -- also the case where the drafter lacks the row
    of the last draft at the next round."""
    tcfg = B16_SMALL.replace(batch=2, kv_len=60)
    prompts = make_prompts(tcfg, [61, 30], seed=42)
    compared, kept = check_model_loop(tcfg, tcfg, prompts, 6, K=3, theta=0.3, W=1)
    assert compared >= 8 and kept >= 8
