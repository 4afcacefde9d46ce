"""Parity at the full sizes of the benchmark workloads, in the launch
configuration bench.py times (same shapes, hence the same kernel plans).

Free-running bf16 agreement at depth means little (rounding flips decorrelate
the two sides at full width), so the full-depth comparison is teacher-forced and
lives in tests/test_gpu_fulldepth.py.  Here:
  * every stage is compared with the oracle at full width on seeded stage
    inputs (one decoder layer from a seeded residual stream; the LM head from
    seeded hidden states, all rows; the 32768-key attention);
  * the acceptance rule runs on the statistics of the 1088-row stress workload
    with drafts drawn three ways;
  * the 8B shape runs free-running end to end at reduced depth with an
    oracle-built draft chain;
  * the full 80-layer 70B-shaped step is checked through properties that hold
    at any size (reproducibility, causality, the acceptance rule applied to the
    device's own statistics, ranges, cache-length bookkeeping).
"""
import numpy as np
import pytest
import torch

import synth
from oracle import fly_oracle as O
from tests import helpers
from tests.gpu_harness import GpuWorkload, compare_tail, compare_verify

pytestmark = pytest.mark.gpu

C2, C3, C4, C5 = (synth.CONFIGS[k] for k in ("c2_8b", "c3_70b", "c4_405b_slice", "c5_stress"))


def one_layer_case(cfg):
    """fly_decoder_layers over one full-width layer vs the oracle's decoder_layer."""
    cfg = cfg.replace(n_layers=1)
    wl = GpuWorkload(cfg)
    fb = wl.fb
    x0 = synth.hash_normal(cfg.seed, 300, (cfg.M, cfg.d), 1.0, torch.float32, "cuda")
    x = x0.clone()
    fb.fly_decoder_layers(wl.model, wl.kv, x, 0, 1, cfg.batch, cfg.K, wl.ws)
    torch.cuda.synchronize()
    got = x.cpu().double().view(cfg.batch, cfg.K + 1, cfg.d)
    w = helpers.oracle_layer_weights(cfg, 0, "cuda")
    kp, vp = (t.to("cpu", torch.float64) for t in synth.make_kv_prefix(cfg, 0, "cuda"))
    num = O.Numerics(cfg.dtype)
    worst_max, worst_rms, worst_row, worst_blk = 0.0, 0.0, 0.0, 0.0
    kc = wl.kv.k[0]
    vc = wl.kv.v[0]
    L = cfg.kv_len
    for b in range(cfg.batch):
        xb = x0.cpu().double().view(cfg.batch, cfg.K + 1, cfg.d)[b]
        ref, k_new, v_new = O.decoder_layer(xb, w, kp[b], vp[b], cfg.n_q_heads, cfg.n_kv_heads,
                                            cfg.head_dim, cfg.rope_theta, cfg.rms_eps, num)
        # The residual stream of a randomly initialised full-width layer has rms 7 (d = 8192) to 21
        # (d = 16384), and with 10^4-10^5 bf16 roundings per row a few always fall on the other
        # side of a rounding boundary (fp32 vs fp64), after which the two sides differ by ordinary
        # bf16 noise (0.1-0.3 % rms).  The check is therefore relative to the reference's rms: a
        # wrong tile, head or row would be off by the order of the rms itself.
        scale = ref.pow(2).mean().sqrt().item()
        err = (got[b] - ref).abs()
        worst_max = max(worst_max, err.max().item() / scale)
        worst_rms = max(worst_rms, err.pow(2).mean().sqrt().item() / scale)
        # the difference must look like rounding noise everywhere: no row and no block of 128
        # columns may carry much more of it than the rest (a wrong tile, head or split would)
        e2 = (got[b] - ref).pow(2)
        overall = e2.mean().sqrt().item()
        worst_row = max(worst_row, e2.mean(dim=1).sqrt().max().item() / overall)
        worst_blk = max(worst_blk, e2.view(e2.shape[0], -1, 128).mean(dim=(0, 2)).sqrt().max().item() / overall)
        assert abs((got[b] - ref).mean().item()) < 0.1 * overall
        gk = kc[b, :, L:L + cfg.K + 1, :].float().cpu().double().permute(1, 0, 2)
        gv = vc[b, :, :, L:L + cfg.K + 1].float().cpu().double().permute(2, 0, 1)
        # Appended rows are bf16 values.  Almost all are identical; where the fp32 and fp64
        # evaluations of a value straddle a rounding boundary they are one bf16 ulp apart, and
        # where that happened to an element of the normalised input row, every q/k/v element
        # of that row moves by ulp(x_i) * W[i, :] (up to about 1e-3 in absolute terms).
        for got_t, ref_t in ((gk, k_new), (gv, v_new)):
            diff = (got_t - ref_t).abs()
            assert torch.all(diff <= ref_t.abs() * 2.0 ** -7 + 1e-3), diff.max()
            assert (diff != 0).double().mean().item() < 0.02
    print(cfg.name, "one full-width layer: residual-stream error / rms(ref): max", worst_max, "rms", worst_rms,
          "; noisiest row / overall", worst_row, "noisiest 128-column block / overall", worst_blk)
    # twice what the shapes of each width show (an fp32 evaluation of the same layer on the CPU with
    # the same rounding points differs from the fp64 oracle by as much as the device does)
    rms_tol, max_tol = {4096: (1.6e-3, 1.0e-2), 8192: (5e-3, 3.5e-2), 16384: (8.5e-3, 6e-2)}[cfg.d]
    assert worst_rms < rms_tol and worst_max < max_tol
    # observed: the noisiest row carries 1.5-2.0 times the overall rms, the noisiest block of 128
    # columns 1.03-1.07 times
    assert worst_row < 3.0 and worst_blk < 1.5, (worst_row, worst_blk)
    return worst_max


def test_c3_one_layer_full_width():
    one_layer_case(C3)


def test_c2_one_layer_full_width():
    one_layer_case(C2)


def test_c4_one_layer_full_width():
    # 136 rows, d = 16384, 272 query rows per KV head, 8192-token caches
    one_layer_case(C4)


@pytest.mark.parametrize("name", ["p70b_k15", "p70b_k15_b16", "p405b_k25_slice"])
def test_paper_sized_blocks_one_layer_full_width(name):
    # K = 15 / 25 at batch 1 (16 / 26 rows; 128 / 416 query rows per KV head) and K = 15 at
    # batch 16 (256 rows: the LDS-tiled GEMMs)
    one_layer_case(synth.CONFIGS[name])


@pytest.mark.parametrize("M", [136, 256])
def test_down_projection_405b_width_is_reproducible(M):
    """The down projection at the 405B width (53248 -> 16384): its activation block does not fit
    the L2, so the loads of one wave return in every order the memory system allows.  Forty
    launches must give the same bits, and the sum of the split-K partials the product.  (A form of
    the 81..256-row kernel that counted the waits for its activation copies by hand failed this in
    about one launch out of twelve.)"""
    from paper_2511_22972_amd import binding as fb
    cfg = synth.CONFIGS["c4_405b_slice"]
    Kd, N = cfg.ffn, cfg.d
    w = synth.hash_normal(cfg.seed, 400, (Kd, N), 0.02, torch.bfloat16, "cuda")
    wp = torch.empty(Kd * N, dtype=torch.bfloat16, device="cuda")
    fb.fly_pack_weight(w, wp, N)
    xa = synth.hash_normal(cfg.seed, 313, (M, Kd), 1.0, torch.bfloat16, "cuda")
    part = torch.empty(16 * M * N, dtype=torch.float32, device="cuda")
    splits = fb.fly_proj_partial(xa, wp, part, N)
    torch.cuda.synchronize()
    first = part[: splits * M * N].clone()
    ref = xa.float() @ w.float()
    assert float((first.view(splits, M, N).sum(0) - ref).abs().max()) < 2e-3
    for i in range(40):
        assert fb.fly_proj_partial(xa, wp, part, N) == splits
        torch.cuda.synchronize()
        assert torch.equal(part[: splits * M * N], first), i


@pytest.mark.parametrize("name", ["c3_70b", "c4_405b_slice", "p70b_k15_b16"])
def test_layer_result_does_not_depend_on_stale_memory(name):
    """One full-width layer with the workspace and the cache rows past the block filled with NaN
    bytes, with huge finite values and with zeros: the result must be the same bits every time (no
    kernel reads workspace it has not written in this call, nor cache rows that are not part of the
    sequence)."""
    cfg = synth.CONFIGS[name].replace(n_layers=1)
    wl = GpuWorkload(cfg)
    fb = wl.fb
    x0 = synth.hash_normal(cfg.seed, 300, (cfg.M, cfg.d), 1.0, torch.float32, "cuda")

    def run():
        x = x0.clone()
        fb.fly_decoder_layers(wl.model, wl.kv, x, 0, 1, cfg.batch, cfg.K, wl.ws)
        torch.cuda.synchronize()
        return x

    ref = run()
    assert torch.isfinite(ref).all()
    end = cfg.kv_len + cfg.K + 1
    for byte, value in ((0xFF, float("nan")), (0x7F, 3e38), (0x00, 0.0)):
        wl.ws.fill_(byte)
        assert torch.equal(run(), ref), ("workspace", byte)
        wl.kv.k[0][:, :, end:, :] = value
        wl.kv.v[0][:, :, :, end:] = value
        assert torch.equal(run(), ref), ("cache padding", byte)


def test_kernels_with_hand_counted_waits_are_reproducible():
    """The LDS-tiled GEMM and the attention kernel count the waits for their LDS-direct loads by hand.
    At sizes that miss every cache (1088 x 28672 activations, a 32768-key cache) a hundred launches
    must give the same bits, and the GEMM the product."""
    from paper_2511_22972_amd import binding as fb
    M, Kd, N = 1088, 28672, 8192
    xa = synth.hash_normal(1, 5, (M, Kd), 1.0, torch.bfloat16, "cuda")
    w = synth.hash_normal(1, 6, (Kd, N), 0.02, torch.bfloat16, "cuda")
    wp = torch.empty(Kd * N, dtype=torch.bfloat16, device="cuda")
    fb.fly_pack_weight(w, wp, N)
    part = torch.empty(16 * M * N, dtype=torch.float32, device="cuda")
    splits = fb.fly_proj_partial(xa, wp, part, N)
    torch.cuda.synchronize()
    first = part[: splits * M * N].clone()
    assert float((first.view(splits, M, N).sum(0) - xa.float() @ w.float()).abs().max()) < 2e-3
    for i in range(100):
        fb.fly_proj_partial(xa, wp, part, N)
        torch.cuda.synchronize()
        assert torch.equal(part[: splits * M * N], first), i
    del xa, w, wp, part, first
    cfg = C5.replace(n_layers=1, batch=16)
    desc = fb.make_desc(cfg)
    cap = (cfg.kv_len + cfg.K + 1 + 63) // 64 * 64
    kv = fb.KVCache(desc, cfg.batch, cap)
    kv.k[0].normal_()
    kv.v[0].normal_()
    kv.set_lengths([cfg.kv_len] * cfg.batch)
    q = synth.hash_normal(2, 7, (cfg.M, cfg.q_dim), 1.0, torch.bfloat16, "cuda")
    o = torch.empty_like(q)
    ws = fb.alloc_workspace(fb.fly_workspace_bytes(desc, cfg.batch, cfg.K, cfg.kv_len))
    fb.fly_attention(desc, kv, 0, q, o, cfg.batch, cfg.K, ws)
    torch.cuda.synchronize()
    first = o.clone()
    assert torch.isfinite(first.float()).all()
    for i in range(100):
        fb.fly_attention(desc, kv, 0, q, o, cfg.batch, cfg.K, ws)
        torch.cuda.synchronize()
        assert torch.equal(o, first), i


def lmhead_full(cfg, M, sample_rows=None, return_logits=False):
    from paper_2511_22972_amd import binding as fb
    d, V = cfg.d, cfg.vocab
    hidden = synth.make_hidden(cfg, M, "cuda")
    w = synth.make_weight(cfg, "w_lm", -1, "cuda")
    wp = torch.empty(d * V, dtype=torch.bfloat16, device="cuda")
    fb.fly_pack_weight(w, wp, V)
    u = synth.hash_uniform(cfg.seed, 777, M, "cuda")
    rs = torch.exp(np.log(0.1) + u * (np.log(10.0) - np.log(0.1))).to(torch.float32)   # 1/T, T log-uniform
    argmax = torch.zeros(M, dtype=torch.int32, device="cuda")
    p1, hn, lse = (torch.zeros(M, dtype=torch.float32, device="cuda") for _ in range(3))
    ws = fb.alloc_workspace(fb.fly_lmhead_workspace_bytes(M, d, V, fb.FLY_BF16))
    fb.fly_lmhead_entropy_argmax(hidden, wp, rs, V, argmax, p1, hn, lse, ws)
    torch.cuda.synchronize()
    rows = np.arange(M) if sample_rows is None else np.asarray(sample_rows)
    logits = O.lm_head_logits(hidden[rows].cpu().double(), w.cpu().double(), rs[rows].cpu())
    ref = O.decision_statistics(logits)
    got = {k: t.cpu().numpy()[rows] for k, t in (("argmax", argmax), ("p_top1", p1), ("h", hn), ("lse", lse))}
    err = {k: float(np.abs(got[k] - ref[k]).max()) for k in ("lse", "h", "p_top1")}
    print(cfg.name, "LM head rows", len(rows), "errors", err, "h range", ref["h"].min(), ref["h"].max())
    for v in err.values():
        assert v < 2e-3          # same bf16 inputs on both sides, fp32 accumulation: far inside 2e-2
    near_tie = ref["margin"] < 1e-3
    assert np.all((got["argmax"] == ref["argmax"]) | near_tie)
    assert ref["h"].min() < 0.3 < ref["h"].max()
    # the same launch shape with a token drawn per row (temperature > 0)
    sampled = torch.zeros(M, dtype=torch.int32, device="cuda")
    argmax2 = torch.zeros(M, dtype=torch.int32, device="cuda")
    fb.fly_lmhead_entropy_sample(hidden, wp, rs, V, cfg.seed, 5, sampled, argmax2, p1, hn, lse, ws)
    torch.cuda.synchronize()
    assert torch.equal(argmax2, argmax)
    drawn = O.sample_rows(logits.numpy(), cfg.seed, 5, rows=rows)
    ok = (sampled.cpu().numpy()[rows] == drawn["token"]) | (drawn["margin"] < 1e-3)
    assert np.all(ok), np.argwhere(~ok)
    assert (drawn["token"] != ref["argmax"]).any()
    if return_logits:
        return got, ref, rs, logits.numpy()
    return got, ref, rs


def test_c3_lm_head_full_vocab():
    lmhead_full(C3, C3.M)


def test_c5_stress_lm_head_and_acceptance_all_rows():
    """The LM-head / acceptance stress workload: 64 sequences x 17 positions = 1088 rows x 128256
    columns, per-row temperature log-uniform in [0.1, 10] so the entropies sweep across the gate
    threshold.  The oracle computes the statistics of ALL rows; then the drafts are drawn three ways
    from the oracle's logits (the target's token w.p. 0.5, the second-best token w.p. 0.2, a uniform
    token otherwise), and fly_accept on the DEVICE's statistics (theta = 0.3, W = 6, K = 16) must give
    the oracle's accepted length, correction token and kept-mismatch count for every sequence none of
    whose rows is a near tie (margin or |h - theta| below 1e-3)."""
    from paper_2511_22972_amd import binding as fb
    cfg = C5
    B, K, R, M = cfg.batch, cfg.K, cfg.K + 1, cfg.M
    got, ref, rs, logits = lmhead_full(cfg, M, return_logits=True)
    # three-way drafts (an input recipe: the rows are independent here, nothing feeds back)
    l32 = logits.astype(np.float32)                     # the precision the target's token is decided in
    best = np.argmax(l32, axis=1)
    assert np.array_equal(best, ref["argmax"])
    l32[np.arange(M), best] = -np.inf
    second = np.argmax(l32, axis=1).reshape(B, R)      # lowest index among the runners-up
    best = best.reshape(B, R)
    _, alt, kind = synth.make_draft_draws(cfg)
    kind, alt = kind.numpy(), alt.numpy()
    draft = np.where(kind < 0.5, best[:, :K], np.where(kind < 0.7, second[:, :K], alt)).astype(np.int32)
    ora = O.accept_block(draft, ref["argmax"].reshape(B, R), ref["h"].reshape(B, R), cfg.theta, cfg.window)
    dev = lambda a, dt: torch.as_tensor(np.ascontiguousarray(a), dtype=dt).cuda()
    acc, nxt, loose = (torch.zeros(B, dtype=torch.int32, device="cuda") for _ in range(3))
    fb.fly_accept(dev(draft, torch.int32), dev(got["argmax"].reshape(B, R), torch.int32),
                  dev(got["h"].reshape(B, R), torch.float32), cfg.theta, cfg.window, acc, nxt, loose)
    torch.cuda.synchronize()
    amb = ((ref["margin"] < 1e-3) | (np.abs(ref["h"] - cfg.theta) < 1e-3)).reshape(B, R)
    clean = ~amb.any(axis=1)
    print("c5 acceptance: clean sequences", int(clean.sum()), "of", B, "accepted lengths",
          np.bincount(ora["accept_len"], minlength=K + 1).tolist(), "kept mismatches", int(ora["n_loose"].sum()))
    assert clean.sum() >= B - 8
    for k, t in (("accept_len", acc), ("next_token", nxt), ("n_loose", loose)):
        assert np.array_equal(t.cpu().numpy()[clean], ora[k][clean]), k
    # the workload does what it is for: rows on both sides of the gate, several outcomes, kept mismatches
    mism = draft != ref["argmax"].reshape(B, R)[:, :K]
    h_at_mismatch = ref["h"].reshape(B, R)[:, :K][mism]
    assert (h_at_mismatch < cfg.theta).any() and (h_at_mismatch >= cfg.theta).any()
    assert len(np.unique(ora["accept_len"])) >= 4 and ora["n_loose"].sum() >= 1
    # and with the loose path off the same drafts give exact-match decoding on the device too
    fb.fly_accept(dev(draft, torch.int32), dev(got["argmax"].reshape(B, R), torch.int32),
                  dev(got["h"].reshape(B, R), torch.float32), 2.0, cfg.window, acc, nxt, loose)
    torch.cuda.synchronize()
    std = np.array([O.s_standard(O.match_indicator(draft[b], got["argmax"].reshape(B, R)[b])) for b in range(B)])
    assert np.array_equal(acc.cpu().numpy() + 1, std) and int(loose.sum()) == 0


def test_c5_stress_attention_32768_keys():
    """The attention half of the stress workload at its full size: 64 sequences, 17 query positions
    x 8 query heads per KV head (136 rows) over 32768 cached keys plus the 17 new rows, against the
    oracle for the first and the last sequence (one rounding, the bf16 output, separates the sides)."""
    from paper_2511_22972_amd import binding as fb
    cfg = C5.replace(n_layers=1)
    B, K, R, L = cfg.batch, cfg.K, cfg.K + 1, cfg.kv_len
    desc = fb.make_desc(cfg)
    cap = (L + R + 63) // 64 * 64
    kv = fb.KVCache(desc, B, cap)
    k, v = synth.make_kv_prefix(cfg.replace(kv_len=L + R), 0, "cuda")   # the last R rows stand for the new rows
    kv.load_prefix(0, k, v)
    kv.set_lengths([L] * B)
    q = synth.hash_normal(cfg.seed, 310, (cfg.M, cfg.q_dim), 2.0, torch.bfloat16, "cuda")
    o = torch.zeros_like(q)
    ws = fb.alloc_workspace(fb.fly_workspace_bytes(desc, B, K, L))
    fb.fly_attention(desc, kv, 0, q, o, B, K, ws)
    torch.cuda.synchronize()
    got = o.float().cpu().double().view(B, R, cfg.n_q_heads, cfg.head_dim)
    num = O.Numerics("bf16")
    for b in (0, B - 1):
        qb = q.float().cpu().double().view(B, R, cfg.n_q_heads, cfg.head_dim)[b]
        ref = num.act(O.attention_one_sequence(qb, k[b].cpu().double(), v[b].cpu().double(), L, num))
        diff = (got[b] - ref).abs()
        same = (diff == 0).double().mean().item()
        print("c5 attention, sequence", b, "max abs diff", diff.max().item(), "identical elements", same)
        # as in the small attention stage test: a probability whose fp32 and fp64 evaluations straddle
        # a bf16 rounding boundary moves an output row by about 2^-8 p_j |v_j| / sum(p)
        assert diff.max().item() <= 4e-3, (b, diff.max())
        assert same > 0.97, (b, same)


def test_c2_shape_end_to_end_reduced_depth():
    """8B shape (d = 4096, 32/8 heads, F = 14336, V = 128256, K = 8, L = 2048), 3 layers,
    free-running with an oracle-built draft chain (floats; integers where no margin is below twice
    the float tolerance), then the oracle's end of the step on the device's residual stream
    (integers outside the 1e-3 exclusions).  All 32 layers: tests/test_gpu_fulldepth.py."""
    cfg = C2.replace(n_layers=3, temperatures=(0.3, 1.0, 3.0))
    model = helpers.oracle_model(cfg, device="cuda")
    tokens = helpers.draft_chain(cfg, model)
    ora = helpers.oracle_verify(cfg, model, tokens)
    wl = GpuWorkload(cfg)
    gpu = wl.verify(tokens, helpers.row_scale(cfg))
    compare_verify(gpu, ora, cfg.theta, 2e-2, O.accept_block, tokens, cfg.window, min_clean=0, int_tol=4e-2)
    tail = helpers.oracle_tail(cfg, gpu["hidden"], tokens, model["g_final"], model["w_lm"])
    compare_tail(gpu, tail, cfg.theta, O.accept_block, tokens, cfg.window, min_clean=1)


def test_c3_full_depth_properties():
    """The benchmark's own configuration: 80 layers, 36 rows, 4 x 4096-token caches."""
    cfg = C3
    wl = GpuWorkload(cfg)
    rng = np.random.default_rng(7)
    rs = (1.0 / synth.make_row_temperature(cfg)).reshape(-1)
    tokens = rng.integers(0, cfg.vocab, size=(cfg.batch, cfg.K + 1)).astype(np.int32)
    a = wl.verify(tokens, rs, want_hidden=False)
    # build a block whose drafts partly match the device's own argmax chain (two passes suffice
    # for position 1 and 2; later positions are whatever they are) so that several outcomes occur
    tokens[:, 1] = a["argmax"][:, 0]
    b = wl.verify(tokens, rs, want_hidden=False)
    tokens[0::2, 2] = b["argmax"][0::2, 1]
    c = wl.verify(tokens, rs, want_hidden=False)
    again = wl.verify(tokens, rs, want_hidden=False)
    for k in c:
        assert np.array_equal(c[k], again[k]), k                         # bit-reproducible
    for k in ("argmax", "h_norm", "p_top1", "lse"):
        assert np.array_equal(a[k][:, :1], c[k][:, :1]), k               # causality: row 0 never changed
        assert np.array_equal(b[k][:, :2], c[k][:, :2]), k
    assert np.all(np.isfinite(c["lse"])) and np.all(c["h_norm"] > 0) and np.all(c["h_norm"] <= 1 + 1e-5)
    assert np.all(c["p_top1"] > 0) and np.all(c["p_top1"] <= 1)
    for theta, W in ((cfg.theta, cfg.window), (2.0, 6), (0.0, 0), (0.3, 1)):
        out = wl.verify(tokens, rs, theta=theta, W=W, want_hidden=False)
        own = O.accept_block(tokens[:, 1:], out["argmax"], out["h_norm"], theta, W)
        for k in ("accept_len", "next_token", "n_loose"):
            assert np.array_equal(out[k], own[k]), (k, theta, W)
        assert np.array_equal(out["kv_len_out"], cfg.kv_len + out["accept_len"] + 1)
    assert np.all(c["accept_len"] >= 1)                                   # draft 1 was the target's token
