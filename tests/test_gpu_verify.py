"""HIP decoder layers and the whole verification step against the CPU oracle,
element by element, on seeded synthetic workloads small enough for the oracle
to finish in seconds but spanning several tiles, ragged tails and ragged
cache lengths."""
import numpy as np
import pytest
import torch

import synth
from oracle import fly_oracle as O
from tests import helpers
from tests.gpu_harness import GpuWorkload, compare_tail, compare_verify

pytestmark = pytest.mark.gpu

C1 = synth.CONFIGS["c1_tiny"]
# bf16 shapes: small multiples of the kernels' tiles, with ragged row counts
B16_SMALL = synth.CONFIGS["c2_8b"].replace(
    name="bf16_small", n_layers=2, d=256, n_q_heads=4, n_kv_heads=2, ffn=512, vocab=2048,
    batch=2, K=4, kv_len=150, weight_std=0.05)
B16_WIDE = synth.CONFIGS["c2_8b"].replace(
    name="bf16_wide", n_layers=2, d=512, n_q_heads=16, n_kv_heads=2, ffn=1056, vocab=4112,
    batch=3, K=8, kv_len=300, weight_std=0.04, temperatures=(0.3, 1.0, 3.0))


def oracle_model_from_gpu(cfg):
    """Oracle-side fp64 copies of the same seeded tensors (generated on the GPU
    by the shared generator, which is bit-identical to the CPU one)."""
    return helpers.oracle_model(cfg, device="cuda")


def ragged_prefix(model, kv_lens):
    """Per-sequence prefixes of different lengths for the oracle."""
    out = []
    for k, v in model["kv_prefix"]:
        out.append(([k[b, :L] for b, L in enumerate(kv_lens)], [v[b, :L] for b, L in enumerate(kv_lens)]))
    return out


def run_layers_case(cfg, kv_lens, x_std=1.0):
    """fly_decoder_layers on a random residual stream vs the oracle's layers."""
    wl = GpuWorkload(cfg, kv_lens=kv_lens)
    fb = wl.fb
    M = cfg.M
    x0 = synth.hash_normal(cfg.seed, 300, (M, cfg.d), x_std, torch.float32, "cuda")
    x = x0.clone()
    fb.fly_decoder_layers(wl.model, wl.kv, x, 0, cfg.n_layers, cfg.batch, cfg.K, wl.ws)
    torch.cuda.synchronize()
    got = x.cpu().double().numpy().reshape(cfg.batch, cfg.K + 1, cfg.d)

    model = oracle_model_from_gpu(cfg)
    prefix = ragged_prefix(model, kv_lens)
    num = O.Numerics(cfg.dtype)
    ref = np.zeros_like(got)
    new_kv = []
    for b in range(cfg.batch):
        xb = x0.cpu().double().view(cfg.batch, cfg.K + 1, cfg.d)[b]
        per_layer = []
        for li, w in enumerate(model["layers"]):
            xb, k_new, v_new = O.decoder_layer(xb, w, prefix[li][0][b], prefix[li][1][b], cfg.n_q_heads,
                                               cfg.n_kv_heads, cfg.head_dim, cfg.rope_theta, cfg.rms_eps, num)
            per_layer.append((k_new, v_new))
        ref[b] = xb.numpy()
        new_kv.append(per_layer)
    return wl, got, ref, new_kv


def check_appended_kv(wl, cfg, kv_lens, new_kv, tol):
    """Rows kv_len..kv_len+K of every layer's cache hold the oracle's new k, v."""
    for li in range(cfg.n_layers):
        kc = wl.kv.k[li].float().cpu().double()          # [B,Hkv,cap,hd]
        vc = wl.kv.v[li].float().cpu().double()          # [B,Hkv,hd,cap]
        for b, L in enumerate(kv_lens):
            k_new, v_new = new_kv[b][li]                 # [R,Hkv,hd]
            got_k = kc[b, :, L:L + cfg.K + 1, :].permute(1, 0, 2)
            got_v = vc[b, :, :, L:L + cfg.K + 1].permute(2, 0, 1)
            for name, g_t, r_t in (("k", got_k, k_new), ("v", got_v, v_new)):
                diff = (g_t - r_t).abs()
                # absolute tolerance for fp32 storage; one bf16 ulp where a rounding flipped
                assert torch.all(diff <= tol + r_t.abs() * 2.0 ** -7), (name, li, b, diff.max())


def test_layers_f32_tiny():
    cfg = C1.replace(batch=2, K=4)
    kv_lens = [128, 77]
    wl, got, ref, new_kv = run_layers_case(cfg, kv_lens)
    assert np.abs(got - ref).max() < 1e-4
    check_appended_kv(wl, cfg, kv_lens, new_kv, 1e-5)


# d = 1056 is 33 k-steps and F = 1184 is 37: ragged last chunks in every projection, 48 rows
B16_RAGGED_K = synth.CONFIGS["c2_8b"].replace(
    name="bf16_ragged_k", n_layers=2, d=1056, n_q_heads=6, n_kv_heads=3, ffn=1184, vocab=2048,
    batch=3, K=15, kv_len=100, weight_std=0.03)


@pytest.mark.parametrize("cfg,kv_lens", [(B16_SMALL, [150, 64]), (B16_WIDE, [300, 1, 129]),
                                         (B16_RAGGED_K, [100, 0, 37]), (B16_SMALL.replace(batch=1, K=1, kv_len=9), [9])])
def test_layers_bf16(cfg, kv_lens):
    wl, got, ref, new_kv = run_layers_case(cfg, kv_lens)
    # residual stream is fp32 on the device; both sides round the same tensors to bf16
    print("layer max abs err", np.abs(got - ref).max(), "max |ref|", np.abs(ref).max())
    assert np.abs(got - ref).max() < 2e-2
    # appended keys/values are bf16 values: equal up to one bf16 ulp at rounding boundaries
    check_appended_kv(wl, cfg, kv_lens, new_kv, 1e-6 if cfg.n_layers == 1 else 2e-2)


def test_layers_bf16_single_row_tile_edges():
    """M = 17 rows (one full 16-row tile plus one) and 136 rows (nine tiles)."""
    for batch, K in ((1, 16), (8, 16)):
        cfg = B16_SMALL.replace(batch=batch, K=K, n_layers=1, kv_len=70)
        wl, got, ref, _ = run_layers_case(cfg, [70] * batch)
        print("layer max abs err", np.abs(got - ref).max(), "max |ref|", np.abs(ref).max())
        assert np.abs(got - ref).max() < 2e-2


def verify_case(cfg, theta=None, W=None):
    model = oracle_model_from_gpu(cfg)
    tokens = helpers.draft_chain(cfg, model)
    ora = helpers.oracle_verify(cfg, model, tokens, theta=theta, W=W)
    wl = GpuWorkload(cfg)
    gpu = wl.verify(tokens, helpers.row_scale(cfg), theta=theta, W=W)
    return wl, tokens, gpu, ora


def test_verify_c1_tiny_fp32():
    """The tiny fp32 configuration end to end, free-running."""
    cfg = C1
    wl, tokens, gpu, ora = verify_case(cfg)
    err = compare_verify(gpu, ora, cfg.theta, 1e-4, O.accept_block, tokens, cfg.window)
    # with W = 6 and K = 4 no window fits: the rule is exact-match decoding here
    std = np.array([O.s_standard(O.match_indicator(tokens[b, 1:], ora["argmax"][b])) for b in range(cfg.batch)])
    assert np.array_equal(ora["s"], std)
    assert np.array_equal(gpu["kv_len_out"], cfg.kv_len + gpu["accept_len"] + 1)
    assert err["n_clean_sequences"] >= 1


@pytest.mark.parametrize("W", [0, 1, 2])
def test_verify_c1_with_fitting_windows(W):
    """Same model with a logit gain so both gate branches occur, windows that fit K = 4,
    and a batch of sequences."""
    cfg = C1.replace(batch=6, logit_gain=12.0, window=W)
    wl, tokens, gpu, ora = verify_case(cfg)
    compare_verify(gpu, ora, cfg.theta, 1e-4, O.accept_block, tokens, W, min_clean=3)
    assert ora["h"][:, :-1].min() < cfg.theta < ora["h"][:, :-1].max()


# 12 x 9 = 108 rows and 20 x 9 = 180 rows: the whole step through the GEMM kernel with 32-row tiles
B16_ROWS108 = B16_SMALL.replace(name="bf16_rows108", batch=12, K=8, kv_len=70)
B16_ROWS180 = B16_SMALL.replace(name="bf16_rows180", batch=20, K=8, kv_len=40)


@pytest.mark.parametrize("cfg", [B16_SMALL, B16_WIDE, B16_RAGGED_K, B16_ROWS108, B16_ROWS180])
def test_verify_bf16_small(cfg):
    """Two comparisons.  Free-running (the oracle runs its own layers): a bf16 rounding that falls
    the other way in fp32 than in fp64 moves a hidden state, so the logits of the two sides differ
    by up to the 2e-2 tolerance and the integer outputs are compared only where no margin is below
    twice that.  Teacher-forced (the oracle's final norm, LM head, statistics and rule on the
    device's own residual stream): the integer outputs must agree outside the 1e-3 exclusions."""
    cfg = cfg.replace(window=2)
    wl, tokens, gpu, ora = verify_case(cfg)
    compare_verify(gpu, ora, cfg.theta, 2e-2, O.accept_block, tokens, cfg.window, min_clean=0, int_tol=4e-2)
    model = oracle_model_from_gpu(cfg)
    tail = helpers.oracle_tail(cfg, gpu["hidden"], tokens, model["g_final"], model["w_lm"])
    err = compare_tail(gpu, tail, cfg.theta, O.accept_block, tokens, cfg.window, min_clean=cfg.batch // 2)
    print(cfg.name, "teacher-forced tail", err)
    assert np.array_equal(gpu["kv_len_out"], cfg.kv_len + gpu["accept_len"] + 1)


def test_verify_longest_block_and_empty_prefix():
    """K = 63 (the longest block one wavefront holds), one sequence with an EMPTY cached prefix and
    one with five cached rows, 128 rows in all; then the same block with the largest window an
    int32 holds, which no draft position can fit: exact-match decoding."""
    cfg = B16_SMALL.replace(name="bf16_k63", batch=2, K=63, kv_len=5, window=6, temperatures=(0.3, 1.0, 3.0))
    kv_lens = [0, 5]
    model = oracle_model_from_gpu(cfg)
    prefix = ragged_prefix(model, kv_lens)
    rng = np.random.default_rng(3)
    tokens = rng.integers(0, cfg.vocab, size=(cfg.batch, cfg.K + 1)).astype(np.int32)
    wl = GpuWorkload(cfg, kv_lens=kv_lens)
    rs = helpers.row_scale(cfg)
    first = wl.verify(tokens, rs)
    # drafts that partly follow the device's own targets, so that long accepted prefixes occur
    keep = rng.random((cfg.batch, cfg.K)) < 0.9
    tokens[:, 1:] = np.where(keep, first["argmax"][:, :-1], tokens[:, 1:])
    gpu = wl.verify(tokens, rs)
    ora = {k: [] for k in ("argmax", "margin", "lse", "h", "p_top1", "accept_len", "next_token", "n_loose")}
    for b, L in enumerate(kv_lens):        # the oracle takes one prefix length per call
        out = O.verify_block(tokens[b:b + 1], model["embed"], model["layers"], model["g_final"], model["w_lm"],
                             [(k[b][None], v[b][None]) for k, v in prefix], rs.view(cfg.batch, -1)[b],
                             n_q_heads=cfg.n_q_heads, n_kv_heads=cfg.n_kv_heads, head_dim=cfg.head_dim,
                             rope_theta=cfg.rope_theta, eps=cfg.rms_eps, theta=cfg.theta, W=cfg.window,
                             storage=cfg.dtype)
        for k in ora:
            ora[k].append(out[k])
    ora = {k: np.concatenate(v) for k, v in ora.items()}
    compare_verify(gpu, ora, cfg.theta, 2e-2, O.accept_block, tokens, cfg.window, min_clean=0, int_tol=4e-2)
    tail = helpers.oracle_tail(cfg, gpu["hidden"], tokens, model["g_final"], model["w_lm"])
    compare_tail(gpu, tail, cfg.theta, O.accept_block, tokens, cfg.window, min_clean=1)
    assert np.array_equal(gpu["kv_len_out"], np.asarray(kv_lens) + gpu["accept_len"] + 1)
    huge = wl.verify(tokens, rs, W=2 ** 31 - 1)
    std = np.array([O.s_standard(O.match_indicator(tokens[b, 1:], huge["argmax"][b])) for b in range(cfg.batch)])
    assert np.array_equal(huge["accept_len"] + 1, std) and not huge["n_loose"].any()


def test_verify_limits_on_device():
    """theta > 1 gives exact-match decoding; theta = 0 with W = 0 accepts everything."""
    cfg = B16_SMALL.replace(batch=4, K=8)
    model = oracle_model_from_gpu(cfg)
    tokens = helpers.draft_chain(cfg, model)
    wl = GpuWorkload(cfg)
    rs = helpers.row_scale(cfg)
    strict = wl.verify(tokens, rs, theta=2.0, W=6)
    std = np.array([O.s_standard(O.match_indicator(tokens[b, 1:], strict["argmax"][b])) for b in range(cfg.batch)])
    assert np.array_equal(strict["accept_len"] + 1, std)
    # re-running on the same cache rewrites the same rows: results are reproducible bit for bit
    again = wl.verify(tokens, rs, theta=2.0, W=6)
    for k in strict:
        assert np.array_equal(strict[k], again[k]), k
    loose = wl.verify(tokens, rs, theta=0.0, W=0)
    assert np.all(loose["accept_len"] == cfg.K)
    assert np.array_equal(loose["next_token"], loose["argmax"][:, -1])


def test_causality_on_device():
    """Changing drafts from position 3 on leaves the statistics of rows 0..2 untouched."""
    cfg = B16_SMALL
    wl = GpuWorkload(cfg)
    rng = np.random.default_rng(0)
    tokens = rng.integers(0, cfg.vocab, size=(cfg.batch, cfg.K + 1)).astype(np.int32)
    a = wl.verify(tokens, None)
    t2 = tokens.copy()
    t2[:, 3:] = (t2[:, 3:] + 1) % cfg.vocab
    b = wl.verify(t2, None)
    for k in ("argmax", "h_norm", "p_top1", "lse"):
        assert np.array_equal(a[k][:, :3], b[k][:, :3]), k
    assert not np.array_equal(a["lse"][:, 3:], b["lse"][:, 3:])


ATTENTION_STAGE_CASES = [
    # (query heads, KV heads, K, query tiles per workgroup; 0 = automatic) -> rows per KV head
    (16, 2, 8, 0),    # 72 rows, 3 tiles: a wave owns (tile, half of a stage's keys)
    (8, 2, 8, 0),     # 36 rows, 2 tiles
    (16, 2, 16, 0),   # 136 rows, 5 tiles: a wave owns a whole tile
    (16, 2, 20, 0),   # 168 rows, 6 tiles
    (16, 2, 23, 0),   # 192 rows, 6 full tiles
    (16, 2, 24, 0),   # 200 rows, 7 tiles
    (32, 2, 19, 0),   # 320 rows: two query blocks of 5 tiles that stream the same keys
    (16, 2, 16, 2),   # 136 rows as three query blocks of 2, 2 and 1 tiles
    (16, 2, 30, 0),   # 248 rows, 8 tiles, the longest block one workgroup holds
]


@pytest.mark.parametrize("phase", [1, 2])
@pytest.mark.parametrize("hq,hkv,K,block_tiles", ATTENTION_STAGE_CASES)
def test_attention_stage_bf16(hq, hkv, K, block_tiles, phase):
    """fly_attention alone on seeded q and cache: one rounding (the bf16 output)
    separates the two sides, so elements agree to one bf16 ulp and almost all
    are identical.  Covers ragged lengths, a cache that ends mid-tile, several
    cache splits, every way the query tiles are dealt to waves and workgroups, and both
    points of a step at which a wave requests its share of the next cache stage."""
    from paper_2511_22972_amd import binding as fb
    cfg = synth.CONFIGS["c3_70b"].replace(n_layers=1, n_q_heads=hq, n_kv_heads=hkv, batch=3, K=K,
                                          kv_len=1000)
    kv_lens = [1000 - K, 517, 3]
    R = cfg.K + 1
    desc = fb.make_desc(cfg)
    kv = fb.KVCache(desc, cfg.batch, 1024)
    k, v = synth.make_kv_prefix(cfg.replace(kv_len=1024), 0, "cuda")    # rows beyond kv_len stand for the new rows
    kv.load_prefix(0, k, v)
    kv.set_lengths(kv_lens)
    q = synth.hash_normal(cfg.seed, 310, (cfg.M, cfg.q_dim), 2.0, torch.bfloat16, "cuda")
    o = torch.zeros_like(q)
    fb.fly_set_tuning("attn_block_tiles", block_tiles)
    fb.fly_set_tuning("attn_phase", phase)
    try:
        ws = fb.alloc_workspace(fb.fly_workspace_bytes(desc, cfg.batch, cfg.K, max(kv_lens)))
        fb.fly_attention(desc, kv, 0, q, o, cfg.batch, cfg.K, ws)
    finally:
        fb.fly_set_tuning("attn_block_tiles", 0)
        fb.fly_set_tuning("attn_phase", 0)
    torch.cuda.synchronize()
    got = o.float().cpu().double().view(cfg.batch, R, cfg.n_q_heads, cfg.head_dim)
    num = O.Numerics("bf16")
    for b, L in enumerate(kv_lens):
        qb = q.float().cpu().double().view(cfg.batch, R, cfg.n_q_heads, cfg.head_dim)[b]
        ref = num.act(O.attention_one_sequence(qb, k[b, :L + R].cpu().double(), v[b, :L + R].cpu().double(), L, num))
        diff = (got[b] - ref).abs()
        # Outputs are bf16: most elements are identical.  A probability whose
        # fp32 and fp64 evaluations straddle a bf16 rounding boundary moves a
        # whole output row by about 2^-8 * p_j / sum(p) * |v_j|, so the bound is
        # absolute (values are O(1)), not one ulp of each element.
        assert diff.max().item() <= 4e-3, (b, diff.max())
        assert (diff == 0).double().mean().item() > 0.97, (b, (diff == 0).double().mean().item())


def test_gateup_swiglu_stage_bf16():
    """The fused gate/up GEMM + SwiGLU alone (ragged M, F not a multiple of the block)."""
    from paper_2511_22972_amd import binding as fb
    for M, d, F in ((36, 512, 1056), (9, 256, 512), (100, 128, 16 * 37), (80, 96, 272)):
        # 81..128 rows default to the kernel with 32-row tiles: keep its nine-tile sibling covered
        fb.fly_set_tuning("gemm_wide", 1 if M > 80 else 0)
        x = synth.hash_normal(5, 320, (M, d), 1.0, torch.bfloat16, "cuda")
        wg = synth.hash_normal(5, 321, (d, F), 0.05, torch.bfloat16, "cuda")
        wu = synth.hash_normal(5, 322, (d, F), 0.05, torch.bfloat16, "cuda")
        wp = torch.empty(d * 2 * F, dtype=torch.bfloat16, device="cuda")
        fb.fly_pack_weight(wg, wp, 2 * F, 0, 2)
        fb.fly_pack_weight(wu, wp, 2 * F, 1, 2)
        a = torch.zeros(M, F, dtype=torch.bfloat16, device="cuda")
        fb.fly_gateup_swiglu(x, wp, a)
        torch.cuda.synchronize()
        xd = x.float().cpu().double()
        ref = O.round_to_bf16(O.silu(xd @ wg.float().cpu().double()) * (xd @ wu.float().cpu().double()))
        diff = (a.float().cpu().double() - ref).abs()
        assert torch.all(diff <= ref.abs() * 2.0 ** -7 + 1e-7), (M, d, F, diff.max())
        assert (diff == 0).double().mean().item() > 0.99


@pytest.mark.gpu
def test_gateup_swiglu_stage_bf16_many_rows():
    """The same stage above 128 rows, where the LDS-tiled GEMM takes over."""
    from paper_2511_22972_amd import binding as fb
    cases = [(M, d, F, 0) for M, d, F in ((200, 128, 16 * 37), (389, 256, 1056), (145, 32, 16), (1088, 64, 512))]
    cases += [(389, 256, 1056, shape) for shape in (2, 3, 4, 6)]
    cases += [(M, 256, 1056, shape) for M in (145, 200) for shape in (2, 3)]  # also where "wide" is the default
    cases += [(389, 256, 1056, -shape) for shape in (2, 6)]  # negative: every wave requests its loads first
    for M, d, F, shape in cases:
        fb.fly_set_tuning("gemm_tiled", abs(shape))
        fb.fly_set_tuning("tiled_phase", 2 if shape < 0 else 0)
        x = synth.hash_normal(6, 320, (M, d), 1.0, torch.bfloat16, "cuda")
        wg = synth.hash_normal(6, 321, (d, F), 0.05, torch.bfloat16, "cuda")
        wu = synth.hash_normal(6, 322, (d, F), 0.05, torch.bfloat16, "cuda")
        wp = torch.empty(d * 2 * F, dtype=torch.bfloat16, device="cuda")
        fb.fly_pack_weight(wg, wp, 2 * F, 0, 2)
        fb.fly_pack_weight(wu, wp, 2 * F, 1, 2)
        a = torch.zeros(M, F, dtype=torch.bfloat16, device="cuda")
        try:
            fb.fly_gateup_swiglu(x, wp, a)
        finally:
            fb.fly_set_tuning("gemm_tiled", 0)
            fb.fly_set_tuning("tiled_phase", 0)
        torch.cuda.synchronize()
        xd = x.float().cpu().double()
        ref = O.round_to_bf16(O.silu(xd @ wg.float().cpu().double()) * (xd @ wu.float().cpu().double()))
        diff = (a.float().cpu().double() - ref).abs()
        assert torch.all(diff <= ref.abs() * 2.0 ** -7 + 1e-7), (M, d, F, shape, diff.max())
        assert (diff == 0).double().mean().item() > 0.99


@pytest.mark.gpu
@pytest.mark.parametrize("phase", [1, 2])
def test_gateup_swiglu_stage_bf16_wide_rows(phase):
    """The same stage at 129..256 rows (weight-streaming kernel with 32 x 32 tiles), every
    row-tile count, ragged rows / columns / k-tiles; with half of the waves requesting their
    loads after multiplying (phase 1) and with every wave requesting first (phase 2)."""
    from paper_2511_22972_amd import binding as fb
    cases = [(129, 256, 1056, 0), (160, 96, 16 * 37, 5), (161, 544, 512, 6), (192, 32, 16, 6),
             (200, 320, 2048 + 16, 0), (256, 64, 144, 8), (100, 160, 272, 5), (150, 1024, 256, 8),
             (81, 256, 1056, 0), (96, 96, 16 * 37, 3), (97, 544, 512, 0), (128, 320, 272, 4), (50, 64, 144, 3)]
    for M, d, F, tiles in cases:
        fb.fly_set_tuning("gemm_wide", tiles)
        fb.fly_set_tuning("wide_phase", phase)
        x = synth.hash_normal(8, 320, (M, d), 1.0, torch.bfloat16, "cuda")
        wg = synth.hash_normal(8, 321, (d, F), 0.05, torch.bfloat16, "cuda")
        wu = synth.hash_normal(8, 322, (d, F), 0.05, torch.bfloat16, "cuda")
        wp = torch.empty(d * 2 * F, dtype=torch.bfloat16, device="cuda")
        fb.fly_pack_weight(wg, wp, 2 * F, 0, 2)
        fb.fly_pack_weight(wu, wp, 2 * F, 1, 2)
        a = torch.zeros(M, F, dtype=torch.bfloat16, device="cuda")
        try:
            fb.fly_gateup_swiglu(x, wp, a)
        finally:
            fb.fly_set_tuning("gemm_wide", 0)
            fb.fly_set_tuning("wide_phase", 0)
        torch.cuda.synchronize()
        xd = x.float().cpu().double()
        ref = O.round_to_bf16(O.silu(xd @ wg.float().cpu().double()) * (xd @ wu.float().cpu().double()))
        diff = (a.float().cpu().double() - ref).abs()
        assert torch.all(diff <= ref.abs() * 2.0 ** -7 + 1e-7), (M, d, F, tiles, diff.max())
        assert (diff == 0).double().mean().item() > 0.99


@pytest.mark.gpu
@pytest.mark.parametrize("phase", [1, 2])
def test_projection_partials_bf16_wide_rows(phase):
    """Split-K projection at 129..256 rows: the partial sums add up to x W (ragged last split,
    more splits asked for than there are chunks; both orders of loads and multiplies)."""
    from paper_2511_22972_amd import binding as fb
    cases = [(136, 4096, 512, 0, 0), (200, 2048, 528, 0, 0), (256, 1056, 1040, 8, 0), (160, 2080, 256, 5, 5),
             (192, 96, 16, 6, 0), (129, 3072, 272, 0, 7), (150, 1024, 256, 6, 16),
             (100, 4096, 512, 0, 0), (96, 2080, 528, 3, 3), (128, 1056, 272, 4, 0), (82, 96, 16, 0, 0)]
    for M, Kd, N, tiles, force_splits in cases:
        fb.fly_set_tuning("gemm_wide", tiles)
        fb.fly_set_tuning("gemm_splits", force_splits)
        fb.fly_set_tuning("wide_phase", phase)
        x = synth.hash_normal(9, 330, (M, Kd), 1.0, torch.bfloat16, "cuda")
        w = synth.hash_normal(9, 331, (Kd, N), 0.05, torch.bfloat16, "cuda")
        wp = torch.empty(Kd * N, dtype=torch.bfloat16, device="cuda")
        fb.fly_pack_weight(w, wp, N)
        partial = torch.full((16 * M * N,), float("nan"), dtype=torch.float32, device="cuda")
        try:
            splits = fb.fly_proj_partial(x, wp, partial, N)
        finally:
            fb.fly_set_tuning("gemm_wide", 0)
            fb.fly_set_tuning("gemm_splits", 0)
            fb.fly_set_tuning("wide_phase", 0)
        torch.cuda.synchronize()
        assert 1 <= splits <= 16
        got = partial[: splits * M * N].view(splits, M, N).double().sum(0).cpu()
        ref = x.float().cpu().double() @ w.float().cpu().double()
        scale = ref.abs().max().item()
        assert torch.isfinite(got).all()
        assert (got - ref).abs().max().item() <= 2e-5 * scale + 1e-6, (M, Kd, N, tiles, splits)


@pytest.mark.gpu
def test_projection_partials_bf16():
    """Split-K projection GEMM alone, both kernels: the partial sums add up to x W."""
    from paper_2511_22972_amd import binding as fb
    # (the 100-row case runs with "gemm_wide" = 1 below: the nine-tile sibling of the default kernel)
    cases = [(M, Kd, N, 0) for M, Kd, N in ((36, 1024, 272), (100, 4096, 512), (200, 2048, 528),
                                            (389, 512, 1040), (1088, 1024, 256), (145, 32, 16))]
    cases += [(389, 2048, 528, shape) for shape in (2, 3, 4, 6)]
    for M, Kd, N, shape in cases:
        fb.fly_set_tuning("gemm_tiled", shape)
        fb.fly_set_tuning("gemm_wide", 1 if 80 < M <= 128 else 0)
        x = synth.hash_normal(7, 330, (M, Kd), 1.0, torch.bfloat16, "cuda")
        w = synth.hash_normal(7, 331, (Kd, N), 0.05, torch.bfloat16, "cuda")
        wp = torch.empty(Kd * N, dtype=torch.bfloat16, device="cuda")
        fb.fly_pack_weight(w, wp, N)
        partial = torch.full((16 * M * N,), float("nan"), dtype=torch.float32, device="cuda")
        try:
            splits = fb.fly_proj_partial(x, wp, partial, N)
        finally:
            fb.fly_set_tuning("gemm_tiled", 0)
            fb.fly_set_tuning("gemm_wide", 0)
        torch.cuda.synchronize()
        assert 1 <= splits <= 16
        got = partial[: splits * M * N].view(splits, M, N).double().sum(0).cpu()
        ref = x.float().cpu().double() @ w.float().cpu().double()
        scale = ref.abs().max().item()
        assert torch.isfinite(got).all()
        assert (got - ref).abs().max().item() <= 2e-5 * scale + 1e-6, (M, Kd, N, shape, splits)


def test_verify_block_replays_from_a_captured_graph():
    """The step enqueues kernels and device copies only (no allocation, no
    synchronisation), so a caller may capture it in a HIP graph.  Every replay,
    with eager work of the program between the replays, gives bit for bit the
    eager result."""
    from paper_2511_22972_amd import binding as fb
    for cfg in (B16_WIDE, C1.replace(batch=2, logit_gain=12.0, window=2)):
        wl = GpuWorkload(cfg)
        tokens = synth.hash_tokens(cfg.seed, 970, cfg.batch * (cfg.K + 1), cfg.vocab, "cuda").view(
            cfg.batch, cfg.K + 1).to(torch.int32)
        rs = helpers.row_scale(cfg).cuda()
        eager = wl.verify(tokens.cpu().numpy(), rs)
        out = fb.VerifyOutputs(cfg.batch, cfg.K, cfg.d, want_hidden=True)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):    # warm-up on the capture stream, as graph capture asks for
            fb.fly_verify_block(wl.model, wl.kv, tokens, rs, cfg.theta, cfg.window, out, wl.ws)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            fb.fly_verify_block(wl.model, wl.kv, tokens, rs, cfg.theta, cfg.window, out, wl.ws)
        for rep in range(3):
            for name in ("accept_len", "next_token", "kv_len_out", "n_loose", "argmax"):
                getattr(out, name).fill_(-7)
            for name in ("h_norm", "p_top1", "lse", "hidden"):
                getattr(out, name).fill_(float("nan"))
            wl.ws.fill_(0x5A)                      # the workspace carries nothing between calls
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            for name in ("accept_len", "next_token", "kv_len_out", "n_loose", "argmax", "h_norm", "p_top1", "lse"):
                assert np.array_equal(getattr(out, name).cpu().numpy(), eager[name]), (cfg.name, rep, name)
            assert np.array_equal(out.hidden.cpu().numpy(), eager["hidden"]), (cfg.name, rep)
