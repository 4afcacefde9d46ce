"""The drawn target token (temperature > 0) on the device against the CPU oracle.

Both sides implement the same counter-based generator and the same Gumbel-max
construction; the device fuses the draw into the LM-head epilogues of all four
GEMM kernels, so every kernel gets its own cases.  A drawn token may differ only
where the two largest perturbed logits are closer than the stated bound.
"""
import math

import numpy as np
import pytest
import torch

import synth
from oracle import fly_oracle as O
from tests import helpers
from tests.gpu_harness import GpuWorkload, check_own_rule, verify_sampled

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fb():
    from paper_2511_22972_amd import binding
    return binding


def sample_case(fb, M, d, V, dtype, seed, offset, data_seed=1, hidden_std=4.0):
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    hidden = synth.hash_normal(data_seed, 201, (M, d), hidden_std, tdt, "cuda")
    w = synth.hash_normal(data_seed, 202, (d, V), 0.02, tdt, "cuda")
    code = fb.dtype_code(dtype)
    wp = torch.empty(fb.fly_packed_weight_bytes(d, V, code) // w.element_size(), dtype=tdt, device="cuda")
    fb.fly_pack_weight(w, wp, V)
    rs = torch.exp(torch.linspace(math.log(0.1), math.log(10.0), M)).to("cuda", torch.float32)
    i32 = lambda: torch.zeros(M, dtype=torch.int32, device="cuda")
    f32 = lambda: torch.zeros(M, dtype=torch.float32, device="cuda")
    ws = fb.alloc_workspace(fb.fly_lmhead_workspace_bytes(M, d, V, code))
    plain = {"argmax": i32(), "p_top1": f32(), "h": f32(), "lse": f32()}
    fb.fly_lmhead_entropy_argmax(hidden, wp, rs, V, plain["argmax"], plain["p_top1"], plain["h"], plain["lse"], ws)
    got = {"sampled": i32(), "argmax": i32(), "p_top1": f32(), "h": f32(), "lse": f32()}
    fb.fly_lmhead_entropy_sample(hidden, wp, rs, V, seed, offset, got["sampled"], got["argmax"], got["p_top1"],
                                 got["h"], got["lse"], ws)
    torch.cuda.synchronize()
    got = {k: v.cpu().numpy() for k, v in got.items()}
    plain = {k: v.cpu().numpy() for k, v in plain.items()}
    logits = O.lm_head_logits(hidden.cpu().double(), w.cpu().double(), rs.cpu()).numpy()
    ref = O.sample_rows(logits, seed, offset)
    return got, plain, ref


def check_sample(got, plain, ref, tol=1e-3):
    # the other statistics are those of the entry point without the draw, bit for bit
    for k in ("argmax", "p_top1", "h", "lse"):
        assert np.array_equal(got[k], plain[k]), k
    near_tie = ref["margin"] < tol
    same = got["sampled"] == ref["token"]
    assert np.all(same | near_tie), np.argwhere(~same & ~near_tie)
    assert (~near_tie).sum() > 0.9 * len(near_tie)
    # the draw is not the argmax everywhere (rows are hot and cold), nor nowhere
    assert 0 < (got["sampled"] != got["argmax"]).sum() < len(same) or len(same) < 4


SEED, OFFSET = (0x9E3779B9 << 32) | 0x7F4A7C15, (3 << 32) | 11


@pytest.mark.parametrize("M,d,V", [(5, 256, 8192), (9, 64, 48), (17, 688, 1040)])
def test_sample_f32(fb, M, d, V):
    check_sample(*sample_case(fb, M, d, V, "f32", SEED, OFFSET))


@pytest.mark.parametrize("M,d,V", [(9, 256, 8192), (36, 1024, 4112), (50, 512, 16 * 131), (80, 128, 1024),
                                   (1, 32, 16)])
def test_sample_bf16_streaming_kernel(fb, M, d, V):
    check_sample(*sample_case(fb, M, d, V, "bf16", SEED, OFFSET))


def test_sample_bf16_nine_tile_streaming_kernel(fb):
    fb.fly_set_tuning("gemm_wide", 1)
    try:
        for M, d, V in ((100, 256, 2048 + 48), (128, 96, 272)):
            check_sample(*sample_case(fb, M, d, V, "bf16", SEED, OFFSET, data_seed=7))
    finally:
        fb.fly_set_tuning("gemm_wide", 0)


@pytest.mark.parametrize("M,d,V,tiles", [(129, 256, 2048 + 48, 0), (160, 96, 16 * 131, 5), (161, 544, 1040, 6),
                                         (256, 64, 272, 8), (96, 96, 16 * 131, 3), (128, 544, 1040, 4)])
@pytest.mark.parametrize("phase", [1, 2])
def test_sample_bf16_wide_kernel(fb, M, d, V, tiles, phase):
    fb.fly_set_tuning("gemm_wide", tiles)
    fb.fly_set_tuning("wide_phase", phase)
    try:
        res = sample_case(fb, M, d, V, "bf16", SEED, OFFSET, data_seed=5)
    finally:
        fb.fly_set_tuning("gemm_wide", 0)
        fb.fly_set_tuning("wide_phase", 0)
    check_sample(*res)


@pytest.mark.parametrize("M,d,V", [(300, 544, 16 * 131), (1088, 512, 4096), (385, 96, 272)])
def test_sample_bf16_tiled_kernel(fb, M, d, V):
    check_sample(*sample_case(fb, M, d, V, "bf16", SEED, OFFSET))
    for wm, phase in ((2, 0), (3, 0), (4, 0), (6, 0), (4, 2)):
        fb.fly_set_tuning("gemm_tiled", wm)
        fb.fly_set_tuning("tiled_phase", phase)
        try:
            res = sample_case(fb, M, d, V, "bf16", SEED, OFFSET, data_seed=3)
        finally:
            fb.fly_set_tuning("gemm_tiled", 0)
            fb.fly_set_tuning("tiled_phase", 0)
        check_sample(*res)


@pytest.mark.parametrize("M,d,V,dtype", [(5, 256, 8192, "f32"), (36, 1024, 4112, "bf16"), (136, 256, 2048 + 48, "bf16"),
                                         (300, 544, 16 * 131, "bf16")])
def test_lmhead_does_not_read_stale_workspace(fb, M, d, V, dtype):
    """Every (row, part) record of the statistics and of the picks is written before the merge reads
    it: the outputs do not change when the workspace is filled with NaN bytes or huge values first."""
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    hidden = synth.hash_normal(2, 201, (M, d), 4.0, tdt, "cuda")
    w = synth.hash_normal(2, 202, (d, V), 0.02, tdt, "cuda")
    code = fb.dtype_code(dtype)
    wp = torch.empty(fb.fly_packed_weight_bytes(d, V, code) // w.element_size(), dtype=tdt, device="cuda")
    fb.fly_pack_weight(w, wp, V)
    ws = fb.alloc_workspace(fb.fly_lmhead_workspace_bytes(M, d, V, code))

    def run():
        outs = [torch.zeros(M, dtype=torch.int32, device="cuda") for _ in range(2)] + \
               [torch.zeros(M, dtype=torch.float32, device="cuda") for _ in range(3)]
        fb.fly_lmhead_entropy_sample(hidden, wp, None, V, 7, 3, outs[0], outs[1], outs[2], outs[3], outs[4], ws)
        torch.cuda.synchronize()
        return outs

    ws.zero_()
    ref = run()
    for byte in (0xFF, 0x7F):
        ws.fill_(byte)
        for a, b in zip(run(), ref):
            assert torch.equal(a, b), byte


def test_seed_and_offset_select_the_draw(fb):
    M, d, V = 64, 64, 1024
    a, _, _ = sample_case(fb, M, d, V, "bf16", 5, 0, hidden_std=0.5)
    again, _, _ = sample_case(fb, M, d, V, "bf16", 5, 0, hidden_std=0.5)
    b, _, ref_b = sample_case(fb, M, d, V, "bf16", 5, 1, hidden_std=0.5)
    c, _, _ = sample_case(fb, M, d, V, "bf16", 6, 0, hidden_std=0.5)
    assert np.array_equal(a["sampled"], again["sampled"])
    assert (a["sampled"] != b["sampled"]).sum() > M // 4
    assert (a["sampled"] != c["sampled"]).sum() > M // 4
    # high words of seed and offset reach the generator too
    hi, _, ref_hi = sample_case(fb, M, d, V, "bf16", 5 | (1 << 40), 1 | (1 << 35), hidden_std=0.5)
    assert (hi["sampled"] != b["sampled"]).sum() > M // 4
    assert np.all((hi["sampled"] == ref_hi["token"]) | (ref_hi["margin"] < 1e-3))


def test_device_draws_follow_the_softmax(fb):
    """Many rows with the same hidden state: the drawn tokens' frequencies follow that row's softmax."""
    from scipy import stats
    M, d, V = 4096, 32, 16
    hidden = synth.hash_normal(3, 201, (1, d), 2.0, torch.float32, "cuda").expand(M, d).contiguous()
    w = synth.hash_normal(3, 202, (d, V), 0.2, torch.float32, "cuda")
    code = fb.dtype_code("f32")
    wp = torch.empty(fb.fly_packed_weight_bytes(d, V, code) // 4, dtype=torch.float32, device="cuda")
    fb.fly_pack_weight(w, wp, V)
    i32 = lambda: torch.zeros(M, dtype=torch.int32, device="cuda")
    f32 = lambda: torch.zeros(M, dtype=torch.float32, device="cuda")
    ws = fb.alloc_workspace(fb.fly_lmhead_workspace_bytes(M, d, V, code))
    sampled = i32()
    fb.fly_lmhead_entropy_sample(hidden, wp, None, V, 17, 4, sampled, i32(), f32(), f32(), None, ws)
    torch.cuda.synchronize()
    logits = (hidden[0].cpu().double() @ w.cpu().double()).numpy()
    p = np.exp(logits - logits.max())
    p /= p.sum()
    counts = np.bincount(sampled.cpu().numpy(), minlength=V)
    keep = p * M >= 5
    assert keep.sum() >= 4
    obs = np.append(counts[keep], counts[~keep].sum())
    exp = np.append(p[keep] * M, p[~keep].sum() * M)
    if exp[-1] < 1e-9:
        obs, exp = obs[:-1], exp[:-1]
    assert stats.chisquare(obs, exp * obs.sum() / exp.sum()).pvalue > 1e-3


C1 = synth.CONFIGS["c1_tiny"]


@pytest.mark.parametrize("W", [0, 1])
def test_verify_sampled_f32(W):
    """The whole step with drawn target tokens, tiny fp32 model, several sequences."""
    cfg = C1.replace(batch=6, logit_gain=12.0, window=W)
    model = helpers.oracle_model(cfg, device="cuda")
    tokens = helpers.draft_chain(cfg, model)
    ora = helpers.oracle_verify(cfg, model, tokens, sample=(SEED, OFFSET))
    wl = GpuWorkload(cfg)
    gpu = verify_sampled(wl, tokens, helpers.row_scale(cfg), SEED, OFFSET)
    plain = wl.verify(tokens, helpers.row_scale(cfg), want_hidden=False)
    for k in ("argmax", "h_norm", "p_top1", "lse"):
        assert np.array_equal(gpu[k], plain[k]), k
    near = ora["sample_margin"] < 1e-3
    same = gpu["sampled"] == ora["sampled"]
    assert np.all(same | near)
    assert (gpu["sampled"] != gpu["argmax"]).any()
    # the rule applied to the device's own drawn tokens and entropies reproduces its decision
    own = O.accept_block(tokens[:, 1:], gpu["sampled"], gpu["h_norm"], cfg.theta, W)
    for k in ("accept_len", "next_token", "n_loose"):
        assert np.array_equal(gpu[k], own[k]), k
    amb = near | (np.abs(ora["h"] - cfg.theta) < 1e-3)
    clean = ~amb[:, :-1].any(axis=1) & same.all(axis=1)
    assert clean.sum() >= 3
    for k in ("accept_len", "next_token", "n_loose"):
        assert np.array_equal(gpu[k][clean], ora[k][clean]), k
    assert np.array_equal(gpu["kv_len_out"], cfg.kv_len + gpu["accept_len"] + 1)


def test_verify_sampled_bf16():
    """bf16 model.  Free-running, the logits of the two sides differ by up to the stated 2e-2, so a
    drawn token is compared only where the perturbed margin is above twice that.  Teacher-forced (the
    oracle's final norm, LM head, draw and rule on the device's own residual stream) the drawn
    tokens and the accept outputs must agree outside the 1e-3 exclusions."""
    cfg = synth.CONFIGS["c2_8b"].replace(
        name="bf16_sampled", n_layers=2, d=256, n_q_heads=4, n_kv_heads=2, ffn=512, vocab=2048 + 16,
        batch=5, K=8, kv_len=90, weight_std=0.05, temperatures=(0.3, 1.0, 3.0), window=2)
    model = helpers.oracle_model(cfg, device="cuda")
    tokens = helpers.draft_chain(cfg, model)
    ora = helpers.oracle_verify(cfg, model, tokens, sample=(SEED, OFFSET))
    wl = GpuWorkload(cfg)
    gpu = verify_sampled(wl, tokens, helpers.row_scale(cfg), SEED, OFFSET)
    check_own_rule(gpu, tokens, cfg.theta, cfg.window, O.accept_block, target_key="sampled")
    free_near = ora["sample_margin"] < 4e-2
    assert np.all((gpu["sampled"] == ora["sampled"]) | free_near)
    tail = helpers.oracle_tail(cfg, gpu["hidden"], tokens, model["g_final"], model["w_lm"], sample=(SEED, OFFSET))
    near = tail["sample_margin"] < 1e-3
    same = gpu["sampled"] == tail["sampled"]
    assert np.all(same | near), np.argwhere(~same & ~near)
    assert (gpu["sampled"] != gpu["argmax"]).any()
    amb = near | (tail["margin"] < 1e-3) | (np.abs(tail["h"] - cfg.theta) < 1e-3)
    clean = ~amb.any(axis=1)
    assert clean.sum() >= 3
    assert np.array_equal(gpu["argmax"][~(tail["margin"] < 1e-3)], tail["argmax"][~(tail["margin"] < 1e-3)])
    for k in ("accept_len", "next_token", "n_loose"):
        assert np.array_equal(gpu[k][clean], tail[k][clean]), k
    for k, r in (("lse", "lse"), ("h_norm", "h"), ("p_top1", "p_top1")):
        assert np.abs(gpu[k] - tail[r]).max() < 2e-3, k
