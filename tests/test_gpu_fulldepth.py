"""Teacher-forced parity at the full depth and width of the benchmark workloads
(the 8B, 70B and 405B-slice shapes, in the launch configuration bench.py times).

A free-running comparison of a deep bf16 model says little: one bf16 rounding
that falls the other way in fp32 than in fp64 moves a hidden state, and after
tens of layers the two sides have decorrelated by ordinary bf16 noise.  So the
oracle is fed the DEVICE's own intermediate results, stage by stage:

  * the device runs the whole model one layer at a time (fly_decoder_layers
    (l, l+1)); for every layer the oracle's decoder_layer gets the device's
    layer input and its output is compared with the device's layer output
    (residual stream relative to its rms, and the difference must be spread like
    rounding noise: no row and no block of 128 columns carries much more of it
    than the rest; the rows appended to the KV cache);
  * the chained per-layer run must equal the one-call step bit for bit;
  * the oracle's final norm, LM head, row statistics (Eq. 1, Eq. 5) and
    acceptance rule (Eqs. 2-11; Algorithm 1 steps 2-4) are applied to the
    device's residual stream after the last layer: argmax, accepted length and
    correction token must agree bit for bit outside the 1e-3 exclusions.

The drafts are built with the library itself (K+1 passes, draft i = the
device's target token w.p. p_match, else a uniform token) -- they are inputs,
the same for both sides.

With FLY_FREE_RUNNING=1 in the environment the oracle also runs its own chain
from the embedding on and the test REPORTS (never asserts) every integer
disagreement of the free-running run beside its top-2 margin and |h - theta|;
the 8B shape always does.
"""
import os
import sys
import time

import numpy as np
import pytest
import torch

import synth
from oracle import fly_oracle as O
from tests import helpers
from tests.gpu_harness import GpuWorkload, check_own_rule, compare_tail

pytestmark = pytest.mark.gpu


def device_draft_chain(wl, cfg, rs):
    """tokens [B, K+1] = y_{-1}, then draft i = the device's target token at position i with
    probability p_match, else a uniform token (K passes of the library; causality fixes position
    i's target once the tokens before it are fixed)."""
    first = synth.make_first_tokens(cfg).numpy()
    u, alt, _ = synth.make_draft_draws(cfg)
    u, alt = u.numpy(), alt.numpy()
    tokens = np.zeros((cfg.batch, cfg.K + 1), dtype=np.int32)
    tokens[:, 0] = first
    for i in range(1, cfg.K + 1):
        y = wl.verify(tokens, rs, want_hidden=False)["argmax"][:, i - 1]
        tokens[:, i] = np.where(u[:, i - 1] < cfg.p_match, y, alt[:, i - 1])
    return tokens


def teacher_forced_depth(cfg, capsys, layer_rms_tol, layer_max_tol, min_clean, free_running, mixed=None):
    def say(*a):
        with capsys.disabled():
            print(*a, flush=True)

    t0 = time.time()
    B, K, R, d, L = cfg.batch, cfg.K, cfg.K + 1, cfg.d, cfg.kv_len
    wl = GpuWorkload(cfg)
    fb = wl.fb
    rs = helpers.row_scale(cfg)
    tokens = device_draft_chain(wl, cfg, rs)
    gpu = wl.verify(tokens, rs)
    say(f"\n[{cfg.name}] model loaded and drafts chained in {time.time() - t0:.0f}s; "
        f"teacher-forced comparison of {cfg.n_layers} layers")

    embed = synth.make_weight(cfg, "embed", -1, "cuda")
    x = embed[torch.as_tensor(tokens.reshape(-1).astype(np.int64), device="cuda")].float().contiguous()
    x_free = x.cpu().double().view(B, R, d).clone() if free_running else None
    num = O.Numerics(cfg.dtype)
    worst = {"rms": 0.0, "max": 0.0, "kv_flips": 0.0, "free_rms": 0.0, "row": 0.0, "blk": 0.0}
    for l in range(cfg.n_layers):
        x_in = x.cpu().double().view(B, R, d)
        fb.fly_decoder_layers(wl.model, wl.kv, x, l, l + 1, B, K, wl.ws)
        torch.cuda.synchronize()
        got = x.cpu().double().view(B, R, d)
        w = helpers.oracle_layer_weights(cfg, l, "cuda")
        kp, vp = (t.to("cpu", torch.float64) for t in synth.make_kv_prefix(cfg, l, "cuda"))
        kc, vc = wl.kv.k[l], wl.kv.v[l]
        for b in range(B):
            ref, k_new, v_new = O.decoder_layer(x_in[b], w, kp[b], vp[b], cfg.n_q_heads, cfg.n_kv_heads,
                                                cfg.head_dim, cfg.rope_theta, cfg.rms_eps, num)
            scale = ref.pow(2).mean().sqrt().item()
            err = (got[b] - ref).abs()
            rel_rms, rel_max = err.pow(2).mean().sqrt().item() / scale, err.max().item() / scale
            worst["rms"], worst["max"] = max(worst["rms"], rel_rms), max(worst["max"], rel_max)
            assert rel_rms < layer_rms_tol and rel_max < layer_max_tol, (cfg.name, "layer", l, "sequence", b,
                                                                         rel_rms, rel_max)
            # ... and it must look like rounding noise everywhere: no row and no block of 128 columns
            # carries much more of it than the rest (a wrong tile, head or split would)
            e2 = (got[b] - ref).pow(2)
            overall = e2.mean().sqrt().item()
            row_ratio = e2.mean(dim=1).sqrt().max().item() / overall
            blk_ratio = e2.view(R, -1, 128).mean(dim=(0, 2)).sqrt().max().item() / overall
            worst["row"], worst["blk"] = max(worst["row"], row_ratio), max(worst["blk"], blk_ratio)
            # (observed over all layers: rows up to 3.0x, blocks up to 1.16x; two weight rows swapped inside
            # one 128-column block of the down projection, planted in an fp32 copy of the oracle's layer on
            # the CPU, move the overall error from 2.47e-3 to 2.55e-3 of the rms but that block to 2.2x)
            assert row_ratio < 4.5 and blk_ratio < 1.5, (cfg.name, "layer", l, "sequence", b, row_ratio, blk_ratio)
            gk = kc[b, :, L:L + R, :].float().cpu().double().permute(1, 0, 2)
            gv = vc[b, :, :, L:L + R].float().cpu().double().permute(2, 0, 1)
            for name, g_t, r_t in (("k", gk, k_new), ("v", gv, v_new)):
                diff = (g_t - r_t).abs()
                # bf16 values: identical, or one ulp apart where the fp32 and the fp64 evaluation
                # straddle a rounding boundary.  Where that happens to an element of the normalised
                # input row (about 2e-3 of its d elements), every q/k/v element of the row moves by
                # ulp(xn_i) W[i, :] ~ 0.004 * 0.02; the sum over those elements has rms
                # 4e-6 sqrt(d), so elements near zero may differ by a few times that in absolute terms
                assert torch.all(diff <= r_t.abs() * 2.0 ** -7 + 3e-5 * d ** 0.5), (cfg.name, name, l, b, diff.max())
                flips = (diff != 0).double().mean().item()
                worst["kv_flips"] = max(worst["kv_flips"], flips)
                assert flips < 0.05, (cfg.name, name, l, b, flips)
            if free_running:
                x_free[b], _, _ = O.decoder_layer(x_free[b], w, kp[b], vp[b], cfg.n_q_heads, cfg.n_kv_heads,
                                                  cfg.head_dim, cfg.rope_theta, cfg.rms_eps, num)
        if free_running:
            fr = ((got - x_free).pow(2).mean().sqrt() / x_free.pow(2).mean().sqrt()).item()
            worst["free_rms"] = max(worst["free_rms"], fr)
        del w, kp, vp
        if l % 4 == 3 or l == cfg.n_layers - 1:
            say(f"[{cfg.name}] layer {l + 1}/{cfg.n_layers}  worst so far: layer error / rms "
                f"{worst['rms']:.2e} (max {worst['max']:.2e}; noisiest row {worst['row']:.2f}x, noisiest 128-column block "
                f"{worst['blk']:.2f}x the layer's rms error), appended cache elements that differ "
                f"{worst['kv_flips']:.2e}" + (f", free-running drift / rms {worst['free_rms']:.2e}" if free_running else "")
                + f"  [{time.time() - t0:.0f}s]")

    # the chained per-layer run IS the step: same kernels, same order, same bits
    assert np.array_equal(x.cpu().numpy(), gpu["hidden"]), "per-layer chain differs from the one-call step"

    g_final = synth.make_weight(cfg, "g_final", -1, "cuda").to("cpu", torch.float64)
    w_lm = synth.make_weight(cfg, "w_lm", -1, "cuda").to("cpu", torch.float64)
    tail = helpers.oracle_tail(cfg, gpu["hidden"], tokens, g_final, w_lm)
    err = compare_tail(gpu, tail, cfg.theta, O.accept_block, tokens, cfg.window, min_clean=min_clean)
    say(f"[{cfg.name}] teacher-forced tail: {err}; accepted lengths {gpu['accept_len'].tolist()}, "
        f"oracle {tail['accept_len'].tolist()}; kept mismatches {gpu['n_loose'].tolist()}; "
        f"h range {tail['h'].min():.3f} .. {tail['h'].max():.3f}")
    assert np.array_equal(gpu["kv_len_out"], cfg.kv_len + gpu["accept_len"] + 1)
    if mixed is not None:
        # the same model and tokens with per-position temperatures that put rows on both sides of
        # the gate (the layers do not depend on them; the LM head, the statistics and the rule do)
        mcfg = cfg.replace(temperatures=mixed)
        mgpu = wl.verify(tokens, helpers.row_scale(mcfg))
        assert np.array_equal(mgpu["hidden"], gpu["hidden"])
        mtail = helpers.oracle_tail(mcfg, mgpu["hidden"], tokens, g_final, w_lm)
        merr = compare_tail(mgpu, mtail, cfg.theta, O.accept_block, tokens, cfg.window, min_clean=min_clean)
        say(f"[{cfg.name}] the same with temperatures {mixed}: {merr}; accepted lengths "
            f"{mgpu['accept_len'].tolist()}, kept mismatches {mgpu['n_loose'].tolist()}; "
            f"h range {mtail['h'].min():.3f} .. {mtail['h'].max():.3f}")
    else:
        mcfg, mtail = cfg, tail
    # shorter windows fit more draft positions, so mismatching drafts are kept more often: the rule
    # on the same oracle statistics against one more device pass per window
    for W in (0, 1, 2):
        wgpu = wl.verify(tokens, helpers.row_scale(mcfg), W=W, want_hidden=False)
        check_own_rule(wgpu, tokens, cfg.theta, W, O.accept_block)
        want = O.accept_block(tokens[:, 1:], mtail["argmax"], mtail["h"], cfg.theta, W)
        amb = (mtail["margin"] < 1e-3) | (np.abs(mtail["h"] - cfg.theta) < 1e-3)
        clean = ~amb.any(axis=1)
        assert clean.sum() >= min_clean
        for k in ("accept_len", "next_token", "n_loose"):
            assert np.array_equal(wgpu[k][clean], want[k][clean]), (cfg.name, "W", W, k)
        say(f"[{cfg.name}] W = {W}: accepted lengths {wgpu['accept_len'].tolist()}, kept mismatches "
            f"{wgpu['n_loose'].tolist()} (oracle {want['n_loose'].tolist()})")

    if free_running:
        free = helpers.oracle_tail(cfg, x_free.view(B * R, d).numpy(), tokens, g_final, w_lm)
        lines = []
        for b in range(B):
            for i in range(R):
                if gpu["argmax"][b, i] != free["argmax"][b, i]:
                    lines.append(f"  argmax  seq {b} pos {i}: device {gpu['argmax'][b, i]} oracle {free['argmax'][b, i]}"
                                 f"  top-2 margin {free['margin'][b, i]:.3e}  |h-theta| {abs(free['h'][b, i] - cfg.theta):.3e}")
            if gpu["accept_len"][b] != free["accept_len"][b] or gpu["next_token"][b] != free["next_token"][b]:
                lines.append(f"  accept  seq {b}: device ({gpu['accept_len'][b]}, {gpu['next_token'][b]}) oracle "
                             f"({free['accept_len'][b]}, {free['next_token'][b]})  smallest margin "
                             f"{free['margin'][b].min():.3e}  smallest |h-theta| {np.abs(free['h'][b] - cfg.theta).min():.3e}")
        say(f"[{cfg.name}] FREE-RUNNING report (not asserted): max |lse| diff {np.abs(gpu['lse'] - free['lse']).max():.3e}, "
            f"|h| diff {np.abs(gpu['h_norm'] - free['h']).max():.3e}, |p_top1| diff "
            f"{np.abs(gpu['p_top1'] - free['p_top1']).max():.3e}; {len(lines)} integer disagreement(s)")
        for line in lines:
            say(line)
    return worst, err


FREE = os.environ.get("FLY_FREE_RUNNING", "0") == "1"


@pytest.mark.timeout(600)
def test_c2_8b_full_depth_teacher_forced(capsys):
    # 32 layers, d = 4096, one sequence of 9 rows against a 2048-token cache
    # (bounds: twice what a layer shows, 1.4e-3 / 1.0e-2; an fp32 evaluation of the same layer on
    # the CPU with the same rounding points differs from the fp64 oracle by as much)
    teacher_forced_depth(synth.CONFIGS["c2_8b"], capsys, 3e-3, 2.1e-2, min_clean=1, free_running=True,
                         mixed=(0.3, 1.0, 3.0))


@pytest.mark.timeout(900)
def test_c3_70b_full_depth_teacher_forced(capsys):
    # the benchmark's own configuration: 80 layers, 36 rows, 4 x 4096-token caches
    # (a layer shows 2.5e-3 / 2.0e-2)
    teacher_forced_depth(synth.CONFIGS["c3_70b"], capsys, 5e-3, 4e-2, min_clean=3, free_running=FREE)


@pytest.mark.timeout(900)
def test_c4_405b_slice_teacher_forced(capsys):
    # 8 layers at d = 16384 with 136 rows, 8 x 8192-token caches, and the full LM head
    # (a layer shows 3.1e-3 / 1.9e-2)
    teacher_forced_depth(synth.CONFIGS["c4_405b_slice"], capsys, 6.5e-3, 4e-2, min_clean=6, free_running=FREE,
                         mixed=(0.3, 1.0, 3.0))
