#!/usr/bin/env python3
"""Benchmark of the FLy verification step on one MI355X.

One "step" is one whole verification pass (embedding, all decoder layers with
KV append and attention, final norm, LM head with fused row statistics,
acceptance rule) over one block of B x (K+1) synthetic tokens.  Inputs are
resident in HBM before the timed region.  Prints one JSON line.

    python bench.py [--workload c3_70b] [--steps 20] [--warmup 5] [--gpus 1]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np
import torch

import synth

HBM_PEAK_GBS = 8000.0
DECODE_ROUNDS = 8           # rounds of the decode-loop line (Algorithm 1 with prompt-lookup drafting)
DECODE_WARMUP = 2
DECODE_NGRAM = 3
MFMA_PEAK_TFLOPS = 2500.0   # dense bf16, published
F32_PEAK_TFLOPS = 157.3     # fp32 vector / matrix, published
# HBM bytes per launch of the dominant kernel.  NOT measured by this run: hardware counters cannot be
# read from inside the process, so the figure comes from two `rocprofv3 --pmc` passes (FETCH_SIZE,
# then WRITE_SIZE) over `bench.py --roofline-only`, each scaled by what the same counter reads for a
# 1 GiB device copy; the summary with the commands is the file named here.
MEASURED_TRAFFIC = {"c3_70b": {"bytes": 946.6e6, "source": "profiles/gateup_gemm_c3_70b_hbm_counters.md"}}
# The paper's own figure where a preset is its setting (Table 3: Llama-3.1-70B target, K = 15,
# batch 1, one MI355X).  Context only: its software stack, prefix length and precision are not
# stated, so vs_baseline stays null.
PAPER_CONTEXT = {"p70b_k15": {"paper_reference": {"verify_ms_per_round": 58.62, "draft_ms_per_round": 245.51,
                                                   "hardware": "1x MI355X",
                                                   "source": "Table 3 (target verification; 8B drafter without "
                                                             "the multi-level acceleration)"}}}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def build_gpu_workload(cfg):
    from paper_2511_22972_amd import binding as fb
    t0 = time.time()
    desc = fb.make_desc(cfg)
    model = fb.PackedModel(desc, lambda name, layer: synth.make_weight(cfg, name, layer, "cuda"))
    log(f"[bench] weights generated and packed in {time.time() - t0:.1f}s")
    # room for the verified block and for the rounds of the decode-loop line
    cap = (cfg.kv_len + (DECODE_ROUNDS + DECODE_WARMUP + 1) * (cfg.K + 1) + 63) // 64 * 64
    kv = fb.KVCache(desc, cfg.batch, cap)
    for l in range(cfg.n_layers):
        k, v = synth.make_kv_prefix(cfg, l, "cuda")
        kv.load_prefix(l, k, v)
    kv.set_lengths([cfg.kv_len] * cfg.batch)
    ws = fb.alloc_workspace(fb.fly_workspace_bytes(desc, cfg.batch, cfg.K, cfg.kv_len))
    torch.cuda.synchronize()
    log(f"[bench] KV cache ready, total setup {time.time() - t0:.1f}s, "
        f"HBM in use {torch.cuda.memory_allocated() / 2**30:.1f} GiB")
    return fb, desc, model, kv, ws


def device_draft_chain(fb, cfg, model, kv, ws, row_scale):
    """Draft tokens for the timed block: draft i equals the target's argmax at
    position i with probability p_match, else a uniform token.  The chain is
    built with K+1 untimed passes of the verification step itself (row i's
    argmax does not depend on later tokens)."""
    first = synth.make_first_tokens(cfg, "cuda")
    u, alt, _ = synth.make_draft_draws(cfg, "cuda")
    tokens = torch.zeros(cfg.batch, cfg.K + 1, dtype=torch.int32, device="cuda")
    tokens[:, 0] = first
    out = fb.VerifyOutputs(cfg.batch, cfg.K)
    for i in range(1, cfg.K + 1):
        fb.fly_verify_block(model, kv, tokens, row_scale, cfg.theta, cfg.window, out, ws)
        y = out.argmax[:, i - 1]
        tokens[:, i] = torch.where(u[:, i - 1] < cfg.p_match, y, alt[:, i - 1])
    torch.cuda.synchronize()
    return tokens


def decode_loop_line(fb, cfg, desc, model, kv, row_scale):
    """Algorithm 1's loop on the device: DECODE_ROUNDS rounds of (prompt-lookup
    draft, verification step, roll-forward), timed as one region.  The prompt is
    synthetic (seeded tokens; the cached prefix is the synthetic one, not the
    cache of these tokens), so tau says nothing about real text: the line shows
    what a round costs beyond the verification step."""
    B, K = cfg.batch, cfg.K
    n0 = cfg.kv_len + 1
    total_rounds = DECODE_ROUNDS + DECODE_WARMUP
    seq = fb.Sequences(kv, n0 + total_rounds * (K + 1) + 1, total_rounds)
    prompt = synth.hash_tokens(cfg.seed, 950, B * n0, cfg.vocab, "cuda").view(B, n0)
    prompt[:, -1] = synth.make_first_tokens(cfg, "cuda")
    seq.ctx[:, :n0] = prompt
    seq.ctx_len.fill_(n0)
    seq.max_ctx_len = n0
    ws = fb.alloc_workspace(fb.fly_decode_workspace_bytes(desc, B, K, cfg.kv_len + total_rounds * (K + 1)))
    fb.fly_decode_rounds(model, kv, seq, row_scale, K, cfg.theta, cfg.window, DECODE_NGRAM, DECODE_WARMUP, ws)
    torch.cuda.synchronize()
    s_before = seq.accepted_total.sum().item()
    t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0.record()
    fb.fly_decode_rounds(model, kv, seq, row_scale, K, cfg.theta, cfg.window, DECODE_NGRAM, DECODE_ROUNDS, ws)
    t1.record()
    torch.cuda.synchronize()
    ms = t0.elapsed_time(t1)
    s_sum = seq.accepted_total.sum().item() - s_before
    kv.set_lengths([cfg.kv_len] * B)             # back to the state the other lines assume
    return {"rounds": DECODE_ROUNDS, "ms_per_round": ms / DECODE_ROUNDS,
            "tokens_per_s": s_sum / (ms * 1e-3), "tau": s_sum / (DECODE_ROUNDS * B),
            "ngram_max": DECODE_NGRAM, "drafter": "prompt lookup on a synthetic prompt"}


def model_drafted_loop_line(fb, cfg, desc, model, kv, row_scale):
    """Algorithm 1 with a draft MODEL as drafter (the paper's own setting: an 8B-shaped drafter for the
    70B-shaped target): K chained greedy passes of the drafter, the verification step, the roll-forward.
    Reports the time of the drafting alone and of the whole round.  Only for targets whose vocabulary is
    the 8B preset's; None otherwise."""
    dcfg = synth.CONFIGS["c2_8b"]
    if cfg.dtype != "bf16" or cfg.vocab != dcfg.vocab or cfg.n_layers < 16:
        return None
    B, K = cfg.batch, cfg.K
    rounds, warm = 3, 1
    dcfg = dcfg.replace(batch=B, K=K, kv_len=cfg.kv_len)
    ddesc = fb.make_desc(dcfg)
    dmodel = fb.PackedModel(ddesc, lambda name, layer: synth.make_weight(dcfg, name, layer, "cuda"))
    n0 = cfg.kv_len + 1
    cap = (n0 + (rounds + warm + 1) * (K + 1) + K + 63) // 64 * 64
    dkv = fb.KVCache(ddesc, B, cap)
    for l in range(dcfg.n_layers):
        k, v = synth.make_kv_prefix(dcfg, l, "cuda")
        dkv.load_prefix(l, k, v)
    seq = fb.Sequences(kv, n0 + (rounds + warm) * (K + 1) + 1, rounds + warm)
    prompt = synth.hash_tokens(cfg.seed, 951, B * n0, cfg.vocab, "cuda").view(B, n0)
    seq.ctx[:, :n0] = prompt
    seq.ctx_len.fill_(n0)
    seq.max_ctx_len = n0
    kv.set_lengths([cfg.kv_len] * B)
    ws = fb.alloc_workspace(fb.fly_decode_model_workspace_bytes(desc, ddesc, B, K, cfg.kv_len + (rounds + warm) * (K + 1)))
    fb.fly_decode_rounds_model(model, kv, dmodel, dkv, seq, row_scale, K, cfg.theta, cfg.window, warm, ws)
    torch.cuda.synchronize()
    s_before = seq.accepted_total.sum().item()
    t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0.record()
    fb.fly_decode_rounds_model(model, kv, dmodel, dkv, seq, row_scale, K, cfg.theta, cfg.window, rounds, ws)
    t1.record()
    torch.cuda.synchronize()
    round_ms = t0.elapsed_time(t1) / rounds
    s_sum = seq.accepted_total.sum().item() - s_before
    # the drafting alone, on the state the loop left
    tokens = torch.empty(B, K + 1, dtype=torch.int32, device="cuda")
    dws = fb.alloc_workspace(fb.fly_model_draft_workspace_bytes(ddesc, B, K, seq.max_ctx_len))
    draft_ms = time_region(lambda: fb.fly_model_draft(dmodel, dkv, seq.ctx, seq.ctx_len, seq.max_ctx_len, K, tokens, dws),
                           3, 1)
    kv.set_lengths([cfg.kv_len] * B)
    kv.max_kv_len = cfg.kv_len
    return {"drafter": "c2_8b-shaped model (32 layers, d=4096), greedy", "rounds": rounds,
            "ms_per_round": round_ms, "draft_ms_per_round": draft_ms, "drafter_passes_per_round": K,
            "tokens_per_s": s_sum / (round_ms * rounds * 1e-3), "tau": s_sum / (rounds * B),
            "note": "random weights: the drafter's tokens are unrelated to the target's, tau says nothing about text"}


def algorithmic_bytes(cfg):
    """Bytes one verification step must move: every weight once, the visible
    cache once, plus the (small) activations."""
    es = 2 if cfg.dtype == "bf16" else 4
    per_layer = sum(a * b for a, b in synth.layer_weight_shapes(cfg).values()) * es
    lm = cfg.d * cfg.vocab * es
    kvb = 2 * cfg.batch * (cfg.kv_len + cfg.K + 1) * cfg.kv_dim * es * cfg.n_layers
    return {"layer_weights": per_layer * cfg.n_layers, "lm_head": lm, "kv": kvb,
            "total": per_layer * cfg.n_layers + lm + kvb}


def time_region(fn, steps, warmup, per_call=False):
    """ms per call over `steps` calls after `warmup` untimed ones (events on the launch stream, one
    region around all calls).  With per_call also the list of per-call times, from one more event
    recorded after every call (the mean is still that of the whole region)."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1 if per_call else 2)]
    marks[0].record()
    for i in range(steps):
        fn()
        if per_call:
            marks[i + 1].record()
    if not per_call:
        marks[1].record()
    torch.cuda.synchronize()
    mean = marks[0].elapsed_time(marks[-1]) / steps
    if per_call:
        return mean, [marks[i].elapsed_time(marks[i + 1]) for i in range(steps)]
    return mean


def graph_replay_ms(step, steps, warmup):
    """The step captured in a HIP graph (it enqueues kernels only) and replayed:
    ms per replay, or None where the runtime refuses the capture."""
    try:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        return time_region(graph.replay, steps, warmup)
    except Exception as e:  # reported, never fatal: the eager number is the headline
        log(f"[bench] graph capture unavailable: {e}")
        return None


def cpu_baseline(cfg, tokens_np, layers_sampled=2):
    """The oracle timed on this host on a bounded sample: `layers_sampled`
    decoder layers plus the LM head, row statistics and acceptance rule for the
    whole block; the full step is extrapolated as n_layers x layer + head."""
    from oracle import fly_oracle as O
    from tests import helpers
    B, R = tokens_np.shape
    num = O.Numerics(cfg.dtype)
    f64 = lambda t: t.to("cpu", torch.float64)
    x0 = f64(synth.make_hidden(cfg, B * R, "cuda")).view(B, R, cfg.d)
    t_layer = 0.0
    t_layer_1 = None
    for l in range(layers_sampled):
        w = helpers.oracle_layer_weights(cfg, l, "cuda")
        kp, vp = (f64(t) for t in synth.make_kv_prefix(cfg, l, "cuda"))
        t0 = time.perf_counter()
        for b in range(B):
            O.decoder_layer(x0[b], w, kp[b], vp[b], cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim,
                            cfg.rope_theta, cfg.rms_eps, num)
        t_layer += time.perf_counter() - t0
        if l == 0:
            # the same layer on one thread, ONE sequence of the batch (the sequences cost the same)
            nthreads = torch.get_num_threads()
            torch.set_num_threads(1)
            t0 = time.perf_counter()
            O.decoder_layer(x0[0], w, kp[0], vp[0], cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim,
                            cfg.rope_theta, cfg.rms_eps, num)
            t_layer_1 = (time.perf_counter() - t0) * B
            torch.set_num_threads(nthreads)
        del w, kp, vp
    t_layer /= layers_sampled
    w_lm = f64(synth.make_weight(cfg, "w_lm", -1, "cuda"))
    g = f64(synth.make_weight(cfg, "g_final", -1, "cuda"))
    rs = (1.0 / synth.make_row_temperature(cfg)).reshape(-1)
    t0 = time.perf_counter()
    xn = num.act(O.rmsnorm(x0.reshape(B * R, cfg.d), g, cfg.rms_eps))
    stats = O.decision_statistics(O.lm_head_logits(xn, w_lm, rs))
    acc = O.accept_block(tokens_np[:, 1:], stats["argmax"].reshape(B, R), stats["h"].reshape(B, R),
                         cfg.theta, cfg.window)
    t_head = time.perf_counter() - t0
    total = cfg.n_layers * t_layer + t_head
    return {"t_layer_s": t_layer, "t_layer_1thread_s": t_layer_1, "t_head_s": t_head, "t_step_s": total,
            "sample": f"{layers_sampled} of {cfg.n_layers} decoder layers + LM head + row statistics + "
                      f"acceptance for all {B * R} rows; step = n_layers x layer + head"}


def roofline_only(cfg, args):
    """Isolated launches of the gate/up GEMM over `n_layers` distinct weight
    matrices, then one 1 GiB device-to-device copy whose traffic is known
    (1 GiB read + 1 GiB written): the calibration for byte counters."""
    from paper_2511_22972_amd import binding as fb
    desc = fb.make_desc(cfg)
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    es = 2 if cfg.dtype == "bf16" else 4
    if args.kernel == "attention":
        # the KV-streaming phase alone: split-KV attention + merge of the splits, one layer's cache
        cap = (cfg.kv_len + cfg.K + 1 + 63) // 64 * 64
        one = cfg.replace(n_layers=1)
        desc1 = fb.make_desc(one)
        kv = fb.KVCache(desc1, cfg.batch, cap)
        k, v = synth.make_kv_prefix(one, 0, "cuda")
        kv.load_prefix(0, k, v)
        del k, v
        kv.set_lengths([cfg.kv_len] * cfg.batch)
        q = synth.hash_normal(cfg.seed, 960, (cfg.M, cfg.q_dim), 1.0, tdt, "cuda")
        o = torch.empty_like(q)
        ws = fb.alloc_workspace(fb.fly_workspace_bytes(desc1, cfg.batch, cfg.K, cfg.kv_len))

        def attention():
            fb.fly_attention(desc1, kv, 0, q, o, cfg.batch, cfg.K, ws)

        ms = time_region(attention, args.steps, args.warmup)
        nbytes = 2 * cfg.batch * (cfg.kv_len + cfg.K + 1) * cfg.kv_dim * es
        flops = 4.0 * cfg.batch * cfg.n_q_heads * (cfg.K + 1) * (cfg.kv_len + cfg.K + 1) * cfg.head_dim
        print(json.dumps({"kernel": "attention (split-KV kernel + merge)", "workload": cfg.name,
                          "launches": args.steps + args.warmup, "avg_launch_us": ms * 1e3,
                          "bytes_per_launch": nbytes, "achieved_GBps": nbytes / (ms * 1e-3) / 1e9,
                          "flops_per_launch": flops, "achieved_TFLOPs": flops / (ms * 1e-3) / 1e12}))
        return
    if args.kernel == "lmhead" or (args.kernel == "auto" and cfg.dtype == "bf16" and cfg.M > 256):
        # contraction regime: the dominant kernel is the LM head with fused row statistics
        w_lm = torch.empty(cfg.d * cfg.vocab, dtype=tdt, device="cuda")
        fb.fly_pack_weight(synth.make_weight(cfg, "w_lm", -1, "cuda"), w_lm, cfg.vocab)
        hidden = synth.make_hidden(cfg, cfg.M, "cuda")
        row_scale = (1.0 / synth.make_row_temperature(cfg, "cuda")).reshape(-1).contiguous()
        out = fb.VerifyOutputs(cfg.batch, cfg.K)
        ws = fb.alloc_workspace(fb.fly_lmhead_workspace_bytes(cfg.M, cfg.d, cfg.vocab, desc.dtype))

        def lmhead():
            fb.fly_lmhead_entropy_argmax(hidden, w_lm, row_scale, cfg.vocab, out.argmax.view(-1),
                                         out.p_top1.view(-1), out.h_norm.view(-1), None, ws)

        ms = time_region(lmhead, args.steps, args.warmup)
        flops = 2.0 * cfg.M * cfg.d * cfg.vocab
        print(json.dumps({"kernel": "LM head + fused row statistics", "workload": cfg.name,
                          "launches": args.steps + args.warmup, "avg_launch_us": ms * 1e3,
                          "flops_per_launch": flops, "achieved_TFLOPs": flops / (ms * 1e-3) / 1e12}))
        return
    packed = []
    for l in range(cfg.n_layers):
        gu = torch.empty(cfg.d * 2 * cfg.ffn, dtype=tdt, device="cuda")
        fb.fly_pack_weight(synth.make_weight(cfg, "wg", l, "cuda"), gu, 2 * cfg.ffn, 0, 2)
        fb.fly_pack_weight(synth.make_weight(cfg, "wu", l, "cuda"), gu, 2 * cfg.ffn, 1, 2)
        packed.append(gu)
    xn = synth.make_hidden(cfg, cfg.M, "cuda")
    a_buf = torch.empty(cfg.M, cfg.ffn, dtype=tdt, device="cuda")
    counter = [0]

    def gateup():
        l = counter[0] % cfg.n_layers
        counter[0] += 1
        fb.fly_gateup_swiglu(xn, packed[l], a_buf)

    ms = time_region(gateup, args.steps, args.warmup)
    nbytes = cfg.d * 2 * cfg.ffn * es + cfg.M * cfg.d * es + cfg.M * cfg.ffn * es
    src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").zero_()
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    dst.copy_(src)
    torch.cuda.synchronize()
    print(json.dumps({"kernel": "gate/up GEMM + SwiGLU", "workload": cfg.name, "launches": args.steps + args.warmup,
                      "avg_launch_us": ms * 1e3, "bytes_per_launch": nbytes,
                      "achieved_GBps": nbytes / (ms * 1e-3) / 1e9,
                      "calibration": "one 1 GiB torch device copy: 1048576 KiB read, 1048576 KiB written"}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c3_70b", choices=sorted(synth.CONFIGS))
    ap.add_argument("--layers", type=int, default=0, help="override the layer count (debugging)")
    ap.add_argument("--batch", type=int, default=0,
                    help="override the number of sequences (other row counts of the same model shape)")
    ap.add_argument("--K", type=int, default=0, help="override the number of draft tokens per sequence")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--step-only", action="store_true",
                    help="only the timed step and the isolated gate/up and LM-head launches: no graph replay, "
                         "no drawn-token step, no decode loops (for profiler runs, where every extra launch "
                         "mixes into the per-kernel averages)")
    ap.add_argument("--kernel", default="auto", choices=["auto", "gateup", "lmhead", "attention"],
                    help="with --roofline-only: which kernel to launch alone (auto = the dominant one)")
    ap.add_argument("--roofline-only", action="store_true",
                    help="run only the dominant kernel (gate/up GEMM, isolated launches) and a 1 GiB "
                         "device copy of known size; for hardware-counter passes (use with --layers)")
    ap.add_argument("--tune", action="append", default=[], metavar="KEY=VALUE",
                    help="library tuning knob (fly_set_tuning), e.g. fuse=1; for experiments")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)",
              file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    for kv_pair in args.tune:
        from paper_2511_22972_amd import binding as _fb
        key, _, val = kv_pair.partition("=")
        _fb.fly_set_tuning(key, int(val))
    cfg = synth.CONFIGS[args.workload]
    if args.layers:
        cfg = cfg.replace(n_layers=args.layers)
    if args.batch:
        cfg = cfg.replace(name=f"{cfg.name}_batch{args.batch}", batch=args.batch)
    if args.K:
        cfg = cfg.replace(name=f"{cfg.name}_K{args.K}", K=args.K)

    if args.roofline_only:
        roofline_only(cfg, args)
        return

    fb, desc, model, kv, ws = build_gpu_workload(cfg)
    row_scale = (1.0 / synth.make_row_temperature(cfg, "cuda")).reshape(-1).contiguous()
    tokens = device_draft_chain(fb, cfg, model, kv, ws, row_scale)
    out = fb.VerifyOutputs(cfg.batch, cfg.K)

    def step():
        fb.fly_verify_block(model, kv, tokens, row_scale, cfg.theta, cfg.window, out, ws)

    ms, per_step = time_region(step, args.steps, args.warmup, per_call=True)
    graph_ms = None if args.step_only else graph_replay_ms(step, args.steps, args.warmup)
    # The same step at temperature > 0: the target's tokens drawn instead of the argmax (a reading of
    # ours, the paper prints no rule for its temperature-1 rows); its own outputs, the headline is the
    # greedy step above.
    out_s = fb.VerifyOutputs(cfg.batch, cfg.K)
    sampled = torch.zeros(cfg.batch, cfg.K + 1, dtype=torch.int32, device="cuda")
    call = [0]

    def step_sampled():
        call[0] += 1
        fb.fly_verify_block_sampled(model, kv, tokens, row_scale, cfg.theta, cfg.window, cfg.seed, call[0],
                                    sampled, out_s, ws)

    sampled_ms = None if args.step_only else time_region(step_sampled, max(args.steps // 2, 3), 2)
    step()  # leave the greedy step's rows in the cache and its outputs in `out`
    torch.cuda.synchronize()
    accept_len = out.accept_len.cpu().numpy()
    s_total = int((accept_len + 1).sum())          # the paper's count: kept drafts + 1
    tokens_per_s = s_total / (ms * 1e-3)
    ab = algorithmic_bytes(cfg)

    # Dominant kernel: the gate/up GEMM with fused SwiGLU (about 55% of a layer's
    # bytes), timed alone with events on the launch stream, cycling through the
    # layers so no launch finds its weights in cache.
    es = 2 if cfg.dtype == "bf16" else 4
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    xn = synth.make_hidden(cfg, cfg.M, "cuda")
    a_buf = torch.empty(cfg.M, cfg.ffn, dtype=tdt, device="cuda")
    gu_ptrs = [model.layers_c[l].w_gateup for l in range(cfg.n_layers)]
    counter = [0]
    import ctypes as C

    def gateup():
        l = counter[0] % cfg.n_layers
        counter[0] += 1
        rc = fb.lib.fly_gateup_swiglu(xn.data_ptr(), gu_ptrs[l], a_buf.data_ptr(), cfg.M, cfg.d,
                                      cfg.ffn, desc.dtype, torch.cuda.current_stream().cuda_stream)
        assert rc == 0, rc

    gu_ms = time_region(gateup, max(args.steps, 20) * 4, 8)
    gu_bytes = cfg.d * 2 * cfg.ffn * es + cfg.M * cfg.d * es + cfg.M * cfg.ffn * es
    gu_gbs = gu_bytes / (gu_ms * 1e-3) / 1e9
    gu_flops = 2.0 * cfg.M * cfg.d * 2 * cfg.ffn

    # The LM head with its fused row statistics, timed alone the same way (GEMM
    # kernel plus the small kernel that merges the per-block statistics).
    hidden = synth.make_hidden(cfg, cfg.M, "cuda")
    lm_ws = fb.alloc_workspace(fb.fly_lmhead_workspace_bytes(cfg.M, cfg.d, cfg.vocab, desc.dtype))
    lm_out = fb.VerifyOutputs(cfg.batch, cfg.K)

    def lmhead():
        fb.fly_lmhead_entropy_argmax(hidden, model.w_lm, row_scale, cfg.vocab, lm_out.argmax.view(-1),
                                     lm_out.p_top1.view(-1), lm_out.h_norm.view(-1), None, lm_ws)

    lm_ms = time_region(lmhead, max(args.steps, 20), 4)
    # the same with a token drawn per row (temperature > 0), fused into the same epilogue
    lm_sampled = torch.zeros(cfg.M, dtype=torch.int32, device="cuda")
    draw = [0]

    def lmhead_sampled():
        draw[0] += 1
        fb.fly_lmhead_entropy_sample(hidden, model.w_lm, row_scale, cfg.vocab, cfg.seed, draw[0], lm_sampled,
                                     lm_out.argmax.view(-1), lm_out.p_top1.view(-1), lm_out.h_norm.view(-1),
                                     None, lm_ws)

    lms_ms = float("nan") if args.step_only else time_region(lmhead_sampled, max(args.steps, 20), 4)
    lm_bytes = cfg.d * cfg.vocab * es + cfg.M * cfg.d * es
    lm_flops = 2.0 * cfg.M * cfg.d * cfg.vocab
    mfma_peak = MFMA_PEAK_TFLOPS if cfg.dtype == "bf16" else F32_PEAK_TFLOPS
    lm_head = {"avg_launch_us": lm_ms * 1e3, "flops_per_launch": lm_flops, "bytes_per_launch": lm_bytes,
               "achieved_TFLOPs": lm_flops / (lm_ms * 1e-3) / 1e12, "achieved_GBps": lm_bytes / (lm_ms * 1e-3) / 1e9,
               "frac_of_mfma_peak": lm_flops / (lm_ms * 1e-3) / 1e12 / mfma_peak,
               "frac_of_hbm_peak": lm_bytes / (lm_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
               "with_drawn_token_us": lms_ms * 1e3}
    # The contraction regime in the same record: the LM head of the stress workload (64 sequences x 17
    # positions = 1088 rows, same width and vocabulary, hence this model's own LM-head weights), where
    # the GEMM is bound by the matrix cores -- the figure the >= 60% MFMA target is about.
    lm_mfma = None
    c5 = synth.CONFIGS["c5_stress"]
    if cfg.dtype == "bf16" and cfg.d == c5.d and cfg.vocab == c5.vocab and cfg.M <= 256 and not args.step_only:
        h5 = synth.make_hidden(c5, c5.M, "cuda")
        rs5 = (1.0 / synth.make_row_temperature(c5, "cuda")).reshape(-1).contiguous()
        ws5 = fb.alloc_workspace(fb.fly_lmhead_workspace_bytes(c5.M, c5.d, c5.vocab, desc.dtype))
        o5 = fb.VerifyOutputs(c5.batch, c5.K)

        def lmhead5():
            fb.fly_lmhead_entropy_argmax(h5, model.w_lm, rs5, c5.vocab, o5.argmax.view(-1), o5.p_top1.view(-1),
                                         o5.h_norm.view(-1), None, ws5)

        ms5 = time_region(lmhead5, 20, 5)
        fl5 = 2.0 * c5.M * c5.d * c5.vocab
        lm_mfma = {"workload": "c5_stress LM head + fused row statistics (1088 rows x 8192 x 128256)",
                   "bound": "mfma", "avg_launch_us": ms5 * 1e3, "flops_per_launch": fl5,
                   "achieved": fl5 / (ms5 * 1e-3) / 1e12, "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                   "frac": fl5 / (ms5 * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS}
        del h5, ws5
    # Up to 256 rows every GEMM is bound by streaming its weights (the weight-
    # streaming kernels; 256 flop per weight byte is still below the ridge) and the
    # dominant kernel is gate/up.  Beyond that the GEMMs are dense contractions
    # (LDS-tiled kernel): the dominant kernel is then the LM head and the bound is
    # the matrix cores.
    contraction = cfg.dtype == "bf16" and cfg.M > 256
    if contraction:
        roofline = {"kernel": "gemm_bf16_tiled_kernel (LM head + fused row statistics)", "bound": "mfma",
                    "achieved": lm_head["achieved_TFLOPs"], "peak": mfma_peak, "unit": "TFLOP/s",
                    "frac": lm_head["frac_of_mfma_peak"], "traffic": None,
                    "flops_per_launch": lm_flops, "avg_launch_us": lm_ms * 1e3}
    else:
        gu_kernel = ("gemm_f32_kernel" if cfg.dtype != "bf16" else
                     "gemm_bf16_kernel" if cfg.M <= 80 else "gemm_bf16_wide_kernel")
        roofline = {"kernel": gu_kernel + " (gate/up projection + SwiGLU)",
                    "bound": "hbm", "achieved": gu_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": gu_gbs / HBM_PEAK_GBS,
                    "traffic": None, "bytes_per_launch": gu_bytes, "avg_launch_us": gu_ms * 1e3}
        if cfg.name in MEASURED_TRAFFIC and not args.layers:
            roofline["traffic"] = MEASURED_TRAFFIC[cfg.name]["bytes"]
            roofline["traffic_source"] = ("hardware counters of a separate profiler run, not of this run: "
                                          + MEASURED_TRAFFIC[cfg.name]["source"])

    res = {
        "metric": "verified tokens/s (FLy verify step)", "value": tokens_per_s, "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
        "verify_step_us": ms * 1e3, "ms_per_step_median": float(np.median(per_step)),
        "ms_per_step_min": float(np.min(per_step)), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name, "n_layers": cfg.n_layers, "d": cfg.d, "heads": f"{cfg.n_q_heads}q/{cfg.n_kv_heads}kv",
                   "ffn": cfg.ffn, "vocab": cfg.vocab, "batch": cfg.batch, "K": cfg.K,
                   "kv_len": cfg.kv_len, "theta": cfg.theta, "W": cfg.window, "rows": cfg.M,
                   "accepted_tokens_per_step": s_total, **PAPER_CONTEXT.get(cfg.name, {})},
        "step_hbm": {"algorithmic_bytes": ab["total"], "achieved_GBps": ab["total"] / (ms * 1e-3) / 1e9,
                     "frac_of_peak": ab["total"] / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS},
        "roofline": roofline,
        "gate_up": {"avg_launch_us": gu_ms * 1e3, "achieved_GBps": gu_gbs, "achieved_TFLOPs": gu_flops / (gu_ms * 1e-3) / 1e12},
        "lm_head": lm_head,
        "lm_head_mfma_regime": lm_mfma,
        "decode_loop": None if args.step_only else decode_loop_line(fb, cfg, desc, model, kv, row_scale),
        "model_drafted_loop": None if args.step_only else model_drafted_loop_line(fb, cfg, desc, model, kv, row_scale),
        "sampled_step": {"ms_per_step": sampled_ms,
                         "note": "fly_verify_block_sampled: target tokens drawn at the rows' temperatures (Gumbel-max fused into the LM head)"},
        "graph_replay": {"ms_per_step": graph_ms,
                         "note": "the same step captured once in a HIP graph and replayed; equal to the eager time when the device, not the host launch path, is the limit"},
    }
    if not args.no_cpu_baseline:
        torch.cuda.synchronize()
        cb = cpu_baseline(cfg, tokens.cpu().numpy())
        res["cpu_baseline"] = {"value": s_total / cb["t_step_s"], "unit": "tokens/s",
                               "cores": torch.get_num_threads(), "host_logical_cpus": os.cpu_count(),
                               "kind": "oracle", "sample": cb["sample"],
                               "oracle_step_s_extrapolated": cb["t_step_s"],
                               "oracle_layer_s": cb["t_layer_s"], "oracle_head_s": cb["t_head_s"],
                               "oracle_layer_1thread_s": cb["t_layer_1thread_s"],
                               "note_1thread": "the sampled layer on one thread: one sequence timed, times the batch"}
    print(json.dumps(res))


if __name__ == "__main__":
    main()
