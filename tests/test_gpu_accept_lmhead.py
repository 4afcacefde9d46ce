"""HIP fly_accept and fly_lmhead_entropy_argmax against the CPU oracle."""
import itertools
import math

import numpy as np
import pytest
import torch

import synth
from oracle import fly_oracle as O

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fb():
    from paper_2511_22972_amd import binding
    return binding


def run_accept(fb, draft, target, h, theta, W):
    B, K = draft.shape
    dev = "cuda"
    acc = torch.zeros(B, dtype=torch.int32, device=dev)
    nxt = torch.zeros(B, dtype=torch.int32, device=dev)
    loose = torch.zeros(B, dtype=torch.int32, device=dev)
    fb.fly_accept(torch.as_tensor(draft, dtype=torch.int32).to(dev),
                  torch.as_tensor(target, dtype=torch.int32).to(dev),
                  torch.as_tensor(h, dtype=torch.float32).to(dev), theta, W, acc, nxt, loose)
    torch.cuda.synchronize()
    return acc.cpu().numpy(), nxt.cpu().numpy(), loose.cpu().numpy()


@pytest.mark.parametrize("K", [1, 2, 5, 8])
def test_accept_exhaustive(fb, K):
    """All mismatch x gate patterns, every W in 0..K+1, as one batch per W."""
    rows = []
    for bits in itertools.product([0, 1], repeat=K):
        for gates in itertools.product([0, 1], repeat=K):
            if any(g and d for g, d in zip(gates, bits)):
                continue
            rows.append((bits, gates))
    B = len(rows)
    target = np.tile(np.arange(100, 100 + K + 1, dtype=np.int32), (B, 1))
    draft = np.array([[target[0, i] if bits[i] else 7 for i in range(K)] for bits, _ in rows], dtype=np.int32)
    h = np.array([[0.9 if g else 0.1 for g in gates] + [0.5] for _, gates in rows], dtype=np.float32)
    for W in range(0, K + 2):
        ref = O.accept_block(draft, target, h, 0.3, W)
        acc, nxt, loose = run_accept(fb, draft, target, h, 0.3, W)
        assert np.array_equal(acc, ref["accept_len"]), W
        assert np.array_equal(nxt, ref["next_token"]), W
        assert np.array_equal(loose, ref["n_loose"]), W


def test_accept_random_and_limits(fb):
    rng = np.random.default_rng(0)
    for K in (3, 15, 16, 25, 62, 63):
        B = 257
        target = rng.integers(0, 128256, size=(B, K + 1)).astype(np.int32)
        draft = np.where(rng.random((B, K)) < 0.8, target[:, :K], rng.integers(0, 128256, size=(B, K))).astype(np.int32)
        h = rng.random((B, K + 1)).astype(np.float32)
        h[::7, :] = np.float32(0.3)                       # equality at the gate defers
        for theta, W in ((0.3, 6), (0.3, 0), (0.0, 0), (2.0, 6), (0.6, 2), (0.3, K), (0.3, 100),
                         (0.3, 2 ** 31 - 1), (0.0, 2 ** 31 - 64)):
            ref = O.accept_block(draft, target, h, theta, W)
            acc, nxt, loose = run_accept(fb, draft, target, h, theta, W)
            assert np.array_equal(acc, ref["accept_len"]), (K, theta, W)
            assert np.array_equal(nxt, ref["next_token"]), (K, theta, W)
            assert np.array_equal(loose, ref["n_loose"]), (K, theta, W)
            if theta == 0.0 and W == 0:
                assert np.all(acc == K)
            if theta == 2.0 or W >= K:
                std = np.array([O.s_standard(O.match_indicator(draft[b], target[b])) for b in range(B)])
                assert np.array_equal(acc + 1, std)


def lmhead_case(fb, M, d, V, dtype, scale_rows=True, seed=1, plant=None, hidden_std=1.0):
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    hidden = synth.hash_normal(seed, 201, (M, d), hidden_std, tdt, "cuda")
    w = synth.hash_normal(seed, 202, (d, V), 0.02, tdt, "cuda")
    if plant is not None:
        w = plant(w, hidden)
    code = fb.dtype_code(dtype)
    wp = torch.empty(fb.fly_packed_weight_bytes(d, V, code) // w.element_size(), dtype=tdt, device="cuda")
    fb.fly_pack_weight(w, wp, V)
    rs = None
    if scale_rows:
        rs = torch.exp(torch.linspace(math.log(0.1), math.log(10.0), M)).to("cuda", torch.float32)
    argmax = torch.zeros(M, dtype=torch.int32, device="cuda")
    p1, hn, lse = (torch.zeros(M, dtype=torch.float32, device="cuda") for _ in range(3))
    ws = fb.alloc_workspace(fb.fly_lmhead_workspace_bytes(M, d, V, code))
    fb.fly_lmhead_entropy_argmax(hidden, wp, rs, V, argmax, p1, hn, lse, ws)
    torch.cuda.synchronize()
    logits = O.lm_head_logits(hidden.cpu().double(), w.cpu().double(), None if rs is None else rs.cpu())
    ref = O.decision_statistics(logits)
    got = {"argmax": argmax.cpu().numpy(), "p_top1": p1.cpu().numpy(), "h": hn.cpu().numpy(),
           "lse": lse.cpu().numpy()}
    return got, ref


def check_lmhead(got, ref, tol):
    assert np.abs(got["lse"] - ref["lse"]).max() <= tol
    assert np.abs(got["h"] - ref["h"]).max() <= tol
    assert np.abs(got["p_top1"] - ref["p_top1"]).max() <= tol
    near_tie = ref["margin"] < 1e-3
    assert np.all((got["argmax"] == ref["argmax"]) | near_tie)
    assert (~near_tie).sum() > 0


@pytest.mark.parametrize("M,d,V", [(5, 256, 8192), (9, 64, 48), (17, 688, 1040)])
def test_lmhead_f32(fb, M, d, V):
    got, ref = lmhead_case(fb, M, d, V, "f32", hidden_std=4.0)
    check_lmhead(got, ref, 1e-4)
    if V >= 1024:
        assert ref["h"].min() < 0.3 < ref["h"].max()      # rows on both sides of the gate


@pytest.mark.parametrize("M,d,V", [(9, 256, 8192), (36, 1024, 4112), (50, 512, 16 * 131),
                                   (136, 256, 2048), (150, 128, 1024), (1, 32, 16)])
def test_lmhead_bf16(fb, M, d, V):
    got, ref = lmhead_case(fb, M, d, V, "bf16", hidden_std=4.0)
    # inputs are bf16 on both sides and accumulation is fp32: far inside 2e-2
    check_lmhead(got, ref, 2e-3)


def test_lmhead_bf16_nine_tile_streaming_kernel(fb):
    """81..128 rows through the 16-row-tile kernel (nine tiles per wave), which the planner no
    longer picks by itself."""
    fb.fly_set_tuning("gemm_wide", 1)
    try:
        for M, d, V in ((100, 256, 2048 + 48), (128, 96, 272)):
            got, ref = lmhead_case(fb, M, d, V, "bf16", hidden_std=4.0, seed=7)
            check_lmhead(got, ref, 2e-3)
    finally:
        fb.fly_set_tuning("gemm_wide", 0)


@pytest.mark.parametrize("M,d,V", [(200, 256, 2048 + 48), (300, 544, 16 * 131), (1088, 512, 4096),
                                   (145, 32, 16), (385, 96, 272)])
def test_lmhead_bf16_many_rows(fb, M, d, V):
    """Row counts that take the LDS-tiled GEMM (workgroups of 128 or 192 rows): ragged last row
    block, a vocabulary that is not a multiple of the 256-column block, fewer k-steps than the
    prefetch ring is deep."""
    got, ref = lmhead_case(fb, M, d, V, "bf16", hidden_std=4.0)
    check_lmhead(got, ref, 2e-3)
    # every workgroup shape; two of them also with every wave requesting its loads first
    # ("tiled_phase" 2; by default the odd waves request theirs in mid-step)
    for wm, phase in ((2, 0), (3, 0), (4, 0), (6, 0), (3, 2), (6, 2)):
        fb.fly_set_tuning("gemm_tiled", wm)
        fb.fly_set_tuning("tiled_phase", phase)
        try:
            got, ref = lmhead_case(fb, M, d, V, "bf16", hidden_std=4.0, seed=3)
        finally:
            fb.fly_set_tuning("gemm_tiled", 0)
            fb.fly_set_tuning("tiled_phase", 0)
        check_lmhead(got, ref, 2e-3)


@pytest.mark.parametrize("M,d,V,tiles", [(129, 256, 2048 + 48, 0), (160, 96, 16 * 131, 5), (161, 544, 1040, 6),
                                         (192, 32, 16, 6), (200, 320, 4096 + 16, 0), (256, 64, 272, 8),
                                         (97, 160, 528, 5), (140, 128, 256, 8), (81, 256, 2048 + 48, 0),
                                         (96, 96, 16 * 131, 3), (128, 544, 1040, 4), (110, 64, 272, 0)])
@pytest.mark.parametrize("phase", [1, 2])
def test_lmhead_bf16_wide_rows(fb, M, d, V, tiles, phase):
    """81..256 rows take the weight-streaming kernel with 32 x 32 tiles (3 to 8 row tiles per
    wave): ragged last tile, a vocabulary that is not a multiple of the 256-column block, an odd
    number of k-tiles, fewer chunks than the register ring is deep; with half of the waves
    requesting their loads after multiplying (phase 1) and with every wave requesting first (2)."""
    fb.fly_set_tuning("gemm_wide", tiles)
    fb.fly_set_tuning("wide_phase", phase)
    try:
        got, ref = lmhead_case(fb, M, d, V, "bf16", hidden_std=4.0, seed=5)
    finally:
        fb.fly_set_tuning("gemm_wide", 0)
        fb.fly_set_tuning("wide_phase", 0)
    check_lmhead(got, ref, 2e-3)


def test_lmhead_planted_argmax_and_ties(fb):
    V, d, M = 8192, 64, 8
    cols = [0, 15, 16, 255, 256, 4095, 8190, 8191]

    for dtype in ("f32", "bf16"):
        tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
        hidden = torch.zeros(M, d, dtype=tdt, device="cuda")
        w = synth.hash_normal(3, 203, (d, V), 0.02, tdt, "cuda")
        w[:M, :] = 0.0
        for m, c in enumerate(cols):
            hidden[m, m] = 1.0            # row m reads row m of W
            w[m, c] = 2.0                 # unique maximum at column c
        # exact ties: same value at a later column must not move the argmax
        for m, c in enumerate(cols):
            if c + 17 < V:
                w[m, c + 17] = 2.0
        code = fb.dtype_code(dtype)
        wp = torch.empty(fb.fly_packed_weight_bytes(d, V, code) // w.element_size(), dtype=tdt, device="cuda")
        fb.fly_pack_weight(w, wp, V)
        argmax = torch.zeros(M, dtype=torch.int32, device="cuda")
        p1, hn, lse = (torch.zeros(M, dtype=torch.float32, device="cuda") for _ in range(3))
        ws = fb.alloc_workspace(fb.fly_lmhead_workspace_bytes(M, d, V, code))
        fb.fly_lmhead_entropy_argmax(hidden, wp, None, V, argmax, p1, hn, lse, ws)
        torch.cuda.synchronize()
        assert argmax.cpu().tolist() == cols, dtype
        ref = O.decision_statistics(O.lm_head_logits(hidden.cpu().double(), w.cpu().double(), None))
        assert ref["argmax"].tolist() == cols
        assert np.abs(hn.cpu().numpy() - ref["h"]).max() < 1e-4


def test_lmhead_closed_forms(fb):
    """Zero hidden state -> uniform row: h = 1, p_top1 = 1/V, argmax = 0, lse = ln V."""
    for dtype, V in (("f32", 8192), ("bf16", 128256)):
        tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
        M, d = 3, 64
        hidden = torch.zeros(M, d, dtype=tdt, device="cuda")
        w = synth.hash_normal(4, 204, (d, V), 0.02, tdt, "cuda")
        code = fb.dtype_code(dtype)
        wp = torch.empty(fb.fly_packed_weight_bytes(d, V, code) // w.element_size(), dtype=tdt, device="cuda")
        fb.fly_pack_weight(w, wp, V)
        argmax = torch.zeros(M, dtype=torch.int32, device="cuda")
        p1, hn, lse = (torch.zeros(M, dtype=torch.float32, device="cuda") for _ in range(3))
        ws = fb.alloc_workspace(fb.fly_lmhead_workspace_bytes(M, d, V, code))
        fb.fly_lmhead_entropy_argmax(hidden, wp, None, V, argmax, p1, hn, lse, ws)
        torch.cuda.synchronize()
        assert argmax.cpu().tolist() == [0, 0, 0]
        assert np.abs(hn.cpu().numpy() - 1.0).max() < 1e-5
        assert np.abs(p1.cpu().numpy() * V - 1.0).max() < 1e-4
        assert np.abs(lse.cpu().numpy() - math.log(V)).max() < 1e-4
