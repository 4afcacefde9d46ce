"""CPU oracle for the FLy verification step.  TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 restatement of what the verification step computes,
written from the FLy paper (arxiv 2511.22972) and from the textbook definition
of a pre-norm Llama-style decoder.  It exists so that the HIP kernels have
something independent to be compared with.  It shares no code, table or
helper with the HIP path and must never be imported by the product package;
only tests, the smoke check and the benchmark's CPU-baseline leg use it.

Parts and what fixes them:
  * acceptance rule            -- paper Sec. 2.1-2.2, Eqs. 2-11, and Algorithm 1;
                                  three independently written forms.
  * row statistics             -- Eq. 1 (softmax, argmax) and Eq. 5 (normalised
                                  entropy), literal sums in fp64.
  * decoder forward            -- the paper treats the target model as a black
                                  box (Sec. 2.1, Algorithm 1 step 2); the
                                  arithmetic here is the standard pre-RMSNorm,
                                  rotary, grouped-query, SwiGLU decoder.

Pins (tests/test_oracle_*.py): closed forms of Eq. 5, the limit statements of
the ablation section (theta=1, theta=0, W=0), the boundary rule j+W>K, brute
force over all mismatch/gate patterns, scipy's logsumexp/entropy, torch's
scaled_dot_product_attention, and the Hugging Face Llama implementation run
in fp64 on a tiny model.  The bf16 mode (`Numerics("bf16")`) is pinned by a
two-key example worked by hand, by its invariance under integer octave shifts
of the scores (and its change under half an octave), by exactness when every
unnormalised probability is a power of two, by the one-rounding-per-term error
bound against torch's softmax, and by the list of tensors it rounds, each of
which matters (tests/test_oracle_bf16_pins.py).

  * prompt-lookup drafting     -- Sec. 2.3 names n-gram retrieval over the
                                  context as the parameter-free drafter and gives
                                  no parameters; the rule written out in
                                  `pld_propose` is this build's reading.  Pinned
                                  by an independently written search and by the
                                  exact continuation of periodic sequences.
  * decode loop                -- Algorithm 1's outer loop with the KV cache
                                  rolled forward by s per round, tau = s/t
                                  (Eq. 12).  Pinned by the fact that with the gate
                                  always strict the output is the target's own
                                  greedy continuation.
  * drafting with a model      -- Algorithm 1 step 1 with a draft model M_D
                                  (the paper's own setting: a small model of the
                                  same family): K greedy tokens of M_D after the
                                  sequence so far.  `model_draft_greedy` states it
                                  as K full passes over the growing sequence;
                                  pinned by an incremental, cache-carrying
                                  evaluation (causality) and by the lossless
                                  property of the strict loop.
  * sampled target tokens      -- the paper reports results at temperature 1
                                  (Tables 1-2) but states its rule with the
                                  argmax only (Eqs. 1-2).  This build's reading:
                                  y_i is drawn from softmax(l_i / T) and takes
                                  the argmax's place in Eq. 2; the entropy gate
                                  reads the same tempered distribution.  The
                                  draw is the Gumbel-max construction over a
                                  Philox4x32-10 stream (`sample_rows`).  Pinned by
                                  the generator's published known-answer vectors,
                                  by a chi-square test of the draws against the
                                  softmax probabilities, and by the limits T -> 0
                                  (the argmax) and a one-hot row.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np
import torch

# ==========================================================================
# 1. Acceptance rule (paper Sec. 2.1-2.2).  Positions are 1-based as in the
#    paper: draft[j-1] is y-hat_j, target[j-1] is y_j (j = 1..K+1),
#    h[j-1] is h_j.
# ==========================================================================


def match_indicator(draft: Sequence[int], target: Sequence[int]) -> List[int]:
    """Delta_i = 1[draft_i == target_i], 1 <= i <= K  (Eq. 2)."""
    K = len(draft)
    return [1 if int(draft[i]) == int(target[i]) else 0 for i in range(K)]


def s_standard(delta: Sequence[int]) -> int:
    """Exact-match speculative decoding count (Eq. 3): the index of the first
    mismatch, or K+1 when every draft matches."""
    K = len(delta)
    for i in range(1, K + 1):
        if delta[i - 1] == 0:
            return i
    return K + 1


def accept_equations(delta: Sequence[int], h: Sequence[float], theta: float,
                     W: int) -> Tuple[int, int, int]:
    """(s_gate, s_defer, s_FLy) computed set-wise from Eqs. 4-11.

    Every quantity is built for all j in J first; the minima are taken last.
    """
    K = len(delta)
    J = [j for j in range(1, K + 1) if delta[j - 1] == 0]  # Eq. 4

    # Eq. 6: gate label per mismatch.
    gate = {j: ("Strict" if h[j - 1] < theta else "Defer") for j in J}
    strict = [j for j in J if gate[j] == "Strict"]
    s_gate = min(strict) if strict else K + 1  # Eq. 7

    # Eqs. 8-9.  The window must fit inside the K drafts (boundary rule of
    # Sec. 2.2); that is tested before the sum so no Delta beyond K is read.
    decide = {}
    for j in J:
        if h[j - 1] >= theta and j + W <= K:
            n_w = sum(1 - delta[i - 1] for i in range(j + 1, j + W + 1))  # Eq. 8
            decide[j] = "Accept" if n_w == 0 else "Reject"
        else:
            decide[j] = "Reject"
    rejected = [j for j in J if decide[j] == "Reject"]
    s_defer = min(rejected) if rejected else K + 1  # Eq. 10

    return s_gate, s_defer, min(s_gate, s_defer)  # Eq. 11


def accept_algorithm(draft: Sequence[int], target: Sequence[int], h: Sequence[float],
                     theta: float, W: int) -> Tuple[int, List[int]]:
    """One round of Algorithm 1, steps 2-4: walk the mismatches in ascending
    order and stop at the first rejected one.

    Returns (s, emitted): s is the paper's accepted count for the round (it
    includes the correction or bonus token) and `emitted` the s tokens
    appended to the sequence.
    """
    K = len(draft)
    delta = match_indicator(draft, target)
    for j in range(1, K + 1):
        if delta[j - 1] == 1:
            continue
        if h[j - 1] < theta:  # strict: reject here
            return j, [int(t) for t in draft[: j - 1]] + [int(target[j - 1])]
        if j + W > K:  # window does not fit: reject here
            return j, [int(t) for t in draft[: j - 1]] + [int(target[j - 1])]
        later_mismatches = 0
        for i in range(j + 1, j + W + 1):
            later_mismatches += 1 - delta[i - 1]
        if later_mismatches != 0:
            return j, [int(t) for t in draft[: j - 1]] + [int(target[j - 1])]
        # mismatch at j is kept (as the draft's token); go on to the next one
    return K + 1, [int(t) for t in draft] + [int(target[K])]


def accept_predicate(delta: Sequence[int], h: Sequence[float], theta: float, W: int) -> int:
    """Third form: a per-position reject predicate, s = first position where
    it holds (K+1 if none).

        rej(j) = not Delta_j and (h_j < theta  or  j + W > K
                                  or  exists i in (j, j+W]: not Delta_i)
    """
    K = len(delta)
    mism = 0
    for j in range(1, K + 1):
        if delta[j - 1] == 0:
            mism |= 1 << j
    for j in range(1, K + 1):
        if not (mism >> j) & 1:
            continue
        if h[j - 1] < theta or j + W > K:
            return j
        window_bits = ((1 << W) - 1) << (j + 1)
        if mism & window_bits:
            return j
    return K + 1


def accept_block(draft, target, h, theta: float, W: int) -> Dict[str, np.ndarray]:
    """Batch wrapper in the exported convention.

    draft [B,K] int, target [B,K+1] int, h [B,K+1] (only the first K columns
    are used; the bonus row takes no part in the rule).  The gate compares in
    float32, the type the entropies are produced in.
    Returns accept_len = s-1 (draft tokens kept), next_token = y_s,
    n_loose = mismatching drafts kept, s = the paper's count.
    """
    draft = np.asarray(draft)
    target = np.asarray(target)
    h32 = np.asarray(h, dtype=np.float32)
    th32 = np.float32(theta)
    B, K = draft.shape
    out = {k: np.zeros(B, dtype=np.int32) for k in ("accept_len", "next_token", "n_loose", "s")}
    for b in range(B):
        s, emitted = accept_algorithm(draft[b], target[b], h32[b], th32, W)
        delta = match_indicator(draft[b], target[b])
        out["s"][b] = s
        out["accept_len"][b] = s - 1
        out["next_token"][b] = emitted[-1]
        out["n_loose"][b] = sum(1 - delta[j - 1] for j in range(1, s))
    return out


# ==========================================================================
# 2. Row statistics (Eq. 1, Eq. 5): literal definitions in fp64.
# ==========================================================================


def row_statistics(logits) -> Dict[str, float]:
    """Statistics of one logit row (fp64).

    argmax  -- lowest index among maxima (Eq. 1)
    margin  -- largest minus second-largest logit (diagnostic for near ties)
    lse     -- log sum exp
    H       -- Shannon entropy in nats, the literal -sum p log p of Eq. 5;
               entries with p == 0 contribute 0
    h       -- H / log V, V = number of columns (Eq. 5)
    p_top1  -- probability of the argmax token
    """
    l = np.asarray(logits, dtype=np.float64)
    V = l.shape[0]
    y = int(np.argmax(l))  # numpy returns the first maximal index
    m = l[y]
    p_unnorm = np.exp(l - m)
    Z = p_unnorm.sum()
    p = p_unnorm / Z
    nz = p > 0
    H = float(-(p[nz] * np.log(p[nz])).sum())
    if V > 1:
        rest = np.delete(l, y)
        margin = float(m - rest.max())
    else:
        margin = float("inf")
    return {"argmax": y, "margin": margin, "lse": float(m + math.log(Z)), "H": H,
            "h": H / math.log(V) if V > 1 else 0.0, "p_top1": float(p[y])}


def block_statistics(logits: np.ndarray) -> Dict[str, np.ndarray]:
    """row_statistics over the rows of an [M, V] array."""
    rows = [row_statistics(r) for r in np.asarray(logits)]
    out = {}
    for key in ("argmax", "margin", "lse", "H", "h", "p_top1"):
        out[key] = np.array([r[key] for r in rows], dtype=np.int64 if key == "argmax" else np.float64)
    return out


# ==========================================================================
# 2b. Drawing the target's token at temperature > 0 (this build's reading of
#     the temperature-1 rows of Tables 1-2: the drawn token replaces the
#     argmax of Eq. 1 in the match indicator of Eq. 2).
# ==========================================================================

_PHILOX_M0, _PHILOX_M1 = 0xD2511F53, 0xCD9E8D57
_PHILOX_W0, _PHILOX_W1 = 0x9E3779B9, 0xBB67AE85


def philox4x32_10(counter: np.ndarray, key: Tuple[int, int]) -> np.ndarray:
    """Philox4x32 with ten rounds (Salmon, Moraes, Dror, Shaw: "Parallel random
    numbers: as easy as 1, 2, 3", SC 2011).  counter [..., 4] uint32 -> [..., 4] uint32.

    One round: (c0, c1, c2, c3) -> (hi(M1 c2) ^ c1 ^ k0, lo(M1 c2), hi(M0 c0) ^ c3 ^ k1,
    lo(M0 c0)); the key advances by the Weyl constants between rounds.
    """
    c = np.asarray(counter, dtype=np.uint64)
    c0, c1, c2, c3 = c[..., 0], c[..., 1], c[..., 2], c[..., 3]
    mask = np.uint64(0xFFFFFFFF)
    sh = np.uint64(32)
    k0, k1 = int(key[0]) & 0xFFFFFFFF, int(key[1]) & 0xFFFFFFFF
    for _ in range(10):
        p0 = np.uint64(_PHILOX_M0) * c0
        p1 = np.uint64(_PHILOX_M1) * c2
        c0, c1, c2, c3 = ((p1 >> sh) ^ c1 ^ np.uint64(k0), p1 & mask,
                          (p0 >> sh) ^ c3 ^ np.uint64(k1), p0 & mask)
        k0 = (k0 + _PHILOX_W0) & 0xFFFFFFFF
        k1 = (k1 + _PHILOX_W1) & 0xFFFFFFFF
    return np.stack([c0, c1, c2, c3], axis=-1).astype(np.uint32)


def sample_bits(M: int, V: int, seed: int, offset: int, rows=None) -> np.ndarray:
    """The 32 random bits of every (row m, column v) of one call: word v % 4 of the
    Philox block with counter (v // 4, m, offset low, offset high) and key
    (seed low, seed high).  `offset` tells calls with the same seed apart.
    `rows` (default 0..M-1) names the rows m of the call that the M output rows stand for."""
    nblk = (V + 3) // 4
    row_ids = np.arange(M, dtype=np.uint64) if rows is None else np.asarray(rows, dtype=np.uint64)
    assert row_ids.shape == (M,)
    ctr = np.zeros((M, nblk, 4), dtype=np.uint64)
    ctr[..., 0] = np.arange(nblk, dtype=np.uint64)[None, :]
    ctr[..., 1] = row_ids[:, None]
    ctr[..., 2] = offset & 0xFFFFFFFF
    ctr[..., 3] = (offset >> 32) & 0xFFFFFFFF
    bits = philox4x32_10(ctr, (seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF))
    return bits.reshape(M, nblk * 4)[:, :V]


def uniform_open01(bits: np.ndarray) -> np.ndarray:
    """u = (top 23 bits + 1/2) / 2^23, strictly inside (0, 1), exact in float32."""
    return ((np.asarray(bits, dtype=np.uint32) >> np.uint32(9)).astype(np.float64) + 0.5) * 2.0 ** -23


def gumbel_noise(bits: np.ndarray) -> np.ndarray:
    """Standard Gumbel variates G = -ln(-ln u)."""
    return -np.log(-np.log(uniform_open01(bits)))


def sample_rows(logits: np.ndarray, seed: int, offset: int, rows=None) -> Dict[str, np.ndarray]:
    """One draw per row from softmax(logits[m]) by the Gumbel-max construction:
    argmax_v (l_v + G_v) with independent standard Gumbel G_v is distributed as
    softmax(l).  The decision is taken in float32 (float32 logits plus float32
    noise), lowest index on ties.

    token   -- the drawn column per row
    margin  -- largest minus second-largest perturbed logit (near-tie diagnostic)
    `rows`: the row numbers within the call, when `logits` holds only some of its rows.
    """
    l = np.asarray(logits, dtype=np.float64)
    M, V = l.shape
    g = gumbel_noise(sample_bits(M, V, seed, offset, rows))
    z = l.astype(np.float32) + g.astype(np.float32)
    token = np.argmax(z, axis=1).astype(np.int64)
    if V > 1:
        part = np.partition(z.astype(np.float64), V - 2, axis=1)
        margin = part[:, V - 1] - part[:, V - 2]
    else:
        margin = np.full(M, np.inf)
    return {"token": token, "margin": margin}


# ==========================================================================
# 3. Decoder forward (textbook pre-norm decoder; shapes come from the
#    workload, the paper only says "a single forward pass", Sec. 2.1).
# ==========================================================================


def round_to_bf16(x: torch.Tensor) -> torch.Tensor:
    """Value-preserving fp64 tensor whose entries are the bf16 roundings of x.

    Two steps, as on the device: the fp64 value is first rounded to fp32 (the
    type the accumulators are held in), then to bf16 by round-to-nearest-even
    on the upper 16 bits.  NaNs are not expected and not handled.
    """
    a = x.detach().to(torch.float64).contiguous().numpy().astype(np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    bias = np.uint64(0x7FFF) + ((u >> np.uint64(16)) & np.uint64(1))
    r = ((u + bias) & np.uint64(0xFFFF0000)).astype(np.uint32)
    return torch.from_numpy(r.view(np.float32).astype(np.float64)).view(x.shape)


def round_to_f32(x: torch.Tensor) -> torch.Tensor:
    return x.to(torch.float32).to(torch.float64)


@dataclasses.dataclass
class Numerics:
    """Where the oracle rounds.

    storage == "f32": nothing is rounded (inputs are fp32 values, all
    arithmetic fp64).
    storage == "bf16": the tensors the device holds in bf16 are rounded to
    bf16 here too -- normalised activations, rotated q/k and v, the
    unnormalised attention probabilities, the attention output, the SwiGLU
    output -- and the rotary cos/sin tables are rounded to fp32.  The residual
    stream, GEMM accumulators and all row statistics are never rounded.
    """
    storage: str = "f32"

    def act(self, x: torch.Tensor) -> torch.Tensor:
        return round_to_bf16(x) if self.storage == "bf16" else x

    def table(self, x: torch.Tensor) -> torch.Tensor:
        return round_to_f32(x) if self.storage == "bf16" else x


def rmsnorm(x: torch.Tensor, g: torch.Tensor, eps: float) -> torch.Tensor:
    """x / sqrt(mean(x^2) + eps) * g along the last axis."""
    ms = (x * x).mean(dim=-1, keepdim=True)
    return x / torch.sqrt(ms + eps) * g


def rope_tables(positions: torch.Tensor, head_dim: int, theta: float):
    """cos/sin of pos * theta^(-2i/hd), i = 0..hd/2-1  ->  each [n_pos, hd/2]."""
    i = torch.arange(head_dim // 2, dtype=torch.float64)
    inv_freq = theta ** (-2.0 * i / head_dim)
    ang = positions.to(torch.float64)[:, None] * inv_freq[None, :]
    return torch.cos(ang), torch.sin(ang)


def apply_rope(x: torch.Tensor, cos: torch.Tensor, sin: torch.Tensor) -> torch.Tensor:
    """Rotate pairs (i, i + hd/2) of x [n_pos, heads, hd] by the position angle."""
    half = x.shape[-1] // 2
    x1, x2 = x[..., :half], x[..., half:]
    c, s = cos[:, None, :], sin[:, None, :]
    return torch.cat([x1 * c - x2 * s, x2 * c + x1 * s], dim=-1)


def silu(x: torch.Tensor) -> torch.Tensor:
    return x / (1.0 + torch.exp(-x))


LOG2E = 1.4426950408889634  # log2(e)


def attention_one_sequence(q: torch.Tensor, k_all: torch.Tensor, v_all: torch.Tensor,
                           prefix_len: int, num: Numerics) -> torch.Tensor:
    """Causal grouped-query attention for the K+1 new rows of one sequence.

    q [R, Hq, hd]; k_all, v_all [prefix_len + R, Hkv, hd] (cached prefix
    followed by the R new rows).  Query row i sees keys 0..prefix_len+i.
    Query head a uses KV head a // (Hq/Hkv).  Returns [R, Hq, hd].
    """
    R, Hq, hd = q.shape
    T, Hkv, _ = k_all.shape
    G = Hq // Hkv
    out = torch.zeros(R, Hq, hd, dtype=torch.float64)
    key_pos = torch.arange(T)
    for a in range(Hq):
        kh = k_all[:, a // G, :]  # [T, hd]
        vh = v_all[:, a // G, :]
        scores = (q[:, a, :] @ kh.T) / math.sqrt(hd)  # [R, T]
        for i in range(R):
            visible = key_pos <= prefix_len + i
            s2 = scores[i][visible] * LOG2E              # exponent in base 2
            # softmax(s) = 2^(s2 - n) / sum 2^(s2 - n) for ANY n.  The device
            # multiplies bf16 probabilities into V, so the unnormalised terms are
            # rounded to bf16; they are taken relative to the integer n = ceil(max s2)
            # (a power-of-two scaling, under which bf16 rounding is exact), and
            # the normalising sum uses the unrounded terms.
            n = torch.ceil(s2.max())
            e = torch.exp2(s2 - n)
            out[i, a, :] = (num.act(e) @ vh[visible]) / e.sum()
    return out


@dataclasses.dataclass
class LayerWeights:
    """Canonical weights of one decoder layer, all [in, out], fp64 tensors."""
    wq: torch.Tensor
    wk: torch.Tensor
    wv: torch.Tensor
    wo: torch.Tensor
    wg: torch.Tensor
    wu: torch.Tensor
    wd: torch.Tensor
    g_attn: torch.Tensor
    g_ffn: torch.Tensor


def decoder_layer(x: torch.Tensor, w: LayerWeights, k_prefix: torch.Tensor,
                  v_prefix: torch.Tensor, n_q_heads: int, n_kv_heads: int, head_dim: int,
                  rope_theta: float, eps: float, num: Numerics):
    """One pre-norm decoder layer over the new rows of ONE sequence.

    x [R, d] residual stream; k_prefix, v_prefix [L, Hkv, hd] cached rows
    (keys already rotated).  Row i sits at absolute position L + i.
    Returns (x_out [R, d], k_new [R, Hkv, hd], v_new [R, Hkv, hd]); the new
    rows are what gets appended to the cache.
    """
    R, d = x.shape
    L = k_prefix.shape[0]
    xn = num.act(rmsnorm(x, w.g_attn, eps))
    q = (xn @ w.wq).view(R, n_q_heads, head_dim)
    k = (xn @ w.wk).view(R, n_kv_heads, head_dim)
    v = (xn @ w.wv).view(R, n_kv_heads, head_dim)
    cos, sin = rope_tables(torch.arange(L, L + R), head_dim, rope_theta)
    cos, sin = num.table(cos), num.table(sin)
    q = num.act(apply_rope(q, cos, sin))
    k = num.act(apply_rope(k, cos, sin))
    v = num.act(v)
    k_all = torch.cat([k_prefix, k], dim=0)
    v_all = torch.cat([v_prefix, v], dim=0)
    o = num.act(attention_one_sequence(q, k_all, v_all, L, num))
    x = x + o.reshape(R, n_q_heads * head_dim) @ w.wo
    xn = num.act(rmsnorm(x, w.g_ffn, eps))
    a = num.act(silu(xn @ w.wg) * (xn @ w.wu))
    x = x + a @ w.wd
    return x, k, v


def lm_head_logits(x_final_normed: torch.Tensor, w_lm: torch.Tensor,
                   row_scale: Optional[torch.Tensor]) -> torch.Tensor:
    """logits[m, v] = (x[m] . W_lm[:, v]) * row_scale[m]."""
    logits = x_final_normed @ w_lm
    if row_scale is not None:
        logits = logits * row_scale.to(torch.float64)[:, None]
    return logits


def decision_statistics(logits: torch.Tensor) -> Dict[str, np.ndarray]:
    """Row statistics with the integer decision taken in float32.

    The argmax is taken over the logits rounded to float32 (the precision the
    device decides in); everything else is fp64 on the unrounded logits.
    """
    l64 = logits.numpy()
    stats = block_statistics(l64)
    l32 = l64.astype(np.float32)
    stats["argmax"] = np.argmax(l32, axis=1).astype(np.int64)
    return stats


def verify_block(tokens, embed: torch.Tensor, layers: Sequence[LayerWeights],
                 g_final: torch.Tensor, w_lm: torch.Tensor,
                 kv_prefix: Sequence[Tuple[torch.Tensor, torch.Tensor]],
                 row_scale: Optional[torch.Tensor], *, n_q_heads: int, n_kv_heads: int,
                 head_dim: int, rope_theta: float, eps: float, theta: float, W: int,
                 storage: str = "f32", return_logits: bool = False,
                 sample: Optional[Tuple[int, int]] = None, sample_row0: int = 0) -> Dict[str, np.ndarray]:
    """The whole verification step for B sequences (Sec. 2.1-2.2, Alg. 1 steps 2-4).

    With sample = (seed, offset) the target's tokens y_1..y_{K+1} are drawn from
    softmax of the scaled logits (`sample_rows`, row m = sample_row0 + b (K+1) + i)
    instead of being their argmax, and the acceptance rule compares the drafts
    with the drawn tokens; "sampled" and "sample_margin" are added to the result.
    sample_row0 lets a block that is part of a larger batch draw what the batch draws.

    tokens [B, K+1] = (y_{-1}, draft_1..draft_K) per sequence.
    kv_prefix[layer] = (k [B, L, Hkv, hd], v [B, L, Hkv, hd]).
    All tensors are fp64 holding values representable in the storage type.
    """
    num = Numerics(storage)
    tokens = np.asarray(tokens)
    B, R = tokens.shape
    K = R - 1
    d = embed.shape[1]
    logits_all = []
    new_kv = []
    for b in range(B):
        x = embed[torch.from_numpy(tokens[b].astype(np.int64))].clone()
        seq_kv = []
        for li, w in enumerate(layers):
            kp, vp = kv_prefix[li]
            x, k_new, v_new = decoder_layer(x, w, kp[b], vp[b], n_q_heads, n_kv_heads,
                                            head_dim, rope_theta, eps, num)
            seq_kv.append((k_new, v_new))
        xn = num.act(rmsnorm(x, g_final, eps))
        rs = None if row_scale is None else row_scale.reshape(B, R)[b]
        logits_all.append(lm_head_logits(xn, w_lm, rs))
        new_kv.append(seq_kv)
    logits = torch.stack(logits_all)  # [B, R, V]
    stats = decision_statistics(logits.reshape(B * R, -1))
    out = {k: v.reshape(B, R) for k, v in stats.items()}
    target = out["argmax"]
    if sample is not None:
        drawn = sample_rows(logits.reshape(B * R, -1).numpy(), sample[0], sample[1],
                            rows=sample_row0 + np.arange(B * R))
        out["sampled"] = drawn["token"].reshape(B, R)
        out["sample_margin"] = drawn["margin"].reshape(B, R)
        target = out["sampled"]
    acc = accept_block(tokens[:, 1:], target, out["h"], theta, W)
    out.update(acc)
    out["new_kv"] = new_kv
    if return_logits:
        out["logits"] = logits.numpy()
    return out


# ==========================================================================
# 4. Drafting by prompt lookup and the decode loop (Sec. 2.3; Algorithm 1)
# ==========================================================================

def pld_propose(y: Sequence[int], n_max: int, K: int) -> Tuple[List[int], int]:
    """K draft tokens for the sequence y by n-gram retrieval (Sec. 2.3).

    The paper names the method and no parameters; the reading taken:
      * for n = n_max, n_max-1, .., 1 look for an earlier occurrence of the last
        n tokens of y, i.e. an end position e < len(y) with y[e-n:e] == y[-n:];
        the longest n that occurs wins, and among its occurrences the latest;
      * the drafts are the tokens that followed that occurrence; where the
        continuation runs past the end of y it goes on through the drafts
        already written (so a periodic sequence is continued periodically);
      * without any occurrence the last token is repeated K times.
    Returns (drafts, n) with n = 0 for "no occurrence".
    """
    y = [int(t) for t in y]
    L = len(y)
    assert L >= 1 and n_max >= 1 and K >= 1
    for n in range(min(n_max, L - 1), 0, -1):
        pattern = y[L - n:]
        for e in range(L - 1, n - 1, -1):     # latest occurrence first
            if y[e - n:e] == pattern:
                ext = list(y)
                for i in range(K):
                    ext.append(ext[e + i])
                return ext[L:], n
    return [y[-1]] * K, 0


def model_draft_greedy(y: Sequence[int], K: int, embed: torch.Tensor, layers: Sequence[LayerWeights],
                       g_final: torch.Tensor, w_lm: torch.Tensor,
                       kv_prefix: Sequence[Tuple[torch.Tensor, torch.Tensor]], first_pos: int, *,
                       n_q_heads: int, n_kv_heads: int, head_dim: int, rope_theta: float, eps: float,
                       storage: str = "f32", return_margins: bool = False):
    """Algorithm 1 step 1 with a draft model M_D: the K tokens M_D emits greedily
    after the sequence y (Sec. 2.1: the drafter proposes, the target verifies).

    kv_prefix[layer] = (k [P, Hkv, hd], v [P, Hkv, hd]) is M_D's cache of the
    positions before first_pos (P >= first_pos; only the first first_pos rows are
    read); M_D itself processes the tokens y[first_pos:].  Draft i is the argmax
    (Eq. 1, lowest index on ties) of M_D's distribution after y and the drafts so
    far.  Written as K full passes over the growing block: no cache is carried
    from one draft to the next.  With return_margins also the top-2 logit margin
    behind every draft (a comparison may skip what hinges on a near tie).
    """
    assert 0 <= first_pos < len(y) and K >= 1
    prefix = [(k[None, :first_pos], v[None, :first_pos]) for k, v in kv_prefix]
    toks = [int(t) for t in y[first_pos:]]
    drafts: List[int] = []
    margins: List[float] = []
    for _ in range(K):
        block = toks + drafts
        if len(block) < 2:                       # verify_block wants at least one position after y_{-1}
            block = block + [0]                  # a dummy last position: causal, so it changes nothing before it
            pos = len(block) - 2
        else:
            pos = len(block) - 1
        out = verify_block(np.asarray([block], dtype=np.int64), embed, layers, g_final, w_lm, prefix, None,
                           n_q_heads=n_q_heads, n_kv_heads=n_kv_heads, head_dim=head_dim,
                           rope_theta=rope_theta, eps=eps, theta=2.0, W=0, storage=storage)
        drafts.append(int(out["argmax"][0, pos]))
        margins.append(float(out["margin"][0, pos]))
    return (drafts, margins) if return_margins else drafts


def decode_rounds(y0: Sequence[int], kv0: Sequence[Tuple[torch.Tensor, torch.Tensor]],
                  embed: torch.Tensor, layers: Sequence[LayerWeights], g_final: torch.Tensor,
                  w_lm: torch.Tensor, row_scale: Optional[torch.Tensor], *, rounds: int, K: int,
                  n_max: int, theta: float, W: int, n_q_heads: int, n_kv_heads: int,
                  head_dim: int, rope_theta: float, eps: float, storage: str = "f32",
                  drafter=None, sample: Optional[Tuple[int, int]] = None, sample_row0: int = 0) -> Dict:
    """Algorithm 1's loop for ONE sequence, `rounds` rounds (no end-of-sequence
    token in the synthetic setting), with `pld_propose` as the drafter (or
    `drafter(y, K) -> (drafts, tag)` when given: Algorithm 1 takes any M_D).

    y0: the sequence so far; its last token is y_{-1}, not yet in the cache.
    kv0[layer] = (k [L, Hkv, hd], v [L, Hkv, hd]): the cache of everything
    before y_{-1}.  Each round keeps s = (kept drafts + 1) tokens: the cache
    grows by the rows of (y_{-1}, kept drafts) -- the rows computed from the
    tokens that ARE in the output, also where a kept draft differs from the
    target's own choice -- and the correction / bonus token becomes the next
    y_{-1}.  Returns the final sequence, s per round, tau = sum(s) / rounds
    (Eq. 12), the per-round statistics and the final cache.

    With sample = (seed, offset) the target's tokens are drawn (see `verify_block`):
    round r uses offset + r, rows sample_row0 .. sample_row0 + K of the draw.
    """
    y = [int(t) for t in y0]
    kv = [(k.clone(), v.clone()) for k, v in kv0]
    trace, loose, per_round = [], [], []
    for rnd in range(rounds):
        drafts, n = pld_propose(y, n_max, K) if drafter is None else drafter(y, K)
        tokens = np.asarray([[y[-1]] + drafts], dtype=np.int64)
        out = verify_block(tokens, embed, layers, g_final, w_lm,
                           [(k[None], v[None]) for k, v in kv], row_scale,
                           n_q_heads=n_q_heads, n_kv_heads=n_kv_heads, head_dim=head_dim,
                           rope_theta=rope_theta, eps=eps, theta=theta, W=W, storage=storage,
                           sample=None if sample is None else (sample[0], sample[1] + rnd),
                           sample_row0=sample_row0)
        a = int(out["accept_len"][0])
        s = a + 1
        y += drafts[:a] + [int(out["next_token"][0])]
        kv = [(torch.cat([k, nk[:s]]), torch.cat([v, nv[:s]]))
              for (k, v), (nk, nv) in zip(kv, out["new_kv"][0])]
        trace.append(s)
        loose.append(int(out["n_loose"][0]))
        per_round.append({"drafts": drafts, "ngram": n, "argmax": out["argmax"][0].copy(),
                          "h": out["h"][0].copy(), "margin": out["margin"][0].copy()})
        if sample is not None:
            per_round[-1]["sampled"] = out["sampled"][0].copy()
            per_round[-1]["sample_margin"] = out["sample_margin"][0].copy()
    return {"y": y, "s": trace, "tau": sum(trace) / max(rounds, 1), "n_loose": loose,
            "rounds": per_round, "kv": kv}
