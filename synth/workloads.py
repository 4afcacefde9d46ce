"""Workload presets and a stateless, device-independent random generator.

Every tensor element is a pure function of (seed, tensor_id, flat_index):
a 64-bit integer hash, an approximately normal variate built from the sum of
eight 16-bit lanes of two hash words (Irwin-Hall, exact integer arithmetic),
one fp32 multiply, and for bf16 tensors one round-to-nearest-even conversion.
All steps are integer ops or single correctly rounded fp32 ops, so the same
call gives bit-identical tensors on the CPU and on a GPU, and any slice of a
tensor can be regenerated without materialising the rest.

Nothing here knows about the verification step itself: no norms, no GEMMs,
no softmax, no acceptance logic.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, Tuple

import torch

# --------------------------------------------------------------------------
# Workload presets (the five configurations the measurements are quoted on).
# --------------------------------------------------------------------------


@dataclasses.dataclass(frozen=True)
class VerifyConfig:
    name: str
    n_layers: int
    d: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    vocab: int
    dtype: str  # "f32" or "bf16": storage type of weights, KV cache, activations
    batch: int  # B sequences
    K: int  # draft tokens per sequence
    kv_len: int  # cached prefix length L (same for every sequence)
    p_match: float  # probability a draft equals the target's argmax
    temperatures: Tuple[float, ...]  # per-position temperature choices
    theta: float = 0.3  # entropy threshold (paper default, Implementation Details)
    window: int = 6  # deferred window length W (paper default)
    rope_theta: float = 500000.0
    rms_eps: float = 1e-5
    weight_std: float = 0.02
    seed: int = 2511_22972
    logit_gain: float = 1.0  # extra multiplier on row_scale (tests only)

    @property
    def M(self) -> int:
        return self.batch * (self.K + 1)

    @property
    def q_dim(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self) -> int:
        return self.n_kv_heads * self.head_dim

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    def replace(self, **kw) -> "VerifyConfig":
        return dataclasses.replace(self, **kw)


CONFIGS: Dict[str, VerifyConfig] = {
    # Tiny fp32 step.
    "c1_tiny": VerifyConfig(
        name="c1_tiny", n_layers=2, d=256, n_q_heads=4, n_kv_heads=2, head_dim=64,
        ffn=688, vocab=8192, dtype="f32", batch=1, K=4, kv_len=128, p_match=0.6,
        temperatures=(0.3, 1.0, 3.0)),
    # Llama-3.1-8B shapes.
    "c2_8b": VerifyConfig(
        name="c2_8b", n_layers=32, d=4096, n_q_heads=32, n_kv_heads=8, head_dim=128,
        ffn=14336, vocab=128256, dtype="bf16", batch=1, K=8, kv_len=2048, p_match=0.7,
        temperatures=(1.0,)),
    # Llama-3.1-70B shapes on one GPU.
    "c3_70b": VerifyConfig(
        name="c3_70b", n_layers=80, d=8192, n_q_heads=64, n_kv_heads=8, head_dim=128,
        ffn=28672, vocab=128256, dtype="bf16", batch=4, K=8, kv_len=4096, p_match=0.7,
        temperatures=(0.3, 1.0, 3.0)),
    # Llama-3.1-405B slice: 8 of 126 layers plus the full LM head.
    "c4_405b_slice": VerifyConfig(
        name="c4_405b_slice", n_layers=8, d=16384, n_q_heads=128, n_kv_heads=8,
        head_dim=128, ffn=53248, vocab=128256, dtype="bf16", batch=8, K=16,
        kv_len=8192, p_match=0.75, temperatures=(1.0,)),
    # LM-head / acceptance stress (hidden states are inputs; attention part uses
    # the 70B head geometry over a 32768-token cache, one layer).
    "c5_stress": VerifyConfig(
        name="c5_stress", n_layers=1, d=8192, n_q_heads=64, n_kv_heads=8, head_dim=128,
        ffn=28672, vocab=128256, dtype="bf16", batch=64, K=16, kv_len=32768,
        p_match=0.5, temperatures=(0.1, 10.0)),
    # The paper's own block sizes (Implementation Details: K=15 for the 70B target,
    # K=25 for the 405B one, batch 1) and the largest batch of its serving table
    # (batch 16).  The prompt length is not stated there: 1024 cached tokens.
    "p70b_k15": VerifyConfig(
        name="p70b_k15", n_layers=80, d=8192, n_q_heads=64, n_kv_heads=8, head_dim=128,
        ffn=28672, vocab=128256, dtype="bf16", batch=1, K=15, kv_len=1024, p_match=0.7,
        temperatures=(0.3, 1.0, 3.0)),
    "p70b_k15_b16": VerifyConfig(
        name="p70b_k15_b16", n_layers=80, d=8192, n_q_heads=64, n_kv_heads=8, head_dim=128,
        ffn=28672, vocab=128256, dtype="bf16", batch=16, K=15, kv_len=1024, p_match=0.7,
        temperatures=(0.3, 1.0, 3.0)),
    "p405b_k25_slice": VerifyConfig(
        name="p405b_k25_slice", n_layers=8, d=16384, n_q_heads=128, n_kv_heads=8,
        head_dim=128, ffn=53248, vocab=128256, dtype="bf16", batch=1, K=25,
        kv_len=1024, p_match=0.75, temperatures=(1.0,)),
}

# Tensor identifiers: one integer per logical tensor; layer tensors add
# 64 * (layer + 1) so every (tensor, layer) pair has its own stream.
TENSOR_IDS = {
    "embed": 1, "w_lm": 2, "g_final": 3,
    "wq": 10, "wk": 11, "wv": 12, "wo": 13, "wg": 14, "wu": 15, "wd": 16,
    "g_attn": 17, "g_ffn": 18,
    "kv_k": 30, "kv_v": 31,
    "temperature": 40, "first_token": 41, "draft_match": 42, "draft_token": 43,
    "draft_kind": 44, "hidden": 45,
}

# --------------------------------------------------------------------------
# Counter-based generator (integer only until the final scale).
# --------------------------------------------------------------------------

_MASK64 = (1 << 64) - 1


def _as_i64(u: int) -> int:
    """Two's-complement int64 value of an unsigned 64-bit constant."""
    u &= _MASK64
    return u - (1 << 64) if u >= (1 << 63) else u


_C_GOLDEN = _as_i64(0x9E3779B97F4A7C15)
_C_MIX1 = _as_i64(0xBF58476D1CE4E5B9)
_C_MIX2 = _as_i64(0x94D049BB133111EB)


def _lsr(z: torch.Tensor, s: int) -> torch.Tensor:
    """Logical right shift of an int64 tensor."""
    return (z >> s) & ((1 << (64 - s)) - 1)


def _mix64(z: torch.Tensor) -> torch.Tensor:
    """A 64-bit finalising bijection (xor-shift / multiply rounds, wrap-around)."""
    z = (z ^ _lsr(z, 30)) * _C_MIX1
    z = (z ^ _lsr(z, 27)) * _C_MIX2
    return z ^ _lsr(z, 31)


def _mix64_int(z: int) -> int:
    z &= _MASK64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK64
    return z ^ (z >> 31)


def _stream_key(seed: int, tensor_id: int) -> int:
    return _as_i64(_mix64_int(_mix64_int(seed) ^ (tensor_id * 0x9E3779B97F4A7C15)))


def _hash_words(seed: int, tensor_id: int, start: int, count: int, word: int,
                device) -> torch.Tensor:
    """64-bit hash word number `word` for flat indices start..start+count-1."""
    idx = torch.arange(start, start + count, dtype=torch.int64, device=device)
    z = idx * 4 + word
    z = z * _C_GOLDEN + _stream_key(seed, tensor_id)
    return _mix64(z)


def _lane_sum16(h: torch.Tensor) -> torch.Tensor:
    return ((h & 0xFFFF) + (_lsr(h, 16) & 0xFFFF) + (_lsr(h, 32) & 0xFFFF)
            + (_lsr(h, 48) & 0xFFFF))


_IH_MEAN = 8 * 32767.5  # mean of the sum of eight uniform 16-bit integers
_IH_STD = math.sqrt(8 * (65536.0 ** 2 - 1.0) / 12.0)

_CHUNK = 1 << 25  # elements generated per pass (bounds temporary memory)


def hash_normal(seed: int, tensor_id: int, shape, std: float, dtype: torch.dtype,
                device="cpu", out: torch.Tensor | None = None) -> torch.Tensor:
    """Approximately N(0, std^2) tensor, bit-identical on every device."""
    n = int(math.prod(shape))
    if out is None:
        out = torch.empty(n, dtype=dtype, device=device)
    flat = out.view(-1)
    scale = torch.tensor(std / _IH_STD, dtype=torch.float32, device=device)
    for start in range(0, n, _CHUNK):
        cnt = min(_CHUNK, n - start)
        s = _lane_sum16(_hash_words(seed, tensor_id, start, cnt, 0, device))
        s = s + _lane_sum16(_hash_words(seed, tensor_id, start, cnt, 1, device))
        # 2*sum - 2*mean is an exact integer below 2^21: exact in fp32.
        centred = (2 * s - int(2 * _IH_MEAN)).to(torch.float32)
        val = centred * (scale * 0.5)
        flat[start:start + cnt] = val.to(dtype)
    return out.view(*shape)


def hash_uniform(seed: int, tensor_id: int, n: int, device="cpu") -> torch.Tensor:
    """float64 uniforms k / 2^24, k in [0, 2^24): exactly representable."""
    h = _hash_words(seed, tensor_id, 0, n, 2, device)
    return (_lsr(h, 40)).to(torch.float64) / float(1 << 24)


def hash_tokens(seed: int, tensor_id: int, n: int, vocab: int, device="cpu") -> torch.Tensor:
    """int32 token ids uniform over [0, vocab) (48-bit hash modulo vocab)."""
    h = _hash_words(seed, tensor_id, 0, n, 3, device)
    return (_lsr(h, 16) % vocab).to(torch.int32)


# --------------------------------------------------------------------------
# Tensors of one verification workload.
# --------------------------------------------------------------------------


def _torch_dtype(cfg: VerifyConfig) -> torch.dtype:
    return torch.float32 if cfg.dtype == "f32" else torch.bfloat16


def layer_weight_shapes(cfg: VerifyConfig) -> Dict[str, Tuple[int, int]]:
    """Canonical (unpacked) weight shapes, all [in_features, out_features]."""
    return {
        "wq": (cfg.d, cfg.q_dim), "wk": (cfg.d, cfg.kv_dim), "wv": (cfg.d, cfg.kv_dim),
        "wo": (cfg.q_dim, cfg.d), "wg": (cfg.d, cfg.ffn), "wu": (cfg.d, cfg.ffn),
        "wd": (cfg.ffn, cfg.d),
    }


def make_weight(cfg: VerifyConfig, name: str, layer: int = -1, device="cpu") -> torch.Tensor:
    """One canonical weight tensor.

    Matrices are [in_features, out_features] row-major ("x @ W"), entries
    ~N(0, weight_std^2); norm gains are all ones; `embed` is [vocab, d]; `w_lm`
    is [d, vocab].
    """
    dt = _torch_dtype(cfg)
    if name in ("g_attn", "g_ffn", "g_final"):
        return torch.ones(cfg.d, dtype=dt, device=device)
    if name == "embed":
        shape = (cfg.vocab, cfg.d)
    elif name == "w_lm":
        shape = (cfg.d, cfg.vocab)
    else:
        shape = layer_weight_shapes(cfg)[name]
    tid = TENSOR_IDS[name] + (64 * (layer + 1) if layer >= 0 else 0)
    return hash_normal(cfg.seed, tid, shape, cfg.weight_std, dt, device)


def make_kv_prefix(cfg: VerifyConfig, layer: int, device="cpu"):
    """Cached prefix keys and values of one layer, each [B, L, Hkv, hd], ~N(0,1).

    The keys are defined to be already position-rotated.
    """
    dt = _torch_dtype(cfg)
    shape = (cfg.batch, cfg.kv_len, cfg.n_kv_heads, cfg.head_dim)
    k = hash_normal(cfg.seed, TENSOR_IDS["kv_k"] + 64 * (layer + 1), shape, 1.0, dt, device)
    v = hash_normal(cfg.seed, TENSOR_IDS["kv_v"] + 64 * (layer + 1), shape, 1.0, dt, device)
    return k, v


def make_row_temperature(cfg: VerifyConfig, device="cpu") -> torch.Tensor:
    """Per-row temperature T[B, K+1] (float32).

    Two listed temperatures: log-uniform between them; otherwise a uniform
    pick from the listed values.  Rows' logits are later divided by T.
    """
    u = hash_uniform(cfg.seed, TENSOR_IDS["temperature"], cfg.M, device)
    temps = cfg.temperatures
    if len(temps) == 2:
        lo, hi = math.log(temps[0]), math.log(temps[1])
        t = torch.exp(lo + u * (hi - lo))
    else:
        pick = torch.clamp((u * len(temps)).to(torch.int64), max=len(temps) - 1)
        t = torch.tensor(temps, dtype=torch.float64, device=device)[pick]
    return t.to(torch.float32).view(cfg.batch, cfg.K + 1)


def make_first_tokens(cfg: VerifyConfig, device="cpu") -> torch.Tensor:
    """The last token of the previous round, y_{-1}, per sequence: int32 [B]."""
    return hash_tokens(cfg.seed, TENSOR_IDS["first_token"], cfg.batch, cfg.vocab, device)


def make_draft_draws(cfg: VerifyConfig, device="cpu"):
    """Random draws that turn a target-argmax chain into draft tokens.

    Returns (u_match float64 [B,K], alt_token int32 [B,K], u_kind float64 [B,K]).
    Draft i equals the target's argmax when u_match < p_match, else alt_token.
    u_kind is a spare uniform for three-way draws (argmax / second best /
    uniform) in the LM-head stress workload.
    """
    n = cfg.batch * cfg.K
    u = hash_uniform(cfg.seed, TENSOR_IDS["draft_match"], n, device).view(cfg.batch, cfg.K)
    alt = hash_tokens(cfg.seed, TENSOR_IDS["draft_token"], n, cfg.vocab, device).view(cfg.batch, cfg.K)
    kind = hash_uniform(cfg.seed, TENSOR_IDS["draft_kind"], n, device).view(cfg.batch, cfg.K)
    return u, alt, kind


def make_hidden(cfg: VerifyConfig, rows: int, device="cpu") -> torch.Tensor:
    """Stand-alone hidden states [rows, d] ~N(0,1) for LM-head / layer tests."""
    return hash_normal(cfg.seed, TENSOR_IDS["hidden"], (rows, cfg.d), 1.0, _torch_dtype(cfg), device)
