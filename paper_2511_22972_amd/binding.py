"""ctypes binding of libfly.so: argument marshalling only.

Every function here has the name of the C entry point it calls
(include/fly.h); torch tensors are used for device memory and streams and
nothing else -- no step of the verification path is computed in Python.
The library must have been built (python -m paper_2511_22972_amd.build);
importing this module without it raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfly.so")

FLY_F32, FLY_BF16 = 0, 1

EXPORTS = [
    "fly_strerror", "fly_set_tuning", "fly_packed_weight_bytes", "fly_pack_weight",
    "fly_workspace_bytes", "fly_lmhead_workspace_bytes", "fly_verify_block", "fly_decoder_layers",
    "fly_lmhead_entropy_argmax", "fly_accept", "fly_attention", "fly_gateup_swiglu", "fly_proj_partial",
    "fly_pld_draft", "fly_decode_workspace_bytes", "fly_decode_rounds",
    "fly_model_draft_workspace_bytes", "fly_model_draft", "fly_decode_model_workspace_bytes",
    "fly_decode_rounds_model", "fly_verify_block_sampled", "fly_lmhead_entropy_sample",
    "fly_decode_rounds_sampled", "fly_lmhead_entropy_argmax_static",
]


class FlyError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} (status {status})")


class fly_model_desc(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("ffn", C.c_int32),
                ("vocab", C.c_int32), ("dtype", C.c_int32), ("rms_eps", C.c_float),
                ("rope_theta", C.c_float)]


class fly_layer_weights(C.Structure):
    _fields_ = [("w_qkv", C.c_void_p), ("w_o", C.c_void_p), ("w_gateup", C.c_void_p),
                ("w_down", C.c_void_p), ("g_attn", C.c_void_p), ("g_ffn", C.c_void_p)]


class fly_weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("layers", C.POINTER(fly_layer_weights)),
                ("g_final", C.c_void_p), ("w_lm", C.c_void_p)]


class fly_kv_cache(C.Structure):
    _fields_ = [("k_layers", C.POINTER(C.c_void_p)), ("v_layers", C.POINTER(C.c_void_p)),
                ("kv_len", C.c_void_p), ("capacity", C.c_int32), ("max_kv_len", C.c_int32)]


class fly_verify_out(C.Structure):
    _fields_ = [("accept_len", C.c_void_p), ("next_token", C.c_void_p), ("kv_len_out", C.c_void_p),
                ("argmax", C.c_void_p), ("h_norm", C.c_void_p), ("p_top1", C.c_void_p),
                ("lse", C.c_void_p), ("n_loose", C.c_void_p), ("hidden_out", C.c_void_p)]


class fly_sequences(C.Structure):
    _fields_ = [("ctx", C.c_void_p), ("ctx_len", C.c_void_p), ("kv_len", C.c_void_p),
                ("ctx_capacity", C.c_int32), ("max_ctx_len", C.c_int32),
                ("accepted_total", C.c_void_p), ("rounds_done", C.c_void_p), ("loose_total", C.c_void_p),
                ("accept_trace", C.c_void_p), ("ngram_trace", C.c_void_p)]


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it first (python -m paper_2511_22972_amd.build). "
            "There is no fallback path.")
    lib = C.CDLL(LIB_PATH)
    lib.fly_strerror.restype = C.c_char_p
    lib.fly_strerror.argtypes = [C.c_int]
    lib.fly_set_tuning.argtypes = [C.c_char_p, C.c_int32]
    lib.fly_packed_weight_bytes.argtypes = [C.c_int64, C.c_int64, C.c_int32, C.POINTER(C.c_size_t)]
    lib.fly_pack_weight.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_int32, C.c_void_p,
                                    C.c_int64, C.c_int64, C.c_int64, C.c_void_p]
    lib.fly_workspace_bytes.argtypes = [C.POINTER(fly_model_desc), C.c_int32, C.c_int32, C.c_int32,
                                        C.POINTER(C.c_size_t)]
    lib.fly_lmhead_workspace_bytes.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                               C.POINTER(C.c_size_t)]
    lib.fly_verify_block.argtypes = [C.POINTER(fly_model_desc), C.POINTER(fly_weights),
                                     C.POINTER(fly_kv_cache), C.c_void_p, C.c_void_p, C.c_int32,
                                     C.c_int32, C.c_float, C.c_int32, C.POINTER(fly_verify_out),
                                     C.c_void_p, C.c_size_t, C.c_void_p]
    lib.fly_verify_block_sampled.argtypes = [C.POINTER(fly_model_desc), C.POINTER(fly_weights),
                                             C.POINTER(fly_kv_cache), C.c_void_p, C.c_void_p, C.c_int32,
                                             C.c_int32, C.c_float, C.c_int32, C.c_uint64, C.c_uint64,
                                             C.c_void_p, C.POINTER(fly_verify_out), C.c_void_p,
                                             C.c_size_t, C.c_void_p]
    lib.fly_lmhead_entropy_sample.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                              C.c_int32, C.c_int32, C.c_uint64, C.c_uint64, C.c_void_p,
                                              C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                              C.c_size_t, C.c_void_p]
    lib.fly_decoder_layers.argtypes = [C.POINTER(fly_model_desc), C.POINTER(fly_weights),
                                       C.POINTER(fly_kv_cache), C.c_void_p, C.c_int32, C.c_int32,
                                       C.c_int32, C.c_int32, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.fly_lmhead_entropy_argmax.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                              C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                              C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.fly_lmhead_entropy_argmax_static.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                                     C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                                     C.c_void_p, C.c_void_p, C.c_void_p]
    lib.fly_accept.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_float,
                               C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.fly_attention.argtypes = [C.POINTER(fly_model_desc), C.POINTER(fly_kv_cache), C.c_int32,
                                  C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_size_t,
                                  C.c_void_p]
    lib.fly_gateup_swiglu.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                      C.c_int32, C.c_int32, C.c_void_p]
    lib.fly_proj_partial.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32,
                                     C.c_int32, C.POINTER(C.c_int32), C.c_size_t, C.c_void_p]
    lib.fly_pld_draft.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                  C.c_void_p, C.c_void_p, C.c_void_p]
    lib.fly_decode_workspace_bytes.argtypes = [C.POINTER(fly_model_desc), C.c_int32, C.c_int32, C.c_int32,
                                               C.POINTER(C.c_size_t)]
    lib.fly_decode_rounds.argtypes = [C.POINTER(fly_model_desc), C.POINTER(fly_weights),
                                      C.POINTER(fly_kv_cache), C.POINTER(fly_sequences), C.c_void_p,
                                      C.c_int32, C.c_int32, C.c_float, C.c_int32, C.c_int32, C.c_int32,
                                      C.c_void_p, C.c_size_t, C.c_void_p]
    lib.fly_decode_rounds_sampled.argtypes = [C.POINTER(fly_model_desc), C.POINTER(fly_weights),
                                              C.POINTER(fly_kv_cache), C.POINTER(fly_sequences), C.c_void_p,
                                              C.c_int32, C.c_int32, C.c_float, C.c_int32, C.c_int32, C.c_int32,
                                              C.c_uint64, C.c_uint64, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.fly_model_draft_workspace_bytes.argtypes = [C.POINTER(fly_model_desc), C.c_int32, C.c_int32, C.c_int32,
                                                    C.POINTER(C.c_size_t)]
    lib.fly_model_draft.argtypes = [C.POINTER(fly_model_desc), C.POINTER(fly_weights), C.POINTER(fly_kv_cache),
                                    C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                    C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.fly_decode_model_workspace_bytes.argtypes = [C.POINTER(fly_model_desc), C.POINTER(fly_model_desc),
                                                     C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_size_t)]
    lib.fly_decode_rounds_model.argtypes = [C.POINTER(fly_model_desc), C.POINTER(fly_weights),
                                            C.POINTER(fly_kv_cache), C.POINTER(fly_model_desc),
                                            C.POINTER(fly_weights), C.POINTER(fly_kv_cache),
                                            C.POINTER(fly_sequences), C.c_void_p, C.c_int32, C.c_int32,
                                            C.c_float, C.c_int32, C.c_int32, C.c_void_p, C.c_size_t, C.c_void_p]
    for name in EXPORTS:
        if name != "fly_strerror":
            getattr(lib, name).restype = C.c_int
    return lib


lib = _load()


def strerror(status: int) -> str:
    return lib.fly_strerror(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != 0:
        raise FlyError(status, where)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream() -> Optional[int]:
    return torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else None


def dtype_code(dtype) -> int:
    if dtype in ("bf16", torch.bfloat16):
        return FLY_BF16
    if dtype in ("f32", torch.float32):
        return FLY_F32
    raise ValueError(f"unsupported dtype {dtype}")


def torch_dtype(code: int) -> torch.dtype:
    return torch.bfloat16 if code == FLY_BF16 else torch.float32


# ---------------------------------------------------------------------------
# Entry points (same names as the C ABI)
# ---------------------------------------------------------------------------

def fly_set_tuning(key: str, value: int) -> None:
    _check(lib.fly_set_tuning(key.encode(), int(value)), "fly_set_tuning")


def fly_packed_weight_bytes(k_in: int, n_dst: int, dtype: int) -> int:
    out = C.c_size_t(0)
    _check(lib.fly_packed_weight_bytes(k_in, n_dst, dtype, C.byref(out)), "fly_packed_weight_bytes")
    return out.value


def fly_pack_weight(src: torch.Tensor, dst: torch.Tensor, n_dst: int, tile_offset: int = 0,
                    tile_stride: int = 1) -> None:
    """src: canonical [k_in, n_src] row-major on the device; dst: flat packed buffer."""
    k_in, n_src = src.shape
    _check(lib.fly_pack_weight(_ptr(src), k_in, n_src, dtype_code(src.dtype), _ptr(dst), n_dst,
                               tile_offset, tile_stride, _stream()), "fly_pack_weight")


def fly_workspace_bytes(desc: fly_model_desc, B: int, K: int, max_kv_len: int) -> int:
    out = C.c_size_t(0)
    _check(lib.fly_workspace_bytes(C.byref(desc), B, K, max_kv_len, C.byref(out)), "fly_workspace_bytes")
    return out.value


def fly_lmhead_workspace_bytes(M: int, d: int, V: int, dtype: int) -> int:
    out = C.c_size_t(0)
    _check(lib.fly_lmhead_workspace_bytes(M, d, V, dtype, C.byref(out)), "fly_lmhead_workspace_bytes")
    return out.value


def fly_accept(draft: torch.Tensor, tgt_argmax: torch.Tensor, h_norm: torch.Tensor, theta: float,
               W: int, accept_len: torch.Tensor, next_token: torch.Tensor,
               n_loose: Optional[torch.Tensor] = None) -> None:
    B, K = draft.shape
    _check(lib.fly_accept(_ptr(draft), _ptr(tgt_argmax), _ptr(h_norm), B, K, theta, W,
                          _ptr(accept_len), _ptr(next_token), _ptr(n_loose), _stream()), "fly_accept")


def fly_lmhead_entropy_argmax(hidden: torch.Tensor, w_lm_packed: torch.Tensor,
                              row_scale: Optional[torch.Tensor], V: int, argmax: torch.Tensor,
                              p_top1: torch.Tensor, h_norm: torch.Tensor,
                              lse: Optional[torch.Tensor], workspace: torch.Tensor) -> None:
    M, d = hidden.shape
    _check(lib.fly_lmhead_entropy_argmax(_ptr(hidden), _ptr(w_lm_packed), _ptr(row_scale), M, d, V,
                                         dtype_code(hidden.dtype), _ptr(argmax), _ptr(p_top1),
                                         _ptr(h_norm), _ptr(lse), _ptr(workspace),
                                         workspace.numel() * workspace.element_size(), _stream()),
           "fly_lmhead_entropy_argmax")


def fly_lmhead_entropy_argmax_static(hidden: torch.Tensor, w_lm_packed: torch.Tensor,
                                     row_scale: Optional[torch.Tensor], V: int, argmax: torch.Tensor,
                                     p_top1: torch.Tensor, h_norm: torch.Tensor,
                                     lse: Optional[torch.Tensor]) -> None:
    M, d = hidden.shape
    _check(lib.fly_lmhead_entropy_argmax_static(_ptr(hidden), _ptr(w_lm_packed), _ptr(row_scale), M, d, V,
                                                dtype_code(hidden.dtype), _ptr(argmax), _ptr(p_top1),
                                                _ptr(h_norm), _ptr(lse), _stream()),
           "fly_lmhead_entropy_argmax_static")


def fly_lmhead_entropy_sample(hidden: torch.Tensor, w_lm_packed: torch.Tensor,
                              row_scale: Optional[torch.Tensor], V: int, seed: int, offset: int,
                              sampled: torch.Tensor, argmax: torch.Tensor, p_top1: torch.Tensor,
                              h_norm: torch.Tensor, lse: Optional[torch.Tensor],
                              workspace: torch.Tensor) -> None:
    M, d = hidden.shape
    _check(lib.fly_lmhead_entropy_sample(_ptr(hidden), _ptr(w_lm_packed), _ptr(row_scale), M, d, V,
                                         dtype_code(hidden.dtype), seed, offset, _ptr(sampled),
                                         _ptr(argmax), _ptr(p_top1), _ptr(h_norm), _ptr(lse),
                                         _ptr(workspace), workspace.numel() * workspace.element_size(),
                                         _stream()), "fly_lmhead_entropy_sample")


# ---------------------------------------------------------------------------
# Holders of device memory (allocation and layout plumbing, no arithmetic)
# ---------------------------------------------------------------------------

def make_desc(cfg) -> fly_model_desc:
    """fly_model_desc from any object with the workload's geometry fields."""
    return fly_model_desc(cfg.n_layers, cfg.d, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.ffn,
                          cfg.vocab, dtype_code(cfg.dtype), cfg.rms_eps, cfg.rope_theta)


class PackedModel:
    """Packed weights on the device plus the C structs that point at them.

    `weight_fn(name, layer)` returns one canonical [in, out] matrix (or a norm
    gain, or `embed` [V, d]) on the device; matrices are packed one at a time
    so the canonical copy of a large model never exists as a whole.
    """

    def __init__(self, desc: fly_model_desc, weight_fn, device="cuda", layers: Optional[Sequence[int]] = None,
                 with_head: bool = True):
        self.desc = desc
        self.device = device
        dt = desc.dtype
        tdt = torch_dtype(dt)
        es = 2 if dt == FLY_BF16 else 4
        self._keep: List[torch.Tensor] = []
        d, F, V = desc.d, desc.ffn, desc.vocab
        hd, Hq, Hkv = desc.head_dim, desc.n_q_heads, desc.n_kv_heads
        qdim, kvdim = Hq * hd, Hkv * hd

        def alloc(k_in, n_dst):
            t = torch.empty(fly_packed_weight_bytes(k_in, n_dst, dt) // es, dtype=tdt, device=device)
            self._keep.append(t)
            return t

        self.layers_c = (fly_layer_weights * max(desc.n_layers, 1))()
        which = range(desc.n_layers) if layers is None else layers
        for l in which:
            qkv = alloc(d, qdim + 2 * kvdim)
            fly_pack_weight(weight_fn("wq", l), qkv, qdim + 2 * kvdim, 0, 1)
            fly_pack_weight(weight_fn("wk", l), qkv, qdim + 2 * kvdim, qdim // 16, 1)
            fly_pack_weight(weight_fn("wv", l), qkv, qdim + 2 * kvdim, (qdim + kvdim) // 16, 1)
            wo = alloc(qdim, d)
            fly_pack_weight(weight_fn("wo", l), wo, d)
            gu = alloc(d, 2 * F)
            fly_pack_weight(weight_fn("wg", l), gu, 2 * F, 0, 2)
            fly_pack_weight(weight_fn("wu", l), gu, 2 * F, 1, 2)
            wd = alloc(F, d)
            fly_pack_weight(weight_fn("wd", l), wd, d)
            ga = weight_fn("g_attn", l).contiguous()
            gf = weight_fn("g_ffn", l).contiguous()
            self._keep += [ga, gf]
            self.layers_c[l] = fly_layer_weights(qkv.data_ptr(), wo.data_ptr(), gu.data_ptr(),
                                                 wd.data_ptr(), ga.data_ptr(), gf.data_ptr())
        self.g_final = weight_fn("g_final", -1).contiguous()
        self.embed = self.w_lm = None
        if with_head:
            self.embed = weight_fn("embed", -1).contiguous()
            self.w_lm = alloc(d, V)
            fly_pack_weight(weight_fn("w_lm", -1), self.w_lm, V)
        torch.cuda.synchronize()
        self.weights_c = fly_weights(_ptr(self.embed), self.layers_c, _ptr(self.g_final), _ptr(self.w_lm))


class KVCache:
    """KV cache in the library's layout: K [B,Hkv,cap,hd], V [B,Hkv,hd,cap] per layer."""

    def __init__(self, desc: fly_model_desc, B: int, capacity: int, device="cuda",
                 layers: Optional[Sequence[int]] = None):
        assert capacity % 64 == 0
        self.desc, self.B, self.capacity = desc, B, capacity
        tdt = torch_dtype(desc.dtype)
        n = max(desc.n_layers, 1)
        self.k: List[Optional[torch.Tensor]] = [None] * n
        self.v: List[Optional[torch.Tensor]] = [None] * n
        for l in (range(desc.n_layers) if layers is None else layers):
            self.k[l] = torch.empty(B, desc.n_kv_heads, capacity, desc.head_dim, dtype=tdt, device=device)
            self.v[l] = torch.empty(B, desc.n_kv_heads, desc.head_dim, capacity, dtype=tdt, device=device)
        self.kv_len = torch.zeros(B, dtype=torch.int32, device=device)
        self.max_kv_len = 0
        self._k_arr = (C.c_void_p * n)(*[_ptr(t) for t in self.k])
        self._v_arr = (C.c_void_p * n)(*[_ptr(t) for t in self.v])

    def load_prefix(self, layer: int, k: torch.Tensor, v: torch.Tensor) -> None:
        """Copy a canonical prefix k, v [B, L, Hkv, hd] into rows 0..L-1 of a layer."""
        L = k.shape[1]
        self.k[layer][:, :, :L, :].copy_(k.permute(0, 2, 1, 3))
        self.v[layer][:, :, :, :L].copy_(v.permute(0, 2, 3, 1))

    def set_lengths(self, lengths) -> None:
        t = torch.as_tensor(lengths, dtype=torch.int32)
        self.kv_len.copy_(t)
        self.max_kv_len = int(t.max())

    def struct(self) -> fly_kv_cache:
        return fly_kv_cache(self._k_arr, self._v_arr, self.kv_len.data_ptr(), self.capacity,
                            self.max_kv_len)


class VerifyOutputs:
    def __init__(self, B: int, K: int, d: int = 0, device="cuda", want_hidden: bool = False):
        i32 = lambda *s: torch.zeros(*s, dtype=torch.int32, device=device)
        f32 = lambda *s: torch.zeros(*s, dtype=torch.float32, device=device)
        self.accept_len, self.next_token, self.kv_len_out, self.n_loose = i32(B), i32(B), i32(B), i32(B)
        self.argmax = i32(B, K + 1)
        self.h_norm, self.p_top1, self.lse = f32(B, K + 1), f32(B, K + 1), f32(B, K + 1)
        self.hidden = f32(B * (K + 1), d) if want_hidden else None

    def struct(self) -> fly_verify_out:
        return fly_verify_out(*[_ptr(t) for t in (self.accept_len, self.next_token, self.kv_len_out,
                                                  self.argmax, self.h_norm, self.p_top1, self.lse,
                                                  self.n_loose, self.hidden)])


def fly_verify_block(model: PackedModel, kv: KVCache, tokens: torch.Tensor,
                     row_scale: Optional[torch.Tensor], theta: float, W: int, out: VerifyOutputs,
                     workspace: torch.Tensor) -> None:
    B, R = tokens.shape
    kvs, outs = kv.struct(), out.struct()
    _check(lib.fly_verify_block(C.byref(model.desc), C.byref(model.weights_c), C.byref(kvs),
                                _ptr(tokens), _ptr(row_scale), B, R - 1, theta, W, C.byref(outs),
                                _ptr(workspace), workspace.numel() * workspace.element_size(),
                                _stream()), "fly_verify_block")


def fly_verify_block_sampled(model: PackedModel, kv: KVCache, tokens: torch.Tensor,
                             row_scale: Optional[torch.Tensor], theta: float, W: int, seed: int,
                             offset: int, sampled: torch.Tensor, out: VerifyOutputs,
                             workspace: torch.Tensor) -> None:
    B, R = tokens.shape
    kvs, outs = kv.struct(), out.struct()
    _check(lib.fly_verify_block_sampled(C.byref(model.desc), C.byref(model.weights_c), C.byref(kvs),
                                        _ptr(tokens), _ptr(row_scale), B, R - 1, theta, W, seed, offset,
                                        _ptr(sampled), C.byref(outs), _ptr(workspace),
                                        workspace.numel() * workspace.element_size(), _stream()),
           "fly_verify_block_sampled")


class Sequences:
    """Device buffers of a multi-round decode: token rows, their lengths and the statistics."""

    def __init__(self, kv: KVCache, ctx_capacity: int, rounds: int, device="cuda"):
        B = kv.B
        self.kv, self.B, self.ctx_capacity, self.rounds = kv, B, ctx_capacity, rounds
        self.ctx = torch.zeros(B, ctx_capacity, dtype=torch.int32, device=device)
        self.ctx_len = torch.zeros(B, dtype=torch.int32, device=device)
        self.max_ctx_len = 0
        self.accepted_total = torch.zeros(B, dtype=torch.int64, device=device)
        self.rounds_done = torch.zeros(B, dtype=torch.int32, device=device)
        self.loose_total = torch.zeros(B, dtype=torch.int64, device=device)
        self.accept_trace = torch.zeros(max(rounds, 1), B, dtype=torch.int32, device=device)
        self.ngram_trace = torch.zeros(max(rounds, 1), B, dtype=torch.int32, device=device)

    def set_sequences(self, rows) -> None:
        """rows: one token list per sequence; also sets the cache lengths to len - 1."""
        lens = [len(r) for r in rows]
        for b, r in enumerate(rows):
            self.ctx[b, :len(r)] = torch.as_tensor(r, dtype=torch.int32)
        self.ctx_len.copy_(torch.as_tensor(lens, dtype=torch.int32))
        self.max_ctx_len = max(lens)
        self.kv.set_lengths([n - 1 for n in lens])

    def struct(self) -> fly_sequences:
        return fly_sequences(self.ctx.data_ptr(), self.ctx_len.data_ptr(), self.kv.kv_len.data_ptr(),
                             self.ctx_capacity, self.max_ctx_len, self.accepted_total.data_ptr(),
                             self.rounds_done.data_ptr(), self.loose_total.data_ptr(),
                             self.accept_trace.data_ptr(), self.ngram_trace.data_ptr())


def fly_pld_draft(ctx: torch.Tensor, ctx_len: torch.Tensor, K: int, ngram_max: int, tokens: torch.Tensor,
                  ngram: Optional[torch.Tensor]) -> None:
    B, cap = ctx.shape
    _check(lib.fly_pld_draft(_ptr(ctx), _ptr(ctx_len), cap, B, K, ngram_max, _ptr(tokens), _ptr(ngram),
                             _stream()), "fly_pld_draft")


def fly_decode_workspace_bytes(desc: fly_model_desc, B: int, K: int, max_kv_len_end: int) -> int:
    out = C.c_size_t(0)
    _check(lib.fly_decode_workspace_bytes(C.byref(desc), B, K, max_kv_len_end, C.byref(out)),
           "fly_decode_workspace_bytes")
    return out.value


def fly_decode_rounds(model: PackedModel, kv: KVCache, seq: Sequences, row_scale: Optional[torch.Tensor],
                      K: int, theta: float, W: int, ngram_max: int, rounds: int,
                      workspace: torch.Tensor) -> None:
    """Runs `rounds` rounds; afterwards the host-side bounds of `kv` and `seq` are moved along."""
    kvs, ss = kv.struct(), seq.struct()
    _check(lib.fly_decode_rounds(C.byref(model.desc), C.byref(model.weights_c), C.byref(kvs), C.byref(ss),
                                 _ptr(row_scale), kv.B, K, theta, W, ngram_max, rounds, _ptr(workspace),
                                 workspace.numel() * workspace.element_size(), _stream()),
           "fly_decode_rounds")
    kv.max_kv_len += rounds * (K + 1)
    seq.max_ctx_len += rounds * (K + 1)


def fly_decode_rounds_sampled(model: PackedModel, kv: KVCache, seq: Sequences, row_scale: Optional[torch.Tensor],
                              K: int, theta: float, W: int, ngram_max: int, rounds: int, seed: int, offset: int,
                              workspace: torch.Tensor) -> None:
    """The loop with drawn target tokens (round r draws with offset + r); moves the host-side bounds along."""
    kvs, ss = kv.struct(), seq.struct()
    _check(lib.fly_decode_rounds_sampled(C.byref(model.desc), C.byref(model.weights_c), C.byref(kvs), C.byref(ss),
                                         _ptr(row_scale), kv.B, K, theta, W, ngram_max, rounds, seed, offset,
                                         _ptr(workspace), workspace.numel() * workspace.element_size(),
                                         _stream()), "fly_decode_rounds_sampled")
    kv.max_kv_len += rounds * (K + 1)
    seq.max_ctx_len += rounds * (K + 1)


def fly_model_draft_workspace_bytes(desc: fly_model_desc, B: int, K: int, max_ctx_len: int) -> int:
    out = C.c_size_t(0)
    _check(lib.fly_model_draft_workspace_bytes(C.byref(desc), B, K, max_ctx_len, C.byref(out)),
           "fly_model_draft_workspace_bytes")
    return out.value


def fly_model_draft(draft_model: PackedModel, draft_kv: KVCache, ctx: torch.Tensor, ctx_len: torch.Tensor,
                    max_ctx_len: int, K: int, tokens: torch.Tensor, workspace: torch.Tensor) -> None:
    """K greedy tokens of the draft model after every sequence; tokens [B, K+1] int32."""
    B, cap = ctx.shape
    kvs = draft_kv.struct()
    _check(lib.fly_model_draft(C.byref(draft_model.desc), C.byref(draft_model.weights_c), C.byref(kvs),
                               _ptr(ctx), _ptr(ctx_len), cap, max_ctx_len, B, K, _ptr(tokens), _ptr(workspace),
                               workspace.numel() * workspace.element_size(), _stream()), "fly_model_draft")


def fly_decode_model_workspace_bytes(desc: fly_model_desc, draft_desc: fly_model_desc, B: int, K: int,
                                     max_kv_len_end: int) -> int:
    out = C.c_size_t(0)
    _check(lib.fly_decode_model_workspace_bytes(C.byref(desc), C.byref(draft_desc), B, K, max_kv_len_end,
                                                C.byref(out)), "fly_decode_model_workspace_bytes")
    return out.value


def fly_decode_rounds_model(model: PackedModel, kv: KVCache, draft_model: PackedModel, draft_kv: KVCache,
                            seq: Sequences, row_scale: Optional[torch.Tensor], K: int, theta: float, W: int,
                            rounds: int, workspace: torch.Tensor) -> None:
    """`rounds` rounds with the draft model as drafter; moves the host-side bounds along."""
    kvs, dkvs, ss = kv.struct(), draft_kv.struct(), seq.struct()
    _check(lib.fly_decode_rounds_model(C.byref(model.desc), C.byref(model.weights_c), C.byref(kvs),
                                       C.byref(draft_model.desc), C.byref(draft_model.weights_c), C.byref(dkvs),
                                       C.byref(ss), _ptr(row_scale), kv.B, K, theta, W, rounds, _ptr(workspace),
                                       workspace.numel() * workspace.element_size(), _stream()),
           "fly_decode_rounds_model")
    kv.max_kv_len += rounds * (K + 1)
    seq.max_ctx_len += rounds * (K + 1)


def fly_decoder_layers(model: PackedModel, kv: KVCache, x: torch.Tensor, layer_begin: int,
                       layer_end: int, B: int, K: int, workspace: torch.Tensor) -> None:
    kvs = kv.struct()
    _check(lib.fly_decoder_layers(C.byref(model.desc), C.byref(model.weights_c), C.byref(kvs), _ptr(x),
                                  layer_begin, layer_end, B, K, _ptr(workspace),
                                  workspace.numel() * workspace.element_size(), _stream()),
           "fly_decoder_layers")


def fly_attention(desc: fly_model_desc, kv: KVCache, layer: int, q: torch.Tensor, o: torch.Tensor,
                  B: int, K: int, workspace: torch.Tensor) -> None:
    kvs = kv.struct()
    _check(lib.fly_attention(C.byref(desc), C.byref(kvs), layer, _ptr(q), _ptr(o), B, K,
                             _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()),
           "fly_attention")


def fly_gateup_swiglu(xn: torch.Tensor, w_gateup_packed: torch.Tensor, a: torch.Tensor) -> None:
    M, d = xn.shape
    F = a.shape[1]
    _check(lib.fly_gateup_swiglu(_ptr(xn), _ptr(w_gateup_packed), _ptr(a), M, d, F,
                                 dtype_code(xn.dtype), _stream()), "fly_gateup_swiglu")


def fly_proj_partial(xn: torch.Tensor, w_packed: torch.Tensor, partial: torch.Tensor, N: int) -> int:
    """Returns the number of split-K partials written to `partial` (float32, flat)."""
    M, Kd = xn.shape
    splits = C.c_int32(0)
    _check(lib.fly_proj_partial(_ptr(xn), _ptr(w_packed), _ptr(partial), M, N, Kd, dtype_code(xn.dtype),
                                C.byref(splits), partial.numel() * 4, _stream()), "fly_proj_partial")
    return splits.value


def alloc_workspace(nbytes: int, device="cuda") -> torch.Tensor:
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)
