"""GPU-side test glue: loads a synthetic workload into the library's buffers,
runs the HIP path through the C ABI and returns numpy results."""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np
import torch

import synth


def binding():
    from paper_2511_22972_amd import binding as fb
    return fb


class GpuWorkload:
    """Packed weights + KV cache + workspace of one synthetic configuration."""

    def __init__(self, cfg: synth.VerifyConfig, kv_lens=None, capacity: Optional[int] = None,
                 weight_fn=None):
        fb = binding()
        self.fb, self.cfg = fb, cfg
        self.desc = fb.make_desc(cfg)
        wf = weight_fn or (lambda name, layer: synth.make_weight(cfg, name, layer, "cuda"))
        self.model = fb.PackedModel(self.desc, wf)
        self.kv_lens = [cfg.kv_len] * cfg.batch if kv_lens is None else list(kv_lens)
        need = max(self.kv_lens) + cfg.K + 1
        cap = capacity or (need + 63) // 64 * 64
        self.kv = fb.KVCache(self.desc, cfg.batch, cap)
        for l in range(cfg.n_layers):
            k, v = synth.make_kv_prefix(cfg, l, "cuda")
            self.kv.load_prefix(l, k, v)
        self.kv.set_lengths(self.kv_lens)
        self.ws = fb.alloc_workspace(fb.fly_workspace_bytes(self.desc, cfg.batch, cfg.K, max(self.kv_lens)))

    def verify(self, tokens: np.ndarray, row_scale: Optional[torch.Tensor], theta=None, W=None,
               want_hidden=True) -> Dict[str, np.ndarray]:
        fb, cfg = self.fb, self.cfg
        tok = torch.as_tensor(np.ascontiguousarray(tokens), dtype=torch.int32).cuda()
        rs = None if row_scale is None else row_scale.to("cuda", torch.float32).contiguous()
        out = fb.VerifyOutputs(cfg.batch, cfg.K, cfg.d, want_hidden=want_hidden)
        fb.fly_verify_block(self.model, self.kv, tok, rs, cfg.theta if theta is None else theta,
                            cfg.window if W is None else W, out, self.ws)
        torch.cuda.synchronize()
        res = {k: getattr(out, k).cpu().numpy() for k in
               ("accept_len", "next_token", "kv_len_out", "n_loose", "argmax", "h_norm", "p_top1", "lse")}
        if want_hidden:
            res["hidden"] = out.hidden.cpu().numpy()
        return res


def verify_sampled(wl: GpuWorkload, tokens: np.ndarray, row_scale: Optional[torch.Tensor], seed: int,
                   offset: int, theta=None, W=None) -> Dict[str, np.ndarray]:
    """fly_verify_block_sampled on a loaded workload."""
    fb, cfg = wl.fb, wl.cfg
    tok = torch.as_tensor(np.ascontiguousarray(tokens), dtype=torch.int32).cuda()
    rs = None if row_scale is None else row_scale.to("cuda", torch.float32).contiguous()
    out = fb.VerifyOutputs(cfg.batch, cfg.K, cfg.d, want_hidden=True)
    sampled = torch.zeros(cfg.batch, cfg.K + 1, dtype=torch.int32, device="cuda")
    fb.fly_verify_block_sampled(wl.model, wl.kv, tok, rs, cfg.theta if theta is None else theta,
                                cfg.window if W is None else W, seed, offset, sampled, out, wl.ws)
    torch.cuda.synchronize()
    res = {k: getattr(out, k).cpu().numpy() for k in
           ("accept_len", "next_token", "kv_len_out", "n_loose", "argmax", "h_norm", "p_top1", "lse")}
    res["sampled"] = sampled.cpu().numpy()
    res["hidden"] = out.hidden.cpu().numpy()
    return res


def ambiguous_rows(oracle_out: Dict[str, np.ndarray], theta: float, tol: float = 1e-3) -> np.ndarray:
    """[B, K+1] mask of positions whose integer outcome may legitimately differ:
    top-2 logit margin or entropy-minus-threshold below `tol`."""
    return (oracle_out["margin"] < tol) | (np.abs(oracle_out["h"] - theta) < tol)


def check_own_rule(gpu: Dict[str, np.ndarray], tokens: np.ndarray, theta: float, W: int, oracle_accept,
                   target_key: str = "argmax") -> None:
    """The device's accept outputs equal the oracle's rule applied to the device's own target tokens
    and entropies -- for every sequence, near ties or not."""
    own = oracle_accept(np.asarray(tokens)[:, 1:], gpu[target_key], gpu["h_norm"], theta, W)
    for k in ("accept_len", "next_token", "n_loose"):
        assert np.array_equal(gpu[k], own[k]), ("own statistics", k, gpu[k], own[k])


def compare_verify(gpu: Dict[str, np.ndarray], ora: Dict[str, np.ndarray], theta: float,
                   float_tol: float, oracle_accept, tokens: np.ndarray, W: int, min_clean: int = 1,
                   int_tol: float = 1e-3) -> Dict[str, float]:
    """Element-by-element comparison of a verification step with the oracle's.

    Floats (lse, h, p_top1) within float_tol.  Integers (argmax, then accept_len, next_token,
    n_loose of the sequences whose K+1 positions are all unambiguous) bit-exact except at positions
    whose top-2 margin or |h - theta| is below int_tol; at least min_clean sequences must be
    unambiguous, so the integer assertions are never vacuous.  And in every case the accept outputs
    equal the rule applied to the device's own (argmax, h).

    int_tol is the 1e-3 of the stated bar whenever the two sides evaluate the SAME logits up to
    rounding order (fp32 models; the teacher-forced tail, see compare_tail).  A free-running bf16
    run may pass a larger one: there the logits themselves differ by up to float_tol."""
    check_own_rule(gpu, tokens, theta, W, oracle_accept)
    amb = ambiguous_rows(ora, theta, int_tol)
    err = {
        "lse": float(np.abs(gpu["lse"] - ora["lse"]).max()),
        "h": float(np.abs(gpu["h_norm"] - ora["h"]).max()),
        "p_top1": float(np.abs(gpu["p_top1"] - ora["p_top1"]).max()),
    }
    print("parity errors", err, "tol", float_tol)
    for k, v in err.items():
        assert v <= float_tol, (k, v, float_tol)
    same = gpu["argmax"] == ora["argmax"]
    assert np.all(same | amb), ("argmax differs at a position that is not a near tie",
                                np.argwhere(~same & ~amb))
    clean = ~amb.any(axis=1)
    assert clean.sum() >= min_clean, ("too few unambiguous sequences", int(clean.sum()), min_clean)
    for k in ("accept_len", "next_token", "n_loose"):
        assert np.array_equal(gpu[k][clean], ora[k][clean]), (k, gpu[k], ora[k])
    err["n_ambiguous"] = float(amb.sum())
    err["n_clean_sequences"] = float(clean.sum())
    return err


def compare_tail(gpu: Dict[str, np.ndarray], tail: Dict[str, np.ndarray], theta: float, oracle_accept,
                 tokens: np.ndarray, W: int, min_clean: int = 1, float_tol: float = 2e-3) -> Dict[str, float]:
    """Teacher-forced comparison of the end of the step: `tail` is the oracle's final norm, LM head,
    row statistics and acceptance rule applied to the DEVICE's residual stream after the last layer
    (helpers.oracle_tail), so both sides evaluate the same logits up to rounding order and the
    integer outputs must agree outside the 1e-3 exclusions, whatever the depth of the model."""
    return compare_verify(gpu, tail, theta, float_tol, oracle_accept, tokens, W, min_clean, 1e-3)
