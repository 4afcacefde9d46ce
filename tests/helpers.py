"""Test-side glue: turns a synthetic workload into oracle inputs and builds the
draft chain with the oracle.  Nothing here touches the HIP path."""
from __future__ import annotations

from typing import Dict, List, Tuple

import numpy as np
import torch

import synth
from oracle import fly_oracle as O


def oracle_layer_weights(cfg: synth.VerifyConfig, layer: int, device="cpu") -> O.LayerWeights:
    g = lambda n: synth.make_weight(cfg, n, layer, device).to("cpu", torch.float64)
    return O.LayerWeights(wq=g("wq"), wk=g("wk"), wv=g("wv"), wo=g("wo"), wg=g("wg"),
                          wu=g("wu"), wd=g("wd"), g_attn=g("g_attn"), g_ffn=g("g_ffn"))


def oracle_model(cfg: synth.VerifyConfig, device="cpu") -> Dict:
    """All oracle-side tensors of a workload (fp64 copies of the seeded inputs)."""
    f64 = lambda t: t.to("cpu", torch.float64)
    return {
        "embed": f64(synth.make_weight(cfg, "embed", -1, device)),
        "layers": [oracle_layer_weights(cfg, l, device) for l in range(cfg.n_layers)],
        "g_final": f64(synth.make_weight(cfg, "g_final", -1, device)),
        "w_lm": f64(synth.make_weight(cfg, "w_lm", -1, device)),
        "kv_prefix": [tuple(f64(t) for t in synth.make_kv_prefix(cfg, l, device))
                      for l in range(cfg.n_layers)],
    }


def row_scale(cfg: synth.VerifyConfig) -> torch.Tensor:
    """float32 [B*(K+1)] multiplier on the logits: logit_gain / temperature."""
    t = synth.make_row_temperature(cfg)
    return (torch.tensor(cfg.logit_gain, dtype=torch.float32) / t).reshape(-1)


def oracle_verify(cfg: synth.VerifyConfig, model: Dict, tokens: np.ndarray, theta=None,
                  W=None, return_logits=False, sample=None) -> Dict:
    return O.verify_block(
        tokens, model["embed"], model["layers"], model["g_final"], model["w_lm"],
        model["kv_prefix"], row_scale(cfg), n_q_heads=cfg.n_q_heads,
        n_kv_heads=cfg.n_kv_heads, head_dim=cfg.head_dim, rope_theta=cfg.rope_theta,
        eps=cfg.rms_eps, theta=cfg.theta if theta is None else theta,
        W=cfg.window if W is None else W, storage=cfg.dtype, return_logits=return_logits,
        sample=sample)


def draft_chain(cfg: synth.VerifyConfig, model: Dict) -> np.ndarray:
    """tokens [B, K+1]: y_{-1} then K drafts, draft i equal to the oracle
    target's argmax at position i with probability p_match, else a uniform
    token.  Causality makes position i's argmax independent of later tokens,
    so the chain is built by K+1 oracle passes over a growing block."""
    first = synth.make_first_tokens(cfg).numpy()
    u, alt, _ = synth.make_draft_draws(cfg)
    u, alt = u.numpy(), alt.numpy()
    B, K = cfg.batch, cfg.K
    tokens = np.zeros((B, K + 1), dtype=np.int32)
    tokens[:, 0] = first
    for i in range(1, K + 1):
        sub = cfg.replace(K=i - 1)
        out = O.verify_block(
            tokens[:, :i], model["embed"], model["layers"], model["g_final"], model["w_lm"],
            model["kv_prefix"], row_scale(cfg).reshape(B, K + 1)[:, :i].reshape(-1),
            n_q_heads=cfg.n_q_heads, n_kv_heads=cfg.n_kv_heads, head_dim=cfg.head_dim,
            rope_theta=cfg.rope_theta, eps=cfg.rms_eps, theta=cfg.theta, W=cfg.window,
            storage=cfg.dtype)
        y_i = out["argmax"][:, i - 1]
        tokens[:, i] = np.where(u[:, i - 1] < cfg.p_match, y_i, alt[:, i - 1])
    return tokens


def oracle_tail(cfg: synth.VerifyConfig, hidden: np.ndarray, tokens: np.ndarray, g_final: torch.Tensor,
                w_lm: torch.Tensor, theta=None, W=None, sample=None) -> Dict:
    """The end of the step on a GIVEN residual stream (Algorithm 1 steps 2-4 after the last layer):
    final norm, LM head, row statistics (Eq. 1, Eq. 5) and the acceptance rule (Eqs. 2-11).
    hidden [B*(K+1), d] is the residual stream after the last decoder layer -- in a teacher-forced
    comparison the device's own."""
    tokens = np.asarray(tokens)
    B, R = tokens.shape
    num = O.Numerics(cfg.dtype)
    x = torch.from_numpy(np.asarray(hidden, dtype=np.float64)).view(B * R, -1)
    xn = num.act(O.rmsnorm(x, g_final, cfg.rms_eps))
    logits = O.lm_head_logits(xn, w_lm, row_scale(cfg))
    out = {k: v.reshape(B, R) for k, v in O.decision_statistics(logits).items()}
    target = out["argmax"]
    if sample is not None:
        drawn = O.sample_rows(logits.numpy(), sample[0], sample[1])
        out["sampled"] = drawn["token"].reshape(B, R)
        out["sample_margin"] = drawn["margin"].reshape(B, R)
        target = out["sampled"]
    out.update(O.accept_block(tokens[:, 1:], target, out["h"], cfg.theta if theta is None else theta,
                              cfg.window if W is None else W))
    return out
