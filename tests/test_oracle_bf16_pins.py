"""Pins for the oracle's bf16 mode (`Numerics("bf16")`), the mode every bf16
parity test compares the device with.

The paper leaves the target model's arithmetic open (Sec. 2.1: one forward
pass of M_T); the rounding contract is this build's: the tensors the device
holds in bf16 are rounded to bf16 (round to nearest even), nothing else is.
Attention probabilities are rounded as 2^(s' - n) with an INTEGER n, because a
power-of-two rescaling commutes with the rounding and the result then does
not depend on how the cache is chunked.  What holds that contract in place
here, without the device:

  * a two-key example worked by hand (literal numbers);
  * shifting every score of a row by an integer number of octaves changes
    nothing, shifting by half an octave does (so n really is an integer);
  * when every unnormalised probability is a power of two, the bf16 result is
    the exact one (so it is these terms that are rounded, not the normalised
    ones, and nothing else inside attention);
  * the error against the unrounded softmax (torch's) obeys the bound of one
    rounding per term, 2^-8 sum|p v|, and has the size that 8 significant bits
    give (not 11, not 24);
  * every declared rounding point is applied to the declared tensor, and each
    one, switched off alone, changes the layer's output.
"""
import math

import numpy as np
import torch

from oracle import fly_oracle as O

F64 = torch.float64
LN2 = math.log(2.0)


def test_two_key_example_by_hand():
    # One query (hd = 1, q = 1), two visible keys k = b ln 2, so the base-2 exponents are
    # b = (0.3, -1.7).  n = ceil(0.3) = 1:
    #   e = (2^-0.7, 2^-2.7) = (0.61557220667..., 0.15389305166...)
    # bf16 keeps 8 significant bits: in [1/2, 1) the spacing is 2^-8, 0.6155722 / 2^-8 = 157.586
    # -> 158 -> 0.6171875; the second term is the first over 4 -> 0.154296875.
    # values v = (1, -3):  numerator 0.6171875 - 3 * 0.154296875 = 0.154296875;
    # the normalising sum keeps the unrounded terms: 0.76946525834...
    b = torch.tensor([0.3, -1.7], dtype=F64)
    q = torch.ones(1, 1, 1, dtype=F64)
    k = (b * LN2).view(2, 1, 1)
    v = torch.tensor([1.0, -3.0], dtype=F64).view(2, 1, 1)
    out = O.attention_one_sequence(q, k, v, 1, O.Numerics("bf16"))[0, 0, 0].item()
    expected = 0.154296875 / (2.0 ** -0.7 + 2.0 ** -2.7)
    assert abs(expected - 0.20052481035) < 1e-10          # the literal, for the reader
    assert abs(out - expected) < 1e-13
    # what the plausible other readings would give, all farther than 3e-4 away:
    #   no rounding                      (e1 - 3 e2) / (e1 + e2)            = 0.2
    #   rounding relative to max (n=0.3) (1 - 0.75) / 1.25                  = 0.2
    #   rounding the normalised p        bf16(0.8) - 3 bf16(0.2)            = 0.2001953125
    #   rounded terms in the sum too     0.154296875 / 0.771484375          = 0.2
    for other in (0.2, 0.2001953125):
        assert abs(out - other) > 3e-4
    # the same example in the unrounded mode is the plain softmax
    exact = O.attention_one_sequence(q, k, v, 1, O.Numerics("f32"))[0, 0, 0].item()
    assert abs(exact - 0.2) < 1e-13


def _random_case(seed, R=5, Hq=4, Hkv=2, hd=32, L=37):
    g = torch.Generator().manual_seed(seed)
    q = torch.randn(R, Hq, hd, generator=g, dtype=F64) * 1.5
    k = torch.randn(L + R, Hkv, hd, generator=g, dtype=F64)
    v = torch.randn(L + R, Hkv, hd, generator=g, dtype=F64)
    return q, k, v, L


def _shift_scores(q, k, octaves):
    """A copy of (q, k) with one more head dimension that adds `octaves` * ln 2 to every
    score of every row (so every base-2 exponent moves by `octaves`); the other
    dimensions are rescaled so that the old part of each score is unchanged.  (The values
    get a zero column to keep the head dimension common; see _pad.)"""
    R, Hq, hd = q.shape
    grow = math.sqrt((hd + 1) / hd)
    q2 = torch.cat([q * grow, torch.full((R, Hq, 1), octaves * LN2 * math.sqrt(hd + 1), dtype=F64)], dim=-1)
    k2 = torch.cat([k, torch.ones(k.shape[0], k.shape[1], 1, dtype=F64)], dim=-1)
    return q2, k2


def _pad(v):
    return torch.cat([v, torch.zeros(v.shape[0], v.shape[1], 1, dtype=F64)], dim=-1)


def test_integer_octave_shift_changes_nothing_half_octave_does():
    num = O.Numerics("bf16")
    q, k, v, L = _random_case(0)
    v = _pad(v)
    q0, k0 = _shift_scores(q, k, 0.0)
    base = O.attention_one_sequence(q0, k0, v, L, num)
    for octaves in (1.0, 7.0, -3.0):
        qs, ks = _shift_scores(q, k, octaves)
        out = O.attention_one_sequence(qs, ks, v, L, num)
        # the exponents move by 1e-15 in fp64, so a term can cross a rounding boundary only with
        # probability ~1e-13: equal up to fp64 noise
        assert torch.allclose(out, base, rtol=0, atol=1e-12), octaves
    qs, ks = _shift_scores(q, k, 0.5)
    half = O.attention_one_sequence(qs, ks, v, L, num)
    diff = (half - base).abs().max().item()
    assert 1e-5 < diff < 2e-2          # the terms are rounded at other places: bf16-sized change
    # in the unrounded mode no shift matters at all
    exact = O.Numerics("f32")
    a = O.attention_one_sequence(q0, k0, v, L, exact)
    c = O.attention_one_sequence(qs, ks, v, L, exact)
    assert torch.allclose(a, c, rtol=0, atol=1e-12)


def test_power_of_two_probabilities_are_exact():
    # keys along one direction with integer base-2 exponents: every unnormalised probability is a
    # power of two, which bf16 holds exactly, so rounding them changes nothing -- whereas rounding
    # the normalised probabilities, the scores or the output would
    hd, T = 16, 12
    g = torch.Generator().manual_seed(3)
    expo = torch.tensor([0, -1, -3, 2, 5, -2, 1, 4, -6, 3, 0, 2], dtype=F64)
    q = torch.zeros(2, 1, hd, dtype=F64)
    q[:, 0, 0] = math.sqrt(hd) * LN2                      # score = k[0] * ln 2  -> exponent k[0]
    k = torch.zeros(T, 1, hd, dtype=F64)
    k[:, 0, 0] = expo
    v = torch.randn(T, 1, hd, generator=g, dtype=F64)
    a = O.attention_one_sequence(q, k, v, T - 2, O.Numerics("bf16"))
    b = O.attention_one_sequence(q, k, v, T - 2, O.Numerics("f32"))
    assert torch.allclose(a, b, rtol=0, atol=1e-14)
    # and the values are NOT rounded inside attention (they are random fp64 numbers here)
    assert not torch.equal(O.round_to_bf16(v), v)


def test_error_against_plain_softmax_has_the_size_of_one_bf16_rounding_per_term():
    q, k, v, L = _random_case(1, R=6, Hq=4, Hkv=2, hd=32, L=200)
    R, Hq, hd = q.shape
    G = Hq // k.shape[1]
    got = O.attention_one_sequence(q, k, v, L, O.Numerics("bf16"))
    ratios = []
    for a in range(Hq):
        kh, vh = k[:, a // G, :], v[:, a // G, :]
        for i in range(R):
            T = L + i + 1
            p = torch.softmax((kh[:T] @ q[i, a]) / math.sqrt(hd), dim=0)      # library softmax
            exact = p @ vh[:T]
            err = (got[i, a] - exact).abs()
            bound = 2.0 ** -8 * (p[:, None] * vh[:T].abs()).sum(0)              # one rounding per term
            assert torch.all(err <= bound * (1 + 1e-9)), (a, i)
            # independent rounding errors, uniform within half a spacing: the spacing of 8-bit
            # significands is 2^-7 of the binade's lower end, i.e. 2^-7 .. 2^-8 of the term itself
            typical = 2.0 ** -7 / math.sqrt(12.0) * torch.sqrt((p[:, None] ** 2 * vh[:T] ** 2).sum(0))
            ratios.append((err.pow(2).mean().sqrt() / typical.pow(2).mean().sqrt()).item())
    r = float(np.mean(ratios))
    # 8 significant bits give a ratio between 1/2 and 1 (where in its binade a term lies; 0.74 for
    # log-uniform terms); 9 bits would give half of that, 11 bits (fp16) ~0.09, 7 bits ~1.4
    assert 0.5 < r < 0.95, r


class RecordingNumerics(O.Numerics):
    """bf16 numerics that records every tensor it is asked to round and can leave one call
    unrounded."""

    def __init__(self, skip=None):
        super().__init__("bf16")
        self.calls = []
        self.skip = skip

    def act(self, x):
        idx = len(self.calls)
        self.calls.append(tuple(x.shape))
        return x if idx == self.skip else super().act(x)


def _layer_case():
    g = torch.Generator().manual_seed(7)
    R, d, Hq, Hkv, hd, F, L = 3, 32, 4, 2, 8, 48, 5
    rnd = lambda *s, std=1.0: torch.randn(*s, generator=g, dtype=F64) * std
    w = O.LayerWeights(wq=rnd(d, Hq * hd, std=0.3), wk=rnd(d, Hkv * hd, std=0.3), wv=rnd(d, Hkv * hd, std=0.3),
                       wo=rnd(Hq * hd, d, std=0.3), wg=rnd(d, F, std=0.3), wu=rnd(d, F, std=0.3),
                       wd=rnd(F, d, std=0.3), g_attn=torch.rand(d, generator=g, dtype=F64) + 0.5,
                       g_ffn=torch.rand(d, generator=g, dtype=F64) + 0.5)
    x = rnd(R, d)
    kp, vp = O.round_to_bf16(rnd(L, Hkv, hd)), O.round_to_bf16(rnd(L, Hkv, hd))
    dims = dict(R=R, d=d, Hq=Hq, Hkv=Hkv, hd=hd, F=F, L=L)
    return x, w, kp, vp, dims


def _run_layer(num, x, w, kp, vp, dims):
    return O.decoder_layer(x, w, kp, vp, dims["Hq"], dims["Hkv"], dims["hd"], 500000.0, 1e-5, num)


def test_declared_rounding_points_and_each_one_matters():
    x, w, kp, vp, dims = _layer_case()
    R, d, Hq, Hkv, hd, F, L = (dims[k] for k in ("R", "d", "Hq", "Hkv", "hd", "F", "L"))
    num = RecordingNumerics()
    base, k_new, v_new = _run_layer(num, x, w, kp, vp, dims)
    # the declared list, in the order a layer meets it: normalised input, rotated q, rotated k, v,
    # the unnormalised probabilities of every (head, row) over its visible keys, the attention
    # output, the second normalised input, the SwiGLU output
    prob_shapes = [(L + i + 1,) for _ in range(Hq) for i in range(R)]
    declared = [(R, d), (R, Hq, hd), (R, Hkv, hd), (R, Hkv, hd)] + prob_shapes + [(R, Hq, hd), (R, d), (R, F)]
    assert num.calls == declared
    # what is appended to the cache is what the device stores: bf16 values
    assert torch.equal(O.round_to_bf16(k_new), k_new) and torch.equal(O.round_to_bf16(v_new), v_new)
    # the residual stream is never rounded
    assert not torch.equal(O.round_to_bf16(base), base)
    # each rounding point, left out alone, moves the output (a misplaced or missing one shows)
    n_calls = len(declared)
    first_prob = 4
    for skip in [0, 1, 2, 3, first_prob, first_prob + len(prob_shapes) - 1, n_calls - 3, n_calls - 2, n_calls - 1]:
        out, _, _ = _run_layer(RecordingNumerics(skip=skip), x, w, kp, vp, dims)
        assert (out - base).abs().max().item() > 1e-7, skip
    # and against the unrounded layer the difference has bf16 size: eight significant bits on
    # activations of order one give 1e-3 .. 1e-1 at this width, not 1e-6 and not order one
    exact, _, _ = _run_layer(O.Numerics("f32"), x, w, kp, vp, dims)
    diff = (base - exact).abs().max().item()
    assert 1e-4 < diff < 0.2, diff


def test_final_norm_and_tables_round_where_declared():
    # the rotary tables are rounded to fp32, not to bf16: an fp32 table entry is in general not a
    # bf16 value, and the fp64 entry not an fp32 one
    num = O.Numerics("bf16")
    cos, _ = O.rope_tables(torch.tensor([17]), 8, 500000.0)
    t = num.table(cos)
    assert torch.equal(t, cos.to(torch.float32).to(F64)) and not torch.equal(t, cos)
    assert not torch.equal(O.round_to_bf16(t), t)
    assert torch.equal(O.Numerics("f32").table(cos), cos)
