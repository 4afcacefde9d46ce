"""The C-ABI library without a GPU: it loads, exports what include/fly.h
declares, and every argument check fires before anything is launched."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2511_22972_amd", "libfly.so")


@pytest.fixture(scope="module")
def fb():
    # a missing library is a failure, not a skip: a skipped file pins nothing
    assert os.path.exists(LIB), "libfly.so is not built: run `python __graft_entry__.py` first"
    from paper_2511_22972_amd import binding
    return binding


def declared_functions():
    text = open(os.path.join(ROOT, "include", "fly.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fly_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(fb):
    names = declared_functions()
    assert "fly_verify_block" in names and "fly_lmhead_entropy_argmax" in names and "fly_accept" in names
    for n in names:
        assert hasattr(fb.lib, n), n
    assert sorted(fb.EXPORTS) == names


def test_strerror(fb):
    assert fb.strerror(0) == "ok"
    seen = {fb.strerror(-i) for i in range(1, 13)}
    assert len(seen) == 12 and "unknown status" not in seen
    assert fb.strerror(-99) == "unknown status"


def _desc(fb, **kw):
    base = dict(n_layers=2, d=256, n_q_heads=4, n_kv_heads=2, head_dim=64, ffn=688, vocab=8192,
                dtype=fb.FLY_F32, rms_eps=1e-5, rope_theta=5e5)
    base.update(kw)
    return fb.fly_model_desc(*[base[k] for k, _ in fb.fly_model_desc._fields_])


def test_workspace_query_and_shape_errors(fb):
    out = C.c_size_t(0)
    d = _desc(fb)
    assert fb.lib.fly_workspace_bytes(C.byref(d), 1, 4, 128, C.byref(out)) == 0 and out.value > 0
    small = out.value
    d16 = _desc(fb, dtype=fb.FLY_BF16, head_dim=128, d=4096, n_q_heads=32, n_kv_heads=8, ffn=14336,
                vocab=128256, n_layers=32)
    assert fb.lib.fly_workspace_bytes(C.byref(d16), 1, 8, 2048, C.byref(out)) == 0 and out.value > small
    assert fb.lib.fly_workspace_bytes(None, 1, 4, 128, C.byref(out)) == -1
    assert fb.lib.fly_workspace_bytes(C.byref(d), 1, 4, 128, None) == -1
    assert fb.lib.fly_workspace_bytes(C.byref(d), 0, 4, 128, C.byref(out)) == -2
    assert fb.lib.fly_workspace_bytes(C.byref(d), 1, 0, 128, C.byref(out)) == -3
    assert fb.lib.fly_workspace_bytes(C.byref(d), 1, 64, 128, C.byref(out)) == -3
    assert fb.lib.fly_workspace_bytes(C.byref(_desc(fb, dtype=7)), 1, 4, 128, C.byref(out)) == -6
    assert fb.lib.fly_workspace_bytes(C.byref(_desc(fb, head_dim=96)), 1, 4, 128, C.byref(out)) == -7
    assert fb.lib.fly_workspace_bytes(C.byref(_desc(fb, dtype=fb.FLY_BF16, head_dim=64)), 1, 4, 128,
                                      C.byref(out)) == -7
    assert fb.lib.fly_workspace_bytes(C.byref(_desc(fb, n_kv_heads=3)), 1, 4, 128, C.byref(out)) == -2
    assert fb.lib.fly_workspace_bytes(C.byref(_desc(fb, vocab=8200)), 1, 4, 128, C.byref(out)) == -2
    # more than 4096 query rows per KV head (17 positions x 256 heads) are refused
    wide = dict(dtype=fb.FLY_BF16, head_dim=128, ffn=704, n_kv_heads=1)
    assert fb.lib.fly_workspace_bytes(C.byref(_desc(fb, n_q_heads=256, **wide)), 1, 16, 128, C.byref(out)) == -2
    assert fb.lib.fly_workspace_bytes(C.byref(_desc(fb, n_q_heads=64, **wide)), 1, 16, 128, C.byref(out)) == 0


def test_accept_argument_checks(fb):
    p = C.c_void_p(4096)   # never dereferenced: every call below fails validation first
    f = fb.lib.fly_accept
    assert f(None, p, p, 1, 4, 0.3, 6, p, p, None, None) == -1
    assert f(p, p, p, 1, 4, 0.3, 6, None, p, None, None) == -1
    assert f(p, p, p, 0, 4, 0.3, 6, p, p, None, None) == -2
    assert f(p, p, p, 65537, 4, 0.3, 6, p, p, None, None) == -2
    assert f(p, p, p, 1, 0, 0.3, 6, p, p, None, None) == -3
    assert f(p, p, p, 1, 64, 0.3, 6, p, p, None, None) == -3
    assert f(p, p, p, 1, 4, 0.3, -1, p, p, None, None) == -4
    assert f(p, p, p, 1, 4, float("nan"), 6, p, p, None, None) == -5


def test_lmhead_argument_checks(fb):
    p, odd = C.c_void_p(4096), C.c_void_p(4100)
    f = fb.lib.fly_lmhead_entropy_argmax
    out = C.c_size_t(0)
    assert fb.lib.fly_lmhead_workspace_bytes(36, 8192, 128256, fb.FLY_BF16, C.byref(out)) == 0
    need = out.value
    assert need >= 36 * (128256 // 64) * 16      # one statistics record per row and 64 columns
    assert f(None, p, None, 36, 8192, 128256, 1, p, p, p, None, p, need, None) == -1
    assert f(p, p, None, 36, 8192, 128256, 1, p, p, p, None, None, need, None) == -9
    assert f(p, p, None, 36, 8192, 128256, 1, p, p, p, None, p, need - 1, None) == -9
    assert f(odd, p, None, 36, 8192, 128256, 1, p, p, p, None, p, need, None) == -8
    assert f(p, p, None, 36, 8192, 128250, 1, p, p, p, None, p, need, None) == -2
    assert f(p, p, None, 36, 8200, 128256, 1, p, p, p, None, p, need, None) == -2
    assert f(p, p, None, 36, 8192, 128256, 5, p, p, p, None, p, need, None) == -6
    assert f(p, p, None, 0, 8192, 128256, 1, p, p, p, None, p, need, None) == -2


def test_static_scratch_lmhead_argument_checks(fb):
    """The entry point without a workspace validates before it touches the device."""
    p, odd = C.c_void_p(4096), C.c_void_p(4100)
    f = fb.lib.fly_lmhead_entropy_argmax_static
    assert f(p, p, None, 1088, 8192, 128256, fb.FLY_BF16, p, p, p, None, None) == -12   # 26 MB > 16 MiB
    assert f(p, p, None, 0, 8192, 128256, fb.FLY_BF16, p, p, p, None, None) == -2
    assert f(p, p, None, 36, 8192, 128250, fb.FLY_BF16, p, p, p, None, None) == -2
    assert f(p, p, None, 36, 8192, 128256, 7, p, p, p, None, None) == -6
    assert f(None, p, None, 36, 8192, 128256, fb.FLY_BF16, p, p, p, None, None) == -1
    assert f(p, p, None, 36, 8192, 128256, fb.FLY_BF16, None, p, p, None, None) == -1
    assert f(odd, p, None, 36, 8192, 128256, fb.FLY_BF16, p, p, p, None, None) == -8
    assert "static scratch" in fb.strerror(-12)


def test_sampled_entry_points_argument_checks(fb):
    """The entry points with a drawn token share the checks of the plain ones and need `sampled`."""
    p = C.c_void_p(4096)
    f = fb.lib.fly_lmhead_entropy_sample
    out = C.c_size_t(0)
    assert fb.lib.fly_lmhead_workspace_bytes(36, 8192, 128256, fb.FLY_BF16, C.byref(out)) == 0
    need = out.value
    assert need >= 36 * (128256 // 64) * 24      # statistics and the pick per row and 64 columns
    assert f(p, p, None, 36, 8192, 128256, 1, 7, 0, None, p, p, p, None, p, need, None) == -1
    assert f(None, p, None, 36, 8192, 128256, 1, 7, 0, p, p, p, p, None, p, need, None) == -1
    assert f(p, p, None, 36, 8192, 128256, 1, 7, 0, p, p, p, p, None, p, need - 1, None) == -9
    assert f(p, p, None, 36, 8192, 128250, 1, 7, 0, p, p, p, p, None, p, need, None) == -2
    q = 4096
    d = _desc(fb)
    lw = (fb.fly_layer_weights * 2)(*[fb.fly_layer_weights(q, q, q, q, q, q)] * 2)
    w = fb.fly_weights(q, lw, q, q)
    karr = (C.c_void_p * 2)(q, q)
    kv = fb.fly_kv_cache(karr, karr, q, 192, 128)
    vout = fb.fly_verify_out(q, q, q, q, q, q, None, None, None)
    ws = C.c_size_t(0)
    fb.lib.fly_workspace_bytes(C.byref(d), 1, 4, 128, C.byref(ws))
    g = fb.lib.fly_verify_block_sampled
    base = [C.byref(d), C.byref(w), C.byref(kv), q, None, 1, 4, 0.3, 6, 1, 2]
    assert g(*base, None, C.byref(vout), q, ws.value, None) == -1
    assert g(*base, q, C.byref(vout), q, ws.value - 1, None) == -9
    base[6] = 70
    assert g(*base, q, C.byref(vout), q, ws.value, None) == -3


def test_verify_block_argument_checks(fb):
    p = 4096
    d = _desc(fb)
    lw = (fb.fly_layer_weights * 2)(*[fb.fly_layer_weights(p, p, p, p, p, p)] * 2)
    w = fb.fly_weights(p, lw, p, p)
    karr = (C.c_void_p * 2)(p, p)
    kv = fb.fly_kv_cache(karr, karr, p, 192, 128)
    out = fb.fly_verify_out(p, p, p, p, p, p, None, None, None)
    f = fb.lib.fly_verify_block
    ws = C.c_size_t(0)
    fb.lib.fly_workspace_bytes(C.byref(d), 1, 4, 128, C.byref(ws))
    args = lambda **kw: [kw.get("desc", C.byref(d)), kw.get("w", C.byref(w)), kw.get("kv", C.byref(kv)),
                         kw.get("tokens", p), None, kw.get("B", 1), kw.get("K", 4),
                         kw.get("theta", 0.3), kw.get("W", 6), kw.get("out", C.byref(out)),
                         kw.get("ws", p), kw.get("wsb", ws.value), None]
    assert f(*args(tokens=None)) == -1
    assert f(*args(K=70)) == -3
    assert f(*args(W=-2)) == -4
    assert f(*args(theta=float("nan"))) == -5
    assert f(*args(ws=None)) == -9
    assert f(*args(wsb=ws.value - 1)) == -9
    assert f(*args(ws=4100)) == -8
    kv_small = fb.fly_kv_cache(karr, karr, p, 128, 128)          # 128 + 5 rows do not fit
    assert f(*args(kv=C.byref(kv_small))) == -10
    kv_odd = fb.fly_kv_cache(karr, karr, p, 200, 128)            # capacity not a multiple of 64
    assert f(*args(kv=C.byref(kv_odd))) == -2
    w_null = fb.fly_weights(p, lw, p, None)
    assert f(*args(w=C.byref(w_null))) == -1
    lw_bad = (fb.fly_layer_weights * 2)(fb.fly_layer_weights(p, p, p, p, p, p),
                                        fb.fly_layer_weights(p, 4100, p, p, p, p))
    assert f(*args(w=C.byref(fb.fly_weights(p, lw_bad, p, p)))) == -8
    out_null = fb.fly_verify_out(p, None, p, p, p, p, None, None, None)
    assert f(*args(out=C.byref(out_null))) == -1


def test_pack_argument_checks(fb):
    p = C.c_void_p(4096)
    out = C.c_size_t(0)
    assert fb.lib.fly_packed_weight_bytes(8192, 10240, fb.FLY_BF16, C.byref(out)) == 0
    assert out.value == 8192 * 10240 * 2
    assert fb.lib.fly_packed_weight_bytes(688, 256, fb.FLY_F32, C.byref(out)) == 0 and out.value == 688 * 256 * 4
    assert fb.lib.fly_packed_weight_bytes(688, 256, fb.FLY_BF16, C.byref(out)) == -2   # 688 % 32 != 0
    f = fb.lib.fly_pack_weight
    assert f(None, 64, 32, 1, p, 32, 0, 1, None) == -1
    assert f(p, 64, 24, 1, p, 32, 0, 1, None) == -2
    assert f(p, 64, 32, 1, p, 32, 1, 1, None) == -2      # last tile would fall outside dst
    assert f(p, 64, 32, 1, p, 64, 2, 2, None) == -2      # tiles 2 and 4 of a 4-tile destination
    assert f(p, 64, 32, 9, p, 32, 0, 1, None) == -6


def test_decode_argument_checks(fb):
    p = C.c_void_p(4096)
    f = fb.lib.fly_pld_draft
    assert f(None, p, 64, 2, 4, 3, p, None, None) == -1
    assert f(p, p, 64, 2, 4, 3, None, None, None) == -1
    assert f(p, p, 64, 0, 4, 3, p, None, None) == -2
    assert f(p, p, 64, 2, 64, 3, p, None, None) == -3
    assert f(p, p, 64, 2, 4, 0, p, None, None) == -2
    assert f(p, p, 64, 2, 4, 65, p, None, None) == -2
    assert f(p, p, 0, 2, 4, 3, p, None, None) == -2
    out = C.c_size_t(0)
    d = _desc(fb)
    assert fb.lib.fly_decode_workspace_bytes(C.byref(d), 2, 4, 256, C.byref(out)) == 0
    ws = C.c_size_t(0)
    fb.lib.fly_workspace_bytes(C.byref(d), 2, 4, 256, C.byref(ws))
    assert out.value > ws.value                                    # verification workspace + round buffers
    assert fb.lib.fly_decode_workspace_bytes(C.byref(d), 2, 4, 256, None) == -1
    lw = (fb.fly_layer_weights * 2)(*[fb.fly_layer_weights(4096, 4096, 4096, 4096, 4096, 4096)] * 2)
    w = fb.fly_weights(4096, lw, 4096, 4096)
    karr = (C.c_void_p * 2)(4096, 4096)
    kv = fb.fly_kv_cache(karr, karr, 4096, 192, 100)
    seq = fb.fly_sequences(4096, 4096, 4096, 256, 101, None, None, None, None, None)
    g = fb.lib.fly_decode_rounds
    args = lambda **kw: [C.byref(d), C.byref(w), kw.get("kv", C.byref(kv)), kw.get("seq", C.byref(seq)), None,
                         2, kw.get("K", 4), kw.get("theta", 0.3), kw.get("W", 6), kw.get("n", 3),
                         kw.get("rounds", 3), kw.get("ws", 4096), kw.get("wsb", out.value), None]
    assert g(*args(seq=None)) == -1
    assert g(*args(K=0)) == -3
    assert g(*args(W=-1)) == -4
    assert g(*args(theta=float("nan"))) == -5
    assert g(*args(n=0)) == -2
    assert g(*args(rounds=-1)) == -2
    assert g(*args(rounds=19)) == -10                               # 100 + 19*5 rows do not fit 192
    seq_small = fb.fly_sequences(4096, 4096, 4096, 110, 101, None, None, None, None, None)
    assert g(*args(seq=C.byref(seq_small))) == -10                  # 101 + 15 tokens do not fit 110
    seq_other = fb.fly_sequences(4096, 4096, 8192, 256, 101, None, None, None, None, None)
    assert g(*args(seq=C.byref(seq_other))) == -2                   # cache lengths must be one array
    assert g(*args(ws=None)) == -9
    assert g(*args(wsb=out.value - 1)) == -9


def test_decode_rounds_sampled_argument_checks(fb):
    q = 4096
    d = _desc(fb)
    lw = (fb.fly_layer_weights * 2)(*[fb.fly_layer_weights(q, q, q, q, q, q)] * 2)
    w = fb.fly_weights(q, lw, q, q)
    karr = (C.c_void_p * 2)(q, q)
    kv = fb.fly_kv_cache(karr, karr, q, 192, 128)
    f = fb.lib.fly_decode_rounds_sampled
    assert f(C.byref(d), C.byref(w), C.byref(kv), None, None, 1, 4, 0.3, 6, 3, 2, 7, 0, q, 1 << 30, None) == -1
    assert f(C.byref(d), C.byref(w), C.byref(kv), None, None, 1, 70, 0.3, 6, 3, 2, 7, 0, q, 1 << 30, None) == -3


def test_model_draft_argument_checks(fb):
    p = C.c_void_p(4096)
    d = _desc(fb)
    out = C.c_size_t(0)
    q = fb.lib.fly_model_draft_workspace_bytes
    assert q(C.byref(d), 2, 4, 64, C.byref(out)) == 0 and out.value > 0
    need = out.value
    assert q(C.byref(d), 2, 4, 64, None) == -1
    assert q(C.byref(d), 2, 0, 64, C.byref(out)) == -3
    assert q(C.byref(d), 2, 4, 1, C.byref(out)) == -2               # a sequence needs two tokens
    lw = (fb.fly_layer_weights * 2)(*[fb.fly_layer_weights(4096, 4096, 4096, 4096, 4096, 4096)] * 2)
    w = fb.fly_weights(4096, lw, 4096, 4096)
    karr = (C.c_void_p * 2)(4096, 4096)
    kv = fb.fly_kv_cache(karr, karr, None, 128, 0)                   # the drafter's cache needs no length array
    f = fb.lib.fly_model_draft
    args = lambda **kw: [C.byref(d), C.byref(w), kw.get("kv", C.byref(kv)), kw.get("ctx", p), p, kw.get("cap", 100),
                         kw.get("maxlen", 64), 2, kw.get("K", 4), kw.get("tok", p), kw.get("ws", 4096),
                         kw.get("wsb", need), None]
    assert f(*args(ctx=None)) == -1
    assert f(*args(tok=None)) == -1
    assert f(*args(K=64)) == -3
    assert f(*args(maxlen=1)) == -2
    assert f(*args(maxlen=101)) == -2                                # bound beyond the token rows
    kv_small = fb.fly_kv_cache(karr, karr, None, 64, 0)
    assert f(*args(kv=C.byref(kv_small))) == -10                     # 64 + 4 rows do not fit 64
    assert f(*args(ws=None)) == -9
    assert f(*args(wsb=need - 1)) == -9
    # the loop with a draft model: one vocabulary, room in both caches
    tq = fb.lib.fly_decode_model_workspace_bytes
    assert tq(C.byref(d), C.byref(d), 2, 4, 128, C.byref(out)) == 0
    both = out.value
    tkv = fb.fly_kv_cache(karr, karr, 4096, 192, 100)
    seq = fb.fly_sequences(4096, 4096, 4096, 256, 101, None, None, None, None, None)
    dkv = fb.fly_kv_cache(karr, karr, None, 192, 0)
    g = fb.lib.fly_decode_rounds_model
    gargs = lambda **kw: [C.byref(d), C.byref(w), C.byref(tkv), kw.get("dd", C.byref(d)), C.byref(w),
                          kw.get("dkv", C.byref(dkv)), kw.get("seq", C.byref(seq)), None, 2, kw.get("K", 4), 0.3,
                          kw.get("W", 6), kw.get("rounds", 3), kw.get("ws", 4096), kw.get("wsb", both), None]
    assert g(*gargs(seq=None)) == -1
    assert g(*gargs(K=0)) == -3
    assert g(*gargs(W=-1)) == -4
    other = _desc(fb, vocab=4096)
    assert g(*gargs(dd=C.byref(other))) == -2                        # two alphabets
    assert g(*gargs(rounds=19)) == -10                               # the target's cache is too short
    dkv_small = fb.fly_kv_cache(karr, karr, None, 64, 0)
    assert g(*gargs(dkv=C.byref(dkv_small))) == -10                  # the drafter's cache is too short
    assert g(*gargs(wsb=both - 1)) == -9
