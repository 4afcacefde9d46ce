"""fly_lmhead_entropy_argmax_static -- the LM head for callers that cannot allocate -- against
fly_lmhead_entropy_argmax through the C ABI: same kernels, so the same bits.  Two calls in a row
share the library's static scratch array, the second with a smaller input (what the first call
left in the array must not matter), then a third at the largest size the array admits."""
import ctypes as C

import numpy as np
import pytest
import torch

import synth

pytestmark = pytest.mark.gpu


def _run(fb, M, d, V, seed, static):
    hidden = synth.hash_normal(seed, 201, (M, d), 4.0, torch.bfloat16, "cuda")
    w = synth.hash_normal(seed, 202, (d, V), 0.02, torch.bfloat16, "cuda")
    wp = torch.empty(d * V, dtype=torch.bfloat16, device="cuda")
    fb.fly_pack_weight(w, wp, V)
    rs = torch.linspace(0.2, 5.0, M).to("cuda", torch.float32)
    argmax = torch.full((M,), -1, dtype=torch.int32, device="cuda")
    p1, hn, lse = (torch.full((M,), float("nan"), dtype=torch.float32, device="cuda") for _ in range(3))
    p = lambda t: C.c_void_p(t.data_ptr())
    if static:
        st = fb.lib.fly_lmhead_entropy_argmax_static(p(hidden), p(wp), p(rs), M, d, V, fb.FLY_BF16, p(argmax),
                                                     p(p1), p(hn), p(lse), None)
    else:
        ws = fb.alloc_workspace(fb.fly_lmhead_workspace_bytes(M, d, V, fb.FLY_BF16))
        st = fb.lib.fly_lmhead_entropy_argmax(p(hidden), p(wp), p(rs), M, d, V, fb.FLY_BF16, p(argmax), p(p1),
                                              p(hn), p(lse), p(ws), ws.numel(), None)
    assert st == 0, fb.strerror(st)
    torch.cuda.synchronize()
    return [t.cpu().numpy() for t in (argmax, p1, hn, lse)]


def test_static_scratch_lm_head_matches_the_workspace_one():
    from paper_2511_22972_amd import binding as fb
    # (rows, d, V): first a larger call, then a smaller one on the same array, then 128 rows at the
    # full vocabulary (11.7 of the 16 MiB)
    for M, d, V in ((36, 1024, 128256), (9, 512, 4112), (128, 256, 128256)):
        assert fb.fly_lmhead_workspace_bytes(M, d, V, fb.FLY_BF16) <= 16 << 20
        got = _run(fb, M, d, V, 3, static=True)
        ref = _run(fb, M, d, V, 3, static=False)
        for g, r in zip(got, ref):
            assert np.array_equal(g, r), (M, d, V)
        assert np.all(got[0] >= 0) and np.all(np.isfinite(got[3]))
    # a request that does not fit is refused, with nothing launched
    p = C.c_void_p(4096)
    assert fb.lib.fly_lmhead_entropy_argmax_static(p, p, None, 1088, 8192, 128256, fb.FLY_BF16, p, p, p, None, None) == -12
