"""The allocation-free scoring entry point against samkv_score: same kernels, scratch inside the library instead of
a caller workspace, so the scores must be bit-identical.  Two calls in a row on the same GPU share the scratch area;
the second is smaller, so anything left over from the first would show."""
import ctypes

import numpy as np
import pytest

from paper_2508_11661_amd import synth
from tests import helpers as H

pytestmark = pytest.mark.gpu


def _both(S, x, use_bias=True):
    import torch
    w = x.workload
    caches = H.upload_caches(x)
    q_tok = H.to_dev(x.q_tok, w.dtype)
    q_loc = H.to_dev(x.q_loc, w.dtype) if use_bias else None
    n_q_tok, w_loc = int(q_tok.shape[1]), (int(q_loc.shape[2]) if use_bias else 0)
    ws = torch.empty((S.samkv_workspace_bytes(len(x.k), w.n_q_heads, w.n_kv_heads, w.head_dim, n_q_tok, 1),),
                     dtype=torch.uint8, device="cuda")
    want = torch.full((w.n_kv_heads, caches.total_len), float("nan"), device="cuda")
    got = torch.full_like(want, float("nan"))
    stream = torch.cuda.current_stream().cuda_stream
    L = S._lib
    rc = L.samkv_score(ctypes.byref(caches.c), q_tok.data_ptr(), n_q_tok, q_loc.data_ptr() if use_bias else None, w_loc,
                       want.data_ptr(), ws.data_ptr(), ws.numel(), stream)
    assert rc == 0
    rc = L.samkv_score_noalloc(ctypes.byref(caches.c), q_tok.data_ptr(), n_q_tok, q_loc.data_ptr() if use_bias else None,
                               w_loc, got.data_ptr(), stream)
    assert rc == 0
    torch.cuda.synchronize()
    assert torch.isfinite(want).all()
    assert torch.equal(got, want), "scores of samkv_score_noalloc differ from samkv_score"
    return got


def test_score_noalloc_matches_score_twice_in_a_row():
    from paper_2508_11661_amd import samkv as S
    # first call: 70 documents (the three-kernel prologue: more than 64 documents), ragged lengths, bf16
    big = synth.make_small(71, "bf16", [130 + 7 * (i % 9) for i in range(70)], 16, 4, 128, 9, 12)
    _both(S, big)
    # second call, right after it and smaller in every dimension (the one-launch prologue), float32
    small = synth.make_small(72, "f32", [257, 64, 100], 4, 2, 64, 3, 5)
    _both(S, small)
    # and once more without the bias term
    _both(S, small, use_bias=False)


def test_score_noalloc_rejects_what_does_not_fit():
    from paper_2508_11661_amd import samkv as S
    import torch
    lens = (ctypes.c_int32 * 128)(*([8] * 128))
    fake = (ctypes.c_void_p * 128)(*([0x1000] * 128))
    c = S._Caches(128, 4096, 64, 128, 1, ctypes.cast(lens, ctypes.POINTER(ctypes.c_int32)),
                  ctypes.cast(fake, ctypes.POINTER(ctypes.c_void_p)), None)
    # 128 documents x 4096 query heads x 128 channels of float32 is far beyond the scratch area: refused, nothing launched
    assert S._lib.samkv_score_noalloc(ctypes.byref(c), 0x1000, 4, 0x1000, 2, 0x1000, None) == -2
    assert S._lib.samkv_score_noalloc(None, 0x1000, 4, None, 0, 0x1000, None) == -1
    torch.cuda.synchronize()
