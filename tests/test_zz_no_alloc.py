"""The decode entry point that allocates nothing (its split partials live in a static device
buffer inside the library): same o and lse as s2_attn_decode, on two calls in a row, the second
with a smaller input; shapes beyond the buffer are refused before any launch."""

import ctypes as C

import numpy as np
import pytest
import torch

from paper_2407_17678_amd import binding as B
from paper_2407_17678_amd import synth
from tests import gpu_util as G

LSE_TOL = 1e-3


def _case(nseq, H, D, max_len, S, Bl, stride, seed, splits):
    rng = np.random.default_rng(seed)
    lens = rng.integers(1, max_len + 1, size=nseq).astype(np.int32)
    lens[0] = max_len
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)
    q = torch.randn((nseq, H, D), device="cuda", generator=gen).to(torch.bfloat16)
    kc = torch.randn((nseq, H, max_len, D), device="cuda", generator=gen).to(torch.bfloat16)
    vc = torch.randn((nseq, H, max_len, D), device="cuda", generator=gen).to(torch.bfloat16)
    sl = torch.from_numpy(lens).cuda()
    p = B.layout_params(H, 1, S, Bl, stride)
    scale = 1.0 / np.sqrt(D)
    # the existing entry point, caller's workspace
    o_ref = torch.empty_like(q)
    lse_ref = torch.empty((nseq, H), dtype=torch.float32, device="cuda")
    ws = torch.full((B.s2_attn_decode_workspace_bytes(nseq, H, D, max_len, splits),), 0xFF, dtype=torch.uint8,
                    device="cuda")
    B.s2_attn_decode(p, q, kc, vc, sl, o_ref, lse_ref, scale, ws, max_len, num_splits=splits)
    # the static-buffer entry point
    o = torch.zeros_like(q)
    lse = torch.zeros((nseq, H), dtype=torch.float32, device="cuda")
    B.s2_attn_decode_static(p, q, kc, vc, sl, o, lse, scale, max_len, num_splits=splits)
    torch.cuda.synchronize()
    return G.to_f64(o), G.to_f64(lse), G.to_f64(o_ref), G.to_f64(lse_ref)


@pytest.mark.gpu
def test_static_decode_matches_workspace_decode_twice():
    # first call: 6 sequences up to 2000 tokens, 5 splits; second call: smaller in every respect,
    # so stale partials of the first call sit beyond (and among) the ones the second call uses
    for args in ((6, 8, 128, 2000, 64, 3, 4, 11, 5), (2, 4, 128, 700, 64, 3, 4, 12, 2),
                 (3, 4, 64, 300, 32, 2, 4, 13, 0)):
        o, lse, o_ref, lse_ref = _case(*args)
        # same kernels, same partial layout: the bar is the tolerance on O and LSE, and in fact equality
        assert G.o_excess(o, o_ref) <= 0 and np.abs(lse - lse_ref).max() <= LSE_TOL, args
        assert np.array_equal(o, o_ref) and np.array_equal(lse, lse_ref), args


@pytest.mark.gpu
def test_static_decode_refuses_what_does_not_fit():
    nseq, H, D, max_len = 512, 64, 128, 65536   # 512 * 64 * 64 splits * 130 floats >> the static buffer
    p = B.layout_params(H, 1, 64, 16, 16)
    need = B.s2_attn_decode_workspace_bytes(nseq, H, D, max_len, 64)
    assert need > 8 << 20
    one = torch.zeros(16, dtype=torch.bfloat16, device="cuda")   # never touched: the call fails first
    a = B.DecodeArgs(one.data_ptr(), one.data_ptr(), one.data_ptr(), one.data_ptr(), one.data_ptr(), None,
                     nseq, H, D, max_len, 64, 8, 8, 8)
    st = B.lib().s2_attn_decode_static(C.byref(p), C.byref(a), 0.1, None)
    assert st == -5   # S2_ERR_WORKSPACE


def test_static_decode_size_check_needs_no_device():
    """The refusal comes from the sizes alone, before any device call (runs without a GPU)."""
    p = B.layout_params(64, 1, 64, 16, 16)
    a = B.DecodeArgs(16, 16, 16, 16, 16, None, 512, 64, 128, 65536, 64, 8, 8, 8)
    assert B.lib().s2_attn_decode_static(C.byref(p), C.byref(a), 0.1, None) == -5   # S2_ERR_WORKSPACE
    assert B.lib().s2_attn_decode_static(None, C.byref(a), 0.1, None) == -1         # S2_ERR_NULL
