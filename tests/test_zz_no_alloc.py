"""stc_decode_step_static (the entry point for callers that cannot allocate: its scratch
memory is a static device array of the library) against stc_decode_step, through the C ABI:
two calls in a row on the shared array, the second on a smaller input, each bit for bit the
result of the workspace form."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2604_21335_amd as stc
from paper_2604_21335_amd import workloads as W

pytestmark = pytest.mark.gpu


def _cache(w, dev, layer):
    inp = W.make_cache_inputs(w, dev, layer=layer)
    c = stc.RoutedCache(w.B, w.Hq, w.Hkv, w.D, w.N, w.G, w.k_pages, device=dev)
    c.build(inp["K"], inp["V"], logits=inp["logits"], kcount=inp["kcount"], mask_in=inp["mask_in"])
    return c


def _both(c, q):
    """(page list, output) of the workspace form and of the static-scratch form."""
    c.page_idx.fill_(-7)
    c.out.fill_(float("nan"))
    c.step(q)                                             # stc_decode_step, its own workspace
    torch.cuda.synchronize()
    ref = (c.page_idx.clone(), c.out.clone())
    idx = torch.full_like(c.page_idx, -9)
    out = torch.full_like(c.out, float("nan"))
    stc.stc_decode_step_static(c.shape, q, c.bounds, c.K, c.vpacked, c.mask, c.tok_off, c.k_eff,
                               idx, out)
    torch.cuda.synchronize()
    return ref, (idx, out)


def test_static_scratch_step_equals_workspace_step_twice_second_smaller():
    dev = "cuda:0"
    base = W.WORKLOADS["qwen25_7b_32k"]
    # several splits per stream and a ragged last page; then a smaller shape (fewer streams,
    # fewer pages, fewer splits) on the array the first call left behind
    big = W.shrink(base, B=3, Hq=14, Hkv=2, N=16 * 700 + 5, k_pages=72)
    small = W.shrink(base, B=1, Hq=14, Hkv=2, N=16 * 90 + 3, k_pages=20)
    for n, w in enumerate((big, small)):
        c = _cache(w, dev, n)
        q = W.make_query(w, n, dev)
        (ridx, rout), (sidx, sout) = _both(c, q)
        assert int(ridx.min()) >= 0 and torch.isfinite(rout).all()
        assert torch.equal(ridx, sidx), "page lists differ (%s)" % w.name
        assert torch.equal(rout.view(torch.int32), sout.view(torch.int32)), \
            "outputs differ (%s)" % w.name


def test_static_scratch_rejects_sizes_beyond_its_array():
    # more split partials than the array holds: refused on the host, nothing enqueued
    s = stc.make_shape(B=256, Hq=32, Hkv=32, D=128, N=4096, G=8, v_cap_groups=4096 * 8)
    assert stc.stc_workspace_bytes(s, stc.STC_WS_STEP, 128) > stc.STC_STATIC_SCRATCH_BYTES
    fake = ctypes.c_void_p(0x1000)
    rc = stc.load_library().stc_decode_step_static(ctypes.byref(s), fake, fake, fake, fake, fake,
                                                   fake, 128, fake, fake, None)
    assert rc == stc.STC_ERR_WORKSPACE
