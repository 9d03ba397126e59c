"""CPU-side checks of the C ABI: the library loads, exports every symbol the
header declares, and rejects bad arguments before touching the GPU."""
import ctypes
import os
import re

import pytest

import paper_2604_21335_amd as stc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "stc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(stc_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = stc.load_library()
    names = _declared_symbols()
    assert set(names) == set(stc.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None
    assert stc.stc_version() >= 1
    assert stc.status_string(0) == "ok"
    assert "aligned" in stc.status_string(stc.STC_ERR_ALIGN)


def _shape(**kw):
    d = dict(B=2, Hq=8, Hkv=2, D=128, N=100, G=8, v_cap_groups=800, N_cap=0)
    d.update(kw)
    return stc.make_shape(**d)


FAKE = ctypes.c_void_p(0x1000)      # aligned, never dereferenced: calls must fail earlier
ODD = ctypes.c_void_p(0x1004)


@pytest.mark.parametrize("kw", [dict(D=96), dict(P=8), dict(G=3), dict(G=32), dict(Hq=7),
                                dict(Hq=64, Hkv=2), dict(N=0), dict(B=0), dict(D=64, G=16),
                                dict(v_cap_groups=-1), dict(B=70000, Hkv=1, Hq=1)])
def test_bad_shapes_are_rejected(kw):
    lib = stc.load_library()
    s = _shape(**kw)
    assert lib.stc_build_page_bounds(ctypes.byref(s), FAKE, FAKE, None) == stc.STC_ERR_SHAPE
    assert stc.stc_workspace_bytes(s, stc.STC_WS_ROUTE) == 0
    assert lib.stc_select_pages(ctypes.byref(s), FAKE, FAKE, 2, FAKE, None, FAKE, 1 << 30,
                                None) == stc.STC_ERR_SHAPE
    assert lib.stc_decode_attention(ctypes.byref(s), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 2, FAKE,
                                    FAKE, 1 << 30, None) == stc.STC_ERR_SHAPE


def test_null_alignment_and_workspace_errors():
    lib = stc.load_library()
    s = _shape()
    r = ctypes.byref(s)
    assert lib.stc_build_page_bounds(r, None, FAKE, None) == stc.STC_ERR_NULL
    assert lib.stc_build_page_bounds(None, FAKE, FAKE, None) == stc.STC_ERR_NULL
    assert lib.stc_build_page_bounds(r, ODD, FAKE, None) == stc.STC_ERR_ALIGN
    # route: mode checks, missing inputs, workspace too small
    big = 1 << 30
    args = lambda mode, logits, kc, fk, min_, ws, wsb: lib.stc_route_and_pack_values(  # noqa: E731
        r, mode, FAKE, logits, kc, fk, min_, FAKE, FAKE, FAKE, None, ws, wsb, None)
    assert args(stc.STC_ROUTE_TOPK, None, None, 2, None, FAKE, big) == stc.STC_ERR_NULL
    assert args(stc.STC_ROUTE_MASK, None, None, 0, None, FAKE, big) == stc.STC_ERR_NULL
    assert args(stc.STC_ROUTE_TOPK, FAKE, None, 9, None, FAKE, big) == stc.STC_ERR_SHAPE
    assert args(stc.STC_ROUTE_TOPK, FAKE, None, -1, None, FAKE, big) == stc.STC_ERR_SHAPE
    assert args(7, FAKE, None, 2, FAKE, FAKE, big) == stc.STC_ERR_SHAPE
    assert args(stc.STC_ROUTE_SHARED | 7, FAKE, None, 2, FAKE, FAKE, big) == stc.STC_ERR_SHAPE
    assert args(stc.STC_ROUTE_SHARED | stc.STC_ROUTE_TOPK, None, None, 2, None, FAKE,
                big) == stc.STC_ERR_NULL
    # shared masks cannot be routed in place (the output has one row per KV head)
    assert args(stc.STC_ROUTE_SHARED | stc.STC_ROUTE_MASK, None, None, 0, FAKE, FAKE,
                big) == stc.STC_ERR_SHAPE
    assert args(stc.STC_ROUTE_GLOBAL, None, None, 2, None, FAKE, big) == stc.STC_ERR_NULL
    assert args(stc.STC_ROUTE_GLOBAL, FAKE, None, 9, None, FAKE, big) == stc.STC_ERR_SHAPE
    assert args(stc.STC_ROUTE_GLOBAL, FAKE, None, 2, None, FAKE, 0) == stc.STC_ERR_WORKSPACE
    assert args(stc.STC_ROUTE_TOPK, FAKE, None, 2, None, FAKE, 0) == stc.STC_ERR_WORKSPACE
    assert args(stc.STC_ROUTE_TOPK, FAKE, None, 2, None, None, big) == stc.STC_ERR_WORKSPACE
    # select: k out of range, scores need a workspace when page_score is NULL
    assert lib.stc_select_pages(r, FAKE, FAKE, 0, FAKE, None, FAKE, big, None) == stc.STC_ERR_SHAPE
    assert lib.stc_select_pages(r, FAKE, FAKE, 2, FAKE, None, None, 0, None) == stc.STC_ERR_WORKSPACE
    assert lib.stc_select_pages(r, None, FAKE, 2, FAKE, None, FAKE, big, None) == stc.STC_ERR_NULL
    assert lib.stc_select_pages(r, FAKE, ODD, 2, FAKE, FAKE, FAKE, big, None) == stc.STC_ERR_ALIGN
    assert lib.stc_score_pages(r, FAKE, FAKE, None, None) == stc.STC_ERR_NULL
    assert lib.stc_score_pages(r, FAKE, ODD, FAKE, None) == stc.STC_ERR_ALIGN
    assert lib.stc_score_pages(ctypes.byref(_shape(G=5)), FAKE, FAKE, FAKE, None) == stc.STC_ERR_SHAPE
    # attention: k_pages beyond NP (= 7), missing workspace
    att = lambda k, ws, wsb, out=FAKE: lib.stc_decode_attention(  # noqa: E731
        r, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, k, out, ws, wsb, None)
    assert att(8, FAKE, big) == stc.STC_ERR_SHAPE
    assert att(0, FAKE, big) == stc.STC_ERR_SHAPE
    assert att(7, FAKE, big, None) == stc.STC_ERR_NULL
    assert stc.stc_workspace_bytes(s, stc.STC_WS_ATTENTION, 7) == 0       # one split: no partials
    s2 = _shape(N=4096, v_cap_groups=4096 * 8)
    need = stc.stc_workspace_bytes(s2, stc.STC_WS_ATTENTION, 64)
    assert need > 0
    att2 = lambda ws, wsb: lib.stc_decode_attention(  # noqa: E731
        ctypes.byref(s2), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 64, FAKE, ws, wsb, None)
    assert att2(FAKE, need - 1) == stc.STC_ERR_WORKSPACE
    assert att2(None, big) == stc.STC_ERR_WORKSPACE
    assert lib.stc_decode_attention(ctypes.byref(_shape(v_cap_groups=0)), FAKE, FAKE, FAKE, FAKE,
                                    FAKE, FAKE, 7, FAKE, FAKE, big, None) == stc.STC_ERR_SHAPE
    # one-call step: workspace = scores + attention partials, page list required
    step = lambda q, idx, k, ws, wsb, sh=s2: lib.stc_decode_step(  # noqa: E731
        ctypes.byref(sh), q, FAKE, FAKE, FAKE, FAKE, FAKE, k, idx, FAKE, ws, wsb, None)
    need_step = stc.stc_workspace_bytes(s2, stc.STC_WS_STEP, 64)
    assert need_step >= need + stc.stc_workspace_bytes(s2, stc.STC_WS_SELECT, 64)
    assert step(FAKE, FAKE, 64, FAKE, need_step - 1) == stc.STC_ERR_WORKSPACE
    assert step(FAKE, FAKE, 64, None, big) == stc.STC_ERR_WORKSPACE
    assert step(FAKE, None, 64, FAKE, big) == stc.STC_ERR_NULL
    assert step(None, FAKE, 64, FAKE, big) == stc.STC_ERR_NULL
    assert step(FAKE, ODD, 64, FAKE, big) == stc.STC_ERR_ALIGN
    assert step(FAKE, FAKE, 0, FAKE, big) == stc.STC_ERR_SHAPE
    assert step(FAKE, FAKE, 257, FAKE, big) == stc.STC_ERR_SHAPE
    assert stc.stc_workspace_bytes(s, stc.STC_WS_STEP, 7) == 0       # every page kept, one split
    stept = lambda n, capt, ws, wsb: lib.stc_decode_step_tail(  # noqa: E731
        ctypes.byref(s2), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 64, FAKE, FAKE, n, capt, FAKE, FAKE,
        ws, wsb, None)
    need_tail = stc.stc_workspace_bytes(s2, stc.STC_WS_STEP_TAIL, 64 + 3)
    assert need_tail >= need_step
    assert stept(40, 48, FAKE, need_tail - 1) == stc.STC_ERR_WORKSPACE
    assert stept(49, 48, FAKE, big) == stc.STC_ERR_SHAPE
    assert stept(-1, 48, FAKE, big) == stc.STC_ERR_SHAPE
    # attention with a tail: tail arguments
    tail = lambda kt, vt, n, capt: lib.stc_decode_attention_tail(  # noqa: E731
        r, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 7, kt, vt, n, capt, FAKE, FAKE, big, None)
    assert tail(None, None, 3, 8) == stc.STC_ERR_NULL
    assert tail(FAKE, FAKE, 9, 8) == stc.STC_ERR_SHAPE
    assert tail(FAKE, FAKE, -1, 8) == stc.STC_ERR_SHAPE
    assert tail(ODD, FAKE, 3, 8) == stc.STC_ERR_ALIGN
    assert stc.stc_workspace_bytes(s, stc.STC_WS_ATTENTION_TAIL, 7 + 1) == 0     # still one split
    assert stc.stc_workspace_bytes(s, stc.STC_WS_ATTENTION_TAIL, 7 + 40) > 0
    assert lib.stc_decode_attention_tail(r, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 7, FAKE, FAKE, 600,
                                         640, FAKE, None, 0, None) == stc.STC_ERR_WORKSPACE
    assert lib.stc_append_tail(r, FAKE, FAKE, FAKE, FAKE, 8, 8, None) == stc.STC_ERR_SHAPE
    assert lib.stc_append_tail(r, FAKE, None, FAKE, FAKE, 0, 8, None) == stc.STC_ERR_NULL
    assert lib.stc_append_tail(r, ODD, FAKE, FAKE, FAKE, 0, 8, None) == stc.STC_ERR_ALIGN
    # per-head calls: same checks, their own workspace sizes
    assert lib.stc_select_pages_per_head(r, FAKE, FAKE, 2, FAKE, None, None, 0,
                                         None) == stc.STC_ERR_WORKSPACE
    assert lib.stc_select_pages_per_head(r, None, FAKE, 2, FAKE, None, FAKE, big,
                                         None) == stc.STC_ERR_NULL
    assert stc.stc_workspace_bytes(s, stc.STC_WS_SELECT_PER_HEAD, 2) == 2 * 8 * 7 * 4
    assert stc.stc_workspace_bytes(s, stc.STC_WS_SELECT, 2) == 2 * 2 * 7 * 4
    assert lib.stc_decode_attention_per_head(r, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 8, FAKE, FAKE,
                                             big, None) == stc.STC_ERR_SHAPE
    assert lib.stc_decode_attention_per_head(r, FAKE, FAKE, FAKE, FAKE, FAKE, ODD, 7, FAKE, FAKE,
                                             big, None) == stc.STC_ERR_ALIGN
    # flush of tail tokens into the cache: needs room (N_cap) and a routing input
    sc = _shape(N_cap=140)
    rc = ctypes.byref(sc)
    fl = lambda shp, n, mode, logits, mask_in, K=FAKE, n_tail=64: lib.stc_flush_tail(  # noqa: E731
        shp, FAKE, FAKE, n, n_tail, 64, mode, logits, None, 2, mask_in, K, FAKE, FAKE, FAKE, FAKE,
        None, None)
    assert fl(r, 8, stc.STC_ROUTE_TOPK, FAKE, None) == stc.STC_ERR_SHAPE        # no capacity
    assert fl(rc, 41, stc.STC_ROUTE_TOPK, FAKE, None) == stc.STC_ERR_SHAPE      # 100 + 41 > 140
    assert fl(rc, 0, stc.STC_ROUTE_TOPK, FAKE, None) == stc.STC_ERR_SHAPE
    assert fl(rc, 8, stc.STC_ROUTE_TOPK, FAKE, None, n_tail=7) == stc.STC_ERR_SHAPE   # more than the tail holds
    assert fl(rc, 8, stc.STC_ROUTE_TOPK, FAKE, None, n_tail=65) == stc.STC_ERR_SHAPE  # beyond tail_cap
    assert fl(rc, 8, stc.STC_ROUTE_GLOBAL, FAKE, None) == stc.STC_ERR_SHAPE
    assert fl(rc, 8, stc.STC_ROUTE_TOPK, None, None) == stc.STC_ERR_NULL
    assert fl(rc, 8, stc.STC_ROUTE_MASK, None, None) == stc.STC_ERR_NULL
    assert fl(rc, 8, stc.STC_ROUTE_MASK, None, FAKE, None) == stc.STC_ERR_NULL
    assert fl(rc, 8, stc.STC_ROUTE_MASK, None, ODD) == stc.STC_ERR_ALIGN
    assert lib.stc_build_page_bounds(ctypes.byref(_shape(N_cap=50)), FAKE, FAKE,
                                     None) == stc.STC_ERR_SHAPE                  # capacity < N
    assert stc.stc_bounds_bytes(sc) == 2 * 2 * 2 * 8 * 128 * 4                   # 9 pages -> 2 tiles
    # union of per-head lists
    un = lambda k, cap, lists=FAKE: lib.stc_union_pages(r, lists, k, FAKE, FAKE, cap, None)  # noqa: E731
    assert un(2, 6) == stc.STC_ERR_SHAPE                       # capacity below min(NP, R*k) = 7
    assert un(0, 7) == stc.STC_ERR_SHAPE
    assert un(2, 7, None) == stc.STC_ERR_NULL
    assert lib.stc_decode_attention_union(r, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None, 7, FAKE,
                                          FAKE, big, None) == stc.STC_ERR_NULL
    # router projection
    rl = lambda B, dm, G, h=FAKE, bias=None, per=0: lib.stc_router_logits(  # noqa: E731
        B, 2, 10, dm, G, h, FAKE, bias, per, FAKE, None)
    assert rl(1, 100, 8) == stc.STC_ERR_SHAPE and rl(1, 256, 3) == stc.STC_ERR_SHAPE
    assert rl(0, 256, 8) == stc.STC_ERR_SHAPE
    assert rl(1, 256, 8, None) == stc.STC_ERR_NULL
    assert rl(1, 256, 8, ODD) == stc.STC_ERR_ALIGN
    assert rl(1, 256, 8, FAKE, ctypes.c_void_p(0x1002)) == stc.STC_ERR_ALIGN
    assert rl(1, 256, 8, FAKE, FAKE, 2) == stc.STC_ERR_SHAPE     # bias_per_batch is 0 or 1
    assert rl(1, 256, 8, FAKE, FAKE, -1) == stc.STC_ERR_SHAPE
    # compact
    assert lib.stc_compact_tokens(FAKE, FAKE, FAKE, 1, 1, 10, 4, 100, None, None) == stc.STC_ERR_SHAPE
    assert lib.stc_compact_tokens(FAKE, None, FAKE, 1, 1, 10, 4, 128, None, None) == stc.STC_ERR_NULL


def test_workspace_sizes():
    s = _shape(N=4096, v_cap_groups=4096 * 8)
    # kept groups and equal keys per chunk of 256 tokens, a 4096-bin histogram and 16 bytes of
    # selection state per stream, each region rounded up to 256 bytes
    assert stc.stc_workspace_bytes(s, stc.STC_WS_ROUTE) == 256 + 256 + 4 * 4096 * 4 + 256
    assert stc.stc_workspace_bytes(s, stc.STC_WS_SELECT, 64) == 2 * 2 * 256 * 4
    assert stc.stc_workspace_bytes(s, stc.STC_WS_SELECT, 256) == 0       # all pages: no scores
    assert stc.stc_workspace_bytes(s, stc.STC_WS_ATTENTION, 300) == 0    # k beyond NP
    assert stc.stc_workspace_bytes(s, 99, 1) == 0


def test_bounds_layout_matches_the_header():
    """stc_bounds_bytes, and bounds_rows() against the index formula stc.h states:
    dword [s][t][j][g][e][col][w] = page 8t+4g+col, channel e*(D/8)+4j+w, (min, max)."""
    import numpy as np
    import torch
    for D, N in ((128, 300), (64, 16 * 8)):
        s = _shape(D=D, N=N, G=4, v_cap_groups=N * 4)
        NP = (N + 15) // 16
        nt = (NP + 7) // 8
        assert stc.stc_bounds_bytes(s) == 2 * 2 * nt * 8 * D * 4
        buf = np.zeros((2 * 2, nt, D // 32, 2, 8, 4, 4, 2), dtype=np.int16)
        want = np.zeros((2 * 2, NP, 2, D), dtype=np.int16)
        for st in range(4):
            for p in range(NP):
                for c in range(D):
                    mn, mx = (st * 7 + p * 131 + c) % 30000, 30000 - ((p * 17 + c * 3 + st) % 999)
                    t, g, col = p // 8, (p % 8) // 4, p % 4
                    e, j, w = c // (D // 8), (c % (D // 8)) // 4, c % 4
                    buf[st, t, j, g, e, col, w] = (mn, mx)
                    want[st, p, 0, c], want[st, p, 1, c] = mn, mx
        got = stc.bounds_rows(torch.from_numpy(buf.reshape(-1)).view(torch.bfloat16), s)
        assert got.shape == (2, 2, NP, 2, D)
        assert np.array_equal(got.view(torch.int16).numpy().reshape(4, NP, 2, D), want)
    assert stc.stc_bounds_bytes(_shape(D=96)) == 0


def test_binding_refuses_host_tensors():
    import torch
    s = _shape()
    with pytest.raises(TypeError):
        stc.stc_build_page_bounds(s, torch.zeros(4, dtype=torch.bfloat16),
                                  torch.zeros(4, dtype=torch.bfloat16))


def test_workload_generator_is_counter_based_and_seeded():
    import torch
    from paper_2604_21335_amd import workloads as W
    a = W.normal(5, W.TAG_K, 1000)
    b = torch.cat([W.normal(5, W.TAG_K, 400), W.normal(5, W.TAG_K, 600, offset=400)])
    assert torch.equal(a, b)
    assert not torch.equal(a, W.normal(6, W.TAG_K, 1000))
    assert not torch.equal(a, W.normal(5, W.TAG_V, 1000))
    big = W.normal(0, W.TAG_K, 200000)
    assert abs(float(big.mean())) < 0.01 and abs(float(big.std()) - 1.0) < 0.01
    w = W.WORKLOADS["qwen25_7b_32k"]
    kc = W.counts_from_pmf(2, W.TAG_KCOUNT, (50000,), W._pmf(w)).to(torch.float64)
    assert kc.min() == 1 and kc.max() == 8 and abs(float(kc.mean()) - 4.01) < 0.05
    w4 = W.WORKLOADS["qwen25_7b_128k"]
    kc = W.counts_from_pmf(4, W.TAG_KCOUNT, (50000,), W._pmf(w4)).to(torch.float64)
    assert kc.min() >= 1 and kc.max() <= 16 and abs(float(kc.mean()) - 4.0) < 0.05
    tiny = W.make_cache_inputs(W.shrink(W.WORKLOADS["tiny"], N=64))
    m = W.u16_numpy(tiny["mask_in"])
    assert m.min() >= 1 and m.max() < 16
    vlm = W.make_cache_inputs(W.shrink(W.WORKLOADS["llava15_7b_prefix"], B=2, Hq=2, Hkv=2))
    ti = vlm["token_idx"]
    assert ti.shape == (2, 208) and bool((ti[:, 1:] > ti[:, :-1]).all())
    assert int(ti[:, 143].max()) < 576 and int(ti[0, 144]) == 576


def test_header_is_plain_c_and_links(tmp_path):
    """include/stc.h compiles as C99 with warnings as errors, and a C program linked against
    libstc.so gets version, status strings, sizes and argument errors without a GPU."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    libdir = os.path.join(root, "paper_2604_21335_amd")
    exe = str(tmp_path / "c_abi_check")
    subprocess.run([gcc, "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror",
                    "-I", os.path.join(root, "include"),
                    os.path.join(root, "tests", "c_abi_check.c"), "-o", exe,
                    "-L", libdir, "-lstc", "-Wl,-rpath," + libdir], check=True)
    out = subprocess.run([exe], capture_output=True, text=True)
    assert out.returncode == 0, out.stdout + out.stderr


@pytest.mark.parametrize("which", ["STC_WS_ATTENTION", "STC_WS_ATTENTION_TAIL", "STC_WS_STEP_TAIL",
                                   "STC_WS_ATTENTION_PER_HEAD"])
@pytest.mark.parametrize("B,Hq,Hkv", [(8, 28, 4), (1, 8, 8), (16, 28, 4), (2, 32, 32)])
def test_attention_workspace_never_shrinks_when_the_page_count_grows(which, B, Hq, Hkv):
    """A buffer sized for the largest number of page slots (selected pages plus tail pages)
    must serve every smaller number: the launch plan changes with the count, the size bound
    may not."""
    s = stc.make_shape(B=B, Hq=Hq, Hkv=Hkv, D=128, N=16 * 400, G=8, v_cap_groups=16 * 400 * 8)
    sizes = [stc.stc_workspace_bytes(s, getattr(stc, which), k) for k in range(1, 401)]
    assert all(b >= a for a, b in zip(sizes, sizes[1:])), which
    assert sizes[-1] > 0


def test_static_scratch_limit_is_checked_on_the_host():
    s = stc.make_shape(B=256, Hq=32, Hkv=32, D=128, N=4096, G=8, v_cap_groups=4096 * 8)
    assert stc.stc_workspace_bytes(s, stc.STC_WS_STEP, 128) > stc.STC_STATIC_SCRATCH_BYTES
    rc = stc.load_library().stc_decode_step_static(ctypes.byref(s), FAKE, FAKE, FAKE, FAKE, FAKE,
                                                   FAKE, 128, FAKE, FAKE, None)
    assert rc == stc.STC_ERR_WORKSPACE
