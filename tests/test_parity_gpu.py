"""GPU parity: the HIP path through the C ABI against the CPU oracle, element by
element.  Bit-exact for bounds, masks, offsets, packed values, page scores and
page indices; max abs error <= 2e-3 for the attention output."""
import numpy as np
import pytest
import torch

import paper_2604_21335_amd as stc
from oracle import stc_oracle as O
from paper_2604_21335_amd import workloads as W
from tests import parity as PT
from tests.helpers import f32_to_bf16_bits, ints_bf16, randn_bf16

pytestmark = pytest.mark.gpu


def _rand_case(seed, B, Hq, Hkv, D, N, G, qscale=1.0, outliers=False):
    rng = np.random.default_rng(seed)
    Kf = rng.standard_normal((B, Hkv, N, D)).astype(np.float32)
    if outliers:
        for h in range(Hkv):
            Kf[:, h, :, rng.choice(D, 4, replace=False)] *= 8.0
    K = f32_to_bf16_bits(Kf)
    V = randn_bf16(rng, (B, Hkv, N, D))
    q = randn_bf16(rng, (B, Hq, D), qscale)
    logits = rng.standard_normal((B, Hkv, N, G)).astype(np.float32)
    kcount = rng.integers(0, G + 1, size=(B, Hkv, N)).astype(np.uint8)
    return K, V, q, logits, kcount


# (B, Hq, Hkv, D, N, G, k_pages): several tiles / chunks, ragged tails, every head-group path
CASES = [
    (1, 8, 8, 64, 1024, 4, 16),        # the tiny config's shape
    (2, 4, 4, 128, 1000, 8, 10),       # N % 16 != 0, N % 256 != 0
    (2, 14, 2, 128, 2500, 8, 40),      # GQA 7:1, ragged
    (1, 8, 1, 128, 777, 16, 13),       # GQA 8:1, G = 16 (8-wide groups)
    (3, 6, 3, 64, 530, 8, 9),          # GQA 2:1, D = 64 with 8-wide groups
    (1, 4, 1, 128, 4096, 1, 64),       # G = 1
    (1, 3, 1, 64, 300, 2, 5),          # group size 3: generic score kernel
    (2, 2, 2, 128, 16, 8, 1),          # a single page
    (1, 1, 1, 64, 5, 4, 1),            # fewer tokens than a page
    (1, 16, 1, 128, 640, 4, 12),       # 16 query heads on one KV head
    (48, 4, 4, 64, 600, 4, 9),         # 192 streams: a workgroup scores and selects a stream
    (49, 28, 4, 128, 1000, 8, 20),     # the same with 7 heads per KV head
    (64, 6, 3, 128, 20, 8, 1),         # 192 streams of two pages
    (2, 10, 2, 128, 1300, 8, 17),      # GQA 5:1 at D = 128: query operands in shared memory
    (1, 12, 2, 128, 905, 4, 11),       # GQA 6:1, ragged, more scoring workgroups than tiles
    (3, 24, 3, 128, 40, 8, 2),         # GQA 8:1 on three pages
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: "B%d_Hq%d_Hkv%d_D%d_N%d_G%d_k%d" % c)
def test_parity_topk_routing(case):
    B, Hq, Hkv, D, N, G, k = case
    K, V, q, logits, kcount = _rand_case(hash(case) % 1000, B, Hq, Hkv, D, N, G, outliers=True)
    hip = PT.run_hip(K, V, q, G, k, logits=logits, kcount=kcount)
    ora = PT.run_oracle(K, V, q, G, k, logits=logits, kcount=kcount)
    assert hip["dev_status"] == 0
    worst = PT.compare(hip, ora, Hq, Hkv)
    assert worst <= PT.TIGHT


@pytest.mark.parametrize("seed", range(24))
def test_random_shapes_and_modes(seed):
    """A seeded sweep over shapes, group sizes, routing modes and tail lengths (small enough for
    the oracle, ragged almost everywhere): every stream against the oracle."""
    rng = np.random.default_rng(1000 + seed)
    D = int(rng.choice([64, 128]))
    G = int(rng.choice([g for g in (1, 2, 4, 8, 16) if D // g >= 8]))
    R = int(rng.choice([1, 2, 3, 4, 5, 6, 7, 8, 12, 16]))
    Hkv, B = int(rng.integers(1, 4)), int(rng.integers(1, 3))
    Hq = Hkv * R
    N = int(rng.integers(1, 1200))
    NP = (N + 15) // 16
    k = int(rng.integers(1, NP + 3))
    ntail = int(rng.choice([0, 0, 1, 16, int(rng.integers(1, 41))]))
    K, V, q, logits, kcount = _rand_case(2000 + seed, B, Hq, Hkv, D, N, G, outliers=bool(seed % 2))
    mode = seed % 4
    kw = {}
    if mode == 0:
        kw = dict(logits=logits, kcount=kcount)
    elif mode == 1:
        kw = dict(logits=logits, kcount=int(rng.integers(0, G + 1)))
    elif mode == 2:
        kw = dict(mask_in=rng.integers(0, 1 << 16, size=(B, Hkv, N)).astype(np.uint16))
    else:
        kw = dict(logits=logits, global_k=int(rng.integers(0, G + 1)))
    hip = PT.run_hip(K, V, q, G, k, **kw)
    ora = PT.run_oracle(K, V, q, G, k, **kw)
    assert hip["dev_status"] == 0
    assert PT.compare(hip, ora, Hq, Hkv) <= PT.TIGHT
    if ntail:
        c = hip["cache"]
        cap_t = ntail + int(rng.integers(0, 9))
        Kt, Vt = randn_bf16(rng, (B, Hkv, cap_t, D)), randn_bf16(rng, (B, Hkv, cap_t, D))
        slots = c.k_eff + (ntail + 15) // 16
        ws = torch.empty(max(16, stc.stc_workspace_bytes(c.shape, stc.STC_WS_ATTENTION_TAIL, slots)),
                         dtype=torch.uint8, device="cuda:0")
        out = torch.full_like(c.out, float("nan"))
        stc.stc_decode_attention_tail(c.shape, PT.to_dev_bf16(q), c.K, c.vpacked, c.mask, c.tok_off,
                                      c.page_idx, c.k_eff, PT.to_dev_bf16(Kt), PT.to_dev_bf16(Vt),
                                      ntail, cap_t, out, ws)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        for b in range(B):
            for h in range(Hkv):
                want = O.decode_attention(q[b, h * R:(h + 1) * R], K[b, h], V[b, h],
                                          hip["mask"][b, h], hip["page_idx"][b, h], G,
                                          K_tail=Kt[b, h, :ntail], V_tail=Vt[b, h, :ntail])
                assert np.abs(got[b, h * R:(h + 1) * R] - want).max() < PT.TIGHT


def test_missing_page_list_means_leading_pages():
    """stc_decode_attention with page_idx == NULL attends pages 0 .. k-1: the same bits as the
    explicit list, for the whole cache and for a prefix of it."""
    B, Hq, Hkv, D, N, G = 2, 8, 2, 128, 700, 8
    K, V, q, logits, kcount = _rand_case(27, B, Hq, Hkv, D, N, G)
    NP = (N + 15) // 16
    hip = PT.run_hip(K, V, q, G, NP, logits=logits, kcount=kcount)     # step() passes no list
    ora = PT.run_oracle(K, V, q, G, NP, logits=logits, kcount=kcount)
    assert PT.compare(hip, ora, Hq, Hkv) <= PT.TIGHT
    c = hip["cache"]
    dq = PT.to_dev_bf16(q)
    for k in (NP, 9):
        idx = torch.arange(k, dtype=torch.int32, device="cuda:0").expand(B, Hkv, k).contiguous()
        a, b_ = torch.empty_like(c.out), torch.empty_like(c.out)
        ws = torch.empty(max(16, stc.stc_workspace_bytes(c.shape, stc.STC_WS_ATTENTION, k)),
                         dtype=torch.uint8, device="cuda:0")
        stc.stc_decode_attention(c.shape, dq, c.K, c.vpacked, c.mask, c.tok_off, idx, k, a, ws)
        stc.stc_decode_attention(c.shape, dq, c.K, c.vpacked, c.mask, c.tok_off, None, k, b_, ws)
        torch.cuda.synchronize()
        assert torch.equal(a, b_)
        if k == NP:
            assert np.array_equal(a.cpu().numpy(), hip["out"])
    # the one-call step with every page kept: no selection, the list 0 .. NP-1 is still written
    # (by the attention kernel itself), the output is the attention call's
    lst = torch.full((B, Hkv, NP), -7, dtype=torch.int32, device="cuda:0")
    o = torch.full_like(c.out, float("nan"))
    ws = torch.empty(max(16, stc.stc_workspace_bytes(c.shape, stc.STC_WS_STEP, NP)),
                     dtype=torch.uint8, device="cuda:0")
    stc.stc_decode_step(c.shape, dq, c.bounds, c.K, c.vpacked, c.mask, c.tok_off, NP, lst, o, ws)
    torch.cuda.synchronize()
    assert torch.equal(lst, torch.arange(NP, dtype=torch.int32, device="cuda:0").expand(B, Hkv, NP))
    assert np.array_equal(o.cpu().numpy(), hip["out"])


@pytest.mark.parametrize("B,Hkv,R,N,k", [
    (16, 4, 2, 32768, 128),     # 64 streams x 8 workgroups: selection inside the attention kernel
    (16, 4, 2, 32768, 144),     # 9 workgroups per stream: selection launch + attention launch
    (2, 2, 7, 32784, 128),      # 2049 pages: one too many for the keys held in registers
    (3, 1, 4, 4000, 7),         # workgroups of 4 wavefronts, ragged last page
    (1, 2, 1, 3333, 100),       # 7 workgroups of 8 wavefronts, ragged list end
])
def test_decode_step_is_the_two_calls_in_one(B, Hkv, R, N, k):
    """stc_decode_step through the C ABI with a workspace of its own, used twice without
    clearing: page list and output bit for bit those of stc_select_pages followed by
    stc_decode_attention, on both sides of every switch between its two launch plans."""
    Hq, D, G = Hkv * R, 128, 8
    dev = "cuda:0"
    g = torch.Generator(device=dev)
    g.manual_seed(N + k)
    K = torch.randn(B, Hkv, N, D, device=dev, generator=g).bfloat16()
    V = torch.randn(B, Hkv, N, D, device=dev, generator=g).bfloat16()
    logits = torch.randn(B, Hkv, N, G, device=dev, generator=g)
    c = stc.RoutedCache(B, Hq, Hkv, D, N, G, k, device=dev)
    c.build(K, V, logits=logits, fixed_k=3)
    ws = torch.full((stc.stc_workspace_bytes(c.shape, stc.STC_WS_STEP, k),), 0xA5,
                    dtype=torch.uint8, device=dev)
    for trial in range(2):
        q = torch.randn(B, Hq, D, device=dev, generator=g).bfloat16()
        c.step(q, one_call=False)
        idx = torch.full_like(c.page_idx, -3)
        out = torch.full_like(c.out, float("nan"))
        stc.stc_decode_step(c.shape, q, c.bounds, c.K, c.vpacked, c.mask, c.tok_off, k, idx, out, ws)
        torch.cuda.synchronize()
        assert torch.equal(idx, c.page_idx)
        assert torch.equal(out, c.out)
    # the list against the oracle on one stream (the two-call path is checked everywhere else)
    b, h = B - 1, Hkv - 1
    sc = O.page_scores(W.bf16_bits(q[b, h * R:(h + 1) * R]), O.page_bounds(W.bf16_bits(K[b, h])))
    assert np.array_equal(idx[b, h].cpu().numpy(), O.select_pages(sc, k))


def test_many_streams_of_2048_pages_select_in_the_scoring_workgroup():
    """192 streams of exactly 2048 pages (the most a scoring workgroup orders by itself) and of
    2049 (one more: separate launches): lists against the oracle on sampled streams, and the
    scores bit for bit."""
    dev = "cuda:0"
    for N in (32768, 32769):
        B, Hq, Hkv, D, G, k = 48, 8, 4, 64, 2, 100
        g = torch.Generator(device=dev)
        g.manual_seed(N)
        K = torch.randn(B, Hkv, N, D, device=dev, generator=g).bfloat16()
        q = torch.randn(B, Hq, D, device=dev, generator=g).bfloat16()
        shape = stc.make_shape(B, Hq, Hkv, D, N, G, N * G)
        bounds = torch.empty(stc.stc_bounds_bytes(shape) // 2, dtype=torch.bfloat16, device=dev)
        stc.stc_build_page_bounds(shape, K, bounds)
        NP = (N + 15) // 16
        idx = torch.full((B, Hkv, k), -1, dtype=torch.int32, device=dev)
        score = torch.full((B, Hkv, NP), float("nan"), dtype=torch.float32, device=dev)
        stc.stc_select_pages(shape, q, bounds, k, idx, score, None)
        idx2 = torch.full_like(idx, -1)
        ws = torch.empty(stc.stc_workspace_bytes(shape, stc.STC_WS_SELECT, k), dtype=torch.uint8,
                         device=dev)
        stc.stc_select_pages(shape, q, bounds, k, idx2, None, ws)      # scores in the workspace
        torch.cuda.synchronize()
        assert torch.equal(idx, idx2)
        for (b, h) in ((0, 0), (47, 3), (20, 1)):
            sc = O.page_scores(W.bf16_bits(q[b, 2 * h:2 * h + 2]), O.page_bounds(W.bf16_bits(K[b, h])))
            assert np.array_equal(score[b, h].cpu().numpy().view(np.uint32), sc.view(np.uint32))
            assert np.array_equal(idx[b, h].cpu().numpy(), O.select_pages(sc, k))


def test_parity_very_long_stream():
    """More than 8192 pages per stream (the selection kernel that re-reads its keys from
    memory) and an attention over 300 pages split over many workgroups."""
    B, Hq, Hkv, D, N, G, k = 1, 2, 1, 64, 16 * 9000 + 7, 2, 300
    K, V, q, logits, kcount = _rand_case(17, B, Hq, Hkv, D, N, G, outliers=True)
    hip = PT.run_hip(K, V, q, G, k, logits=logits, kcount=kcount)
    ora = PT.run_oracle(K, V, q, G, k, logits=logits, kcount=kcount)
    assert hip["dev_status"] == 0
    assert PT.compare(hip, ora, Hq, Hkv) <= PT.TIGHT


def test_parity_mask_mode_fixed_k_and_all_pages():
    B, Hq, Hkv, D, N, G = 2, 8, 2, 128, 333, 8
    K, V, q, logits, _ = _rand_case(3, B, Hq, Hkv, D, N, G)
    rng = np.random.default_rng(4)
    mask_in = rng.integers(0, 1 << 16, size=(B, Hkv, N)).astype(np.uint16)   # junk above bit G
    NP = (N + 15) // 16
    for k in (NP, NP + 5):                                  # k >= NP: every page, no scoring
        hip = PT.run_hip(K, V, q, G, k, mask_in=mask_in)
        ora = PT.run_oracle(K, V, q, G, k, mask_in=mask_in)
        assert PT.compare(hip, ora, Hq, Hkv) <= PT.TIGHT
        assert np.all(np.isnan(hip["page_score"]))          # scores are not written
    for fk in (0, 3, G):
        hip = PT.run_hip(K, V, q, G, 7, logits=logits, kcount=fk)
        ora = PT.run_oracle(K, V, q, G, 7, logits=logits, kcount=fk)
        assert PT.compare(hip, ora, Hq, Hkv) <= PT.TIGHT
        if fk == 0:
            assert np.all(hip["out"] == 0.0)
        if fk == G:                                          # full budget: packed == V
            assert np.array_equal(hip["vpacked"].reshape(B, Hkv, N, D), V)


def test_selection_ties_and_signed_zero():
    """Scores with many exact ties (small-integer keys) and all-zero scores."""
    rng = np.random.default_rng(5)
    B, Hq, Hkv, D, N, G = 2, 4, 2, 64, 1600, 4
    page_key = ints_bf16(rng, (B, Hkv, N // 16, D), -1, 1)
    K = np.repeat(page_key, 16, axis=2)                      # constant pages: min == max
    V = randn_bf16(rng, (B, Hkv, N, D))
    q = ints_bf16(rng, (B, Hq, D), -1, 1)
    mask_in = rng.integers(0, 1 << G, size=(B, Hkv, N)).astype(np.uint16)
    hip = PT.run_hip(K, V, q, G, 23, mask_in=mask_in)
    ora = PT.run_oracle(K, V, q, G, 23, mask_in=mask_in)
    PT.compare(hip, ora, Hq, Hkv)
    sc = hip["page_score"]
    assert len(np.unique(sc[0, 0])) < 40                     # really tied
    q0 = np.full((B, Hq, D), 0x8000, dtype=np.uint16)        # q = -0: all scores +0
    hip = PT.run_hip(K, V, q0, G, 9, mask_in=mask_in)
    assert np.array_equal(hip["page_score"].view(np.uint32), np.zeros_like(sc, dtype=np.uint32))
    assert np.array_equal(hip["page_idx"], np.broadcast_to(np.arange(9, dtype=np.int32), (B, Hkv, 9)))


@pytest.mark.parametrize("Hq,Hkv,D", [(3, 1, 128), (5, 1, 64), (12, 2, 128), (6, 1, 64), (9, 1, 64),
                                      (16, 1, 128)])
def test_scores_for_every_head_group_size(Hq, Hkv, D):
    """Page scores bit for bit for group sizes served by the matrix-core kernel (1..8 heads
    per KV head) and by the general one (9..16); N leaves a ragged last page and tile."""
    B, N, G = 2, 16 * 37 + 5, 4
    K, V, q, logits, kcount = _rand_case(40 + Hq, B, Hq, Hkv, D, N, G, outliers=True)
    hip = PT.run_hip(K, V, q, G, 9, logits=logits, kcount=kcount)
    R = Hq // Hkv
    for b in range(B):
        for h in range(Hkv):
            bounds = O.page_bounds(K[b, h])
            assert np.array_equal(hip["bounds"][b, h], bounds)
            want = O.page_scores(q[b, h * R:(h + 1) * R], bounds)
            assert np.array_equal(hip["page_score"][b, h].view(np.uint32), want.view(np.uint32))
            assert np.array_equal(hip["page_idx"][b, h], O.select_pages(want, 9))
    # pages past the last one in the last tile of every stream are zero-filled
    NP, nt = (N + 15) // 16, ((N + 15) // 16 + 7) // 8
    raw = hip["bounds_raw"].reshape(B * Hkv, nt, D // 32, 2, 8, 4, 4, 2)
    last = raw[:, nt - 1]                                # [s][j][g][e][col][w][2]
    for pt in range(NP - 8 * (nt - 1), 8):
        assert not last[:, :, pt // 4, :, pt % 4].any()


@pytest.mark.parametrize("N,G,D,gk", [(1000, 8, 128, 3), (2500, 4, 64, 1), (777, 16, 128, 5),
                                      (4096, 8, 128, 0), (300, 4, 64, 4), (1024, 1, 64, 1),
                                      (999, 2, 64, 1), (333, 1, 64, 1),   # N*G not a multiple of 4
                                      (40000, 8, 128, 5)])                # several histogram slices
def test_global_budget_routing(N, G, D, gk):
    """Global token-group budget: masks (tokens with no group included), offsets and packed
    values bit for bit; exactly N*K groups kept; attention over the result within the bar."""
    B, Hq, Hkv = 2, 4, 2
    K, V, q, logits, _ = _rand_case(60 + N % 7, B, Hq, Hkv, D, N, G)
    hip = PT.run_hip(K, V, q, G, 12, logits=logits, global_k=gk)
    ora = PT.run_oracle(K, V, q, G, 12, logits=logits, global_k=gk)
    assert hip["dev_status"] == 0
    assert (hip["tok_off"][:, :, -1] == N * gk).all()
    err = PT.compare(hip, ora, Hq, Hkv)
    assert err < PT.TIGHT
    if 0 < gk < G and G > 1:
        kept = O.popcount(hip["mask"], G)
        assert kept.min() == 0 or kept.max() > gk          # allocation is not uniform


def test_global_budget_routing_with_ties_everywhere():
    """Logits drawn from five values (with -0 and +0): the cut falls inside a run of equal
    logits spanning many tokens and several 1024-token tiles."""
    rng = np.random.default_rng(71)
    B, Hq, Hkv, D, N, G = 1, 2, 2, 64, 3000, 4
    K, V, q, _, _ = _rand_case(72, B, Hq, Hkv, D, N, G)
    logits = rng.choice(np.array([-1.5, -0.0, 0.0, 0.25, 2.0], dtype=np.float32),
                        size=(B, Hkv, N, G))
    for gk in (1, 2, 3):
        hip = PT.run_hip(K, V, q, G, 10, logits=logits, global_k=gk)
        ora = PT.run_oracle(K, V, q, G, 10, logits=logits, global_k=gk)
        PT.compare(hip, ora, Hq, Hkv)
        assert (hip["tok_off"][:, :, -1] == N * gk).all()


@pytest.mark.parametrize("B,Hq,Hkv,D,N,G,k,ntail", [
    (1, 4, 1, 128, 700, 8, 9, 1), (2, 14, 2, 128, 1500, 8, 20, 37), (1, 8, 8, 64, 333, 4, 21, 16),
    (2, 2, 2, 64, 100, 4, 3, 15), (1, 16, 1, 128, 2048, 16, 128, 64), (1, 3, 1, 64, 64, 2, 4, 17)])
def test_attention_with_uncompressed_tail(B, Hq, Hkv, D, N, G, k, ntail):
    """Selected pages of the compressed cache plus an always-attended dense tail of recent
    tokens (ragged last tail page included), against the oracle; an empty tail gives the bits
    of the plain entry point."""
    K, V, q, logits, kcount = _rand_case(80 + ntail, B, Hq, Hkv, D, N, G)
    rng = np.random.default_rng(81 + ntail)
    cap_t = ntail + 5
    Kt, Vt = randn_bf16(rng, (B, Hkv, cap_t, D)), randn_bf16(rng, (B, Hkv, cap_t, D))
    hip = PT.run_hip(K, V, q, G, k, logits=logits, kcount=kcount)
    c = hip["cache"]
    shp = c.shape
    dq, dKt, dVt = PT.to_dev_bf16(q), PT.to_dev_bf16(Kt), PT.to_dev_bf16(Vt)
    slots = c.k_eff + (ntail + 15) // 16
    ws = torch.zeros(max(16, stc.stc_workspace_bytes(shp, stc.STC_WS_ATTENTION_TAIL, slots)),
                     dtype=torch.uint8, device="cuda:0")
    out = torch.full_like(c.out, float("nan"))
    stc.stc_decode_attention_tail(shp, dq, c.K, c.vpacked, c.mask, c.tok_off, c.page_idx, c.k_eff,
                                  dKt, dVt, ntail, cap_t, out, ws)
    out0 = torch.full_like(c.out, float("nan"))
    stc.stc_decode_attention_tail(shp, dq, c.K, c.vpacked, c.mask, c.tok_off, c.page_idx, c.k_eff,
                                  None, None, 0, 0, out0, ws)
    # selection + attention with the tail in one call: the bits of the two calls
    ws1 = torch.full((max(16, stc.stc_workspace_bytes(shp, stc.STC_WS_STEP_TAIL, slots)),), 0x5A,
                     dtype=torch.uint8, device="cuda:0")
    out1, idx1 = torch.full_like(c.out, float("nan")), torch.full_like(c.page_idx, -9)
    stc.stc_decode_step_tail(shp, dq, c.bounds, c.K, c.vpacked, c.mask, c.tok_off, c.k_eff, dKt, dVt,
                             ntail, cap_t, idx1, out1, ws1)
    torch.cuda.synchronize()
    assert torch.equal(idx1, c.page_idx) and torch.equal(out1, out)
    assert np.array_equal(out0.cpu().numpy(), hip["out"])
    got = out.cpu().numpy()
    R = Hq // Hkv
    worst = 0.0
    for b in range(B):
        for h in range(Hkv):
            want = O.decode_attention(q[b, h * R:(h + 1) * R], K[b, h], V[b, h], hip["mask"][b, h],
                                      hip["page_idx"][b, h], G, K_tail=Kt[b, h, :ntail],
                                      V_tail=Vt[b, h, :ntail])
            worst = max(worst, float(np.abs(got[b, h * R:(h + 1) * R] - want).max()))
    assert worst < PT.TIGHT


def test_append_then_attend_step_by_step():
    """Twenty decode steps: each appends the new token's key and value to the tail and attends
    cache + tail; checked against the oracle at every step (tail lengths 1..20, crossing a page)."""
    B, Hq, Hkv, D, N, G, k, steps = 2, 8, 2, 128, 600, 8, 10, 20
    K, V, q, logits, kcount = _rand_case(90, B, Hq, Hkv, D, N, G)
    rng = np.random.default_rng(91)
    c = stc.RoutedCache(B, Hq, Hkv, D, N, G, k, device="cuda:0", tail_cap=24)
    c.K_tail.view(torch.int16).fill_(0x7FC0)               # NaN: rows not yet appended
    c.V_tail.view(torch.int16).fill_(0x7FC0)
    c.build(PT.to_dev_bf16(K), PT.to_dev_bf16(V), logits=torch.from_numpy(logits).cuda(),
            kcount=torch.from_numpy(kcount).cuda())
    mask = O.route_and_pack_all(V, G, logits=logits, kcount=kcount)[0]
    new_k, new_v = randn_bf16(rng, (steps, B, Hkv, D)), randn_bf16(rng, (steps, B, Hkv, D))
    R = Hq // Hkv
    for s_ in range(steps):
        qs = randn_bf16(rng, (B, Hq, D))
        c.append(PT.to_dev_bf16(new_k[s_]), PT.to_dev_bf16(new_v[s_]))
        c.step(PT.to_dev_bf16(qs), one_call=False)
        torch.cuda.synchronize()
        two = (c.page_idx.clone(), c.out.clone())
        c.page_idx.fill_(-5)
        c.out.fill_(float("nan"))
        c.step(PT.to_dev_bf16(qs))
        torch.cuda.synchronize()
        assert torch.equal(two[0], c.page_idx) and torch.equal(two[1], c.out)
        assert c.n_tail == s_ + 1
        got, idx = c.out.cpu().numpy(), c.page_idx.cpu().numpy()
        for (b, h) in ((0, 0), (1, 1)):
            sc = O.page_scores(qs[b, h * R:(h + 1) * R], O.page_bounds(K[b, h]))
            assert np.array_equal(idx[b, h], O.select_pages(sc, k))
            want = O.decode_attention(qs[b, h * R:(h + 1) * R], K[b, h], V[b, h], mask[b, h],
                                      idx[b, h], G, K_tail=new_k[:s_ + 1, b, h],
                                      V_tail=new_v[:s_ + 1, b, h])
            assert np.abs(got[b, h * R:(h + 1) * R] - want).max() < PT.TIGHT
    assert np.array_equal(PT.host_bf16(c.K_tail)[:, :, :steps], new_k.transpose(1, 2, 0, 3))
    assert np.array_equal(PT.host_bf16(c.V_tail)[:, :, :steps], new_v.transpose(1, 2, 0, 3))


@pytest.mark.parametrize("B,Hq,Hkv,D,N,G,k", [
    (2, 14, 2, 128, 3000, 8, 20), (1, 8, 2, 64, 1000, 4, 9), (2, 4, 4, 128, 700, 8, 5),
    (1, 12, 1, 128, 2048, 8, 100), (1, 16, 1, 64, 500, 2, 30), (1, 10, 2, 128, 1100, 8, 12),
    (2, 12, 2, 128, 333, 8, 7)])
def test_per_head_selection_and_attention(B, Hq, Hkv, D, N, G, k):
    """Every query head selects and attends its own pages: scores and indices bit for bit per
    head, output within the bar; for MHA the calls equal the shared ones bit for bit."""
    K, V, q, logits, kcount = _rand_case(100 + Hq, B, Hq, Hkv, D, N, G, outliers=True)
    hip = PT.run_hip(K, V, q, G, k, logits=logits, kcount=kcount)
    c = hip["cache"]
    NP = (N + 15) // 16
    dq = PT.to_dev_bf16(q)
    dev = "cuda:0"
    idx = torch.full((B, Hq, k), -9, dtype=torch.int32, device=dev)
    score = torch.full((B, Hq, NP), float("nan"), dtype=torch.float32, device=dev)
    ws_s = torch.empty(max(16, stc.stc_workspace_bytes(c.shape, stc.STC_WS_SELECT_PER_HEAD, k)),
                       dtype=torch.uint8, device=dev)
    ws_a = torch.empty(max(16, stc.stc_workspace_bytes(c.shape, stc.STC_WS_ATTENTION_PER_HEAD, k)),
                       dtype=torch.uint8, device=dev)
    out = torch.full((B, Hq, D), float("nan"), dtype=torch.float32, device=dev)
    stc.stc_select_pages_per_head(c.shape, dq, c.bounds, k, idx, score, ws_s)
    stc.stc_decode_attention_per_head(c.shape, dq, c.K, c.vpacked, c.mask, c.tok_off, idx, k, out,
                                      ws_a)
    idx2 = torch.full_like(idx, -9)
    stc.stc_select_pages_per_head(c.shape, dq, c.bounds, k, idx2, None, ws_s)  # scores in ws
    torch.cuda.synchronize()
    assert torch.equal(idx, idx2)
    bounds = O.build_page_bounds_all(K)
    want_idx, want_score = O.select_pages_per_head_all(q, bounds, k)
    assert np.array_equal(score.cpu().numpy().view(np.uint32), want_score.view(np.uint32))
    assert np.array_equal(idx.cpu().numpy(), want_idx)
    want = O.decode_attention_per_head_all(q, K, V, hip["mask"], want_idx, G)
    assert np.abs(out.cpu().numpy() - want).max() < PT.TIGHT
    if Hq == Hkv:
        assert np.array_equal(idx.cpu().numpy(), hip["page_idx"])
        assert np.array_equal(out.cpu().numpy(), hip["out"])
    else:
        assert not np.array_equal(want_idx[:, 0], want_idx[:, 1])   # heads really differ
    # the same attention with the group's lists merged: every K page and V run read once
    R = Hq // Hkv
    U = min(NP, R * k)
    uidx = torch.full((B, Hkv, U), -5, dtype=torch.int32, device=dev)
    uheads = torch.full((B, Hkv, U), -1, dtype=torch.int16, device=dev)
    stc.stc_union_pages(c.shape, idx, k, uidx, uheads)
    ws_u = torch.empty(max(16, stc.stc_workspace_bytes(c.shape, stc.STC_WS_ATTENTION, U)),
                       dtype=torch.uint8, device=dev)
    out_u = torch.full_like(out, float("nan"))
    stc.stc_decode_attention_union(c.shape, dq, c.K, c.vpacked, c.mask, c.tok_off, uidx, uheads,
                                   out_u, ws_u)
    torch.cuda.synchronize()
    gi, gh = uidx.cpu().numpy(), PT.host_u16(uheads)
    for b in range(B):
        for h in range(Hkv):
            pages, heads = O.union_pages(want_idx[b, h * R:(h + 1) * R], NP)
            n = len(pages)
            assert np.array_equal(gi[b, h, :n], pages) and np.array_equal(gh[b, h, :n], heads)
            assert (gi[b, h, n:] == -1).all() and (gh[b, h, n:] == 0).all()
    assert np.abs(out_u.cpu().numpy() - want).max() < PT.TIGHT


@pytest.mark.parametrize("B,Hkv,R,NP,k", [(2, 1, 7, 9003, 300),      # three tiles of head sets
                                          (1, 2, 16, 5000, 1000),    # 62.5 KiB of lists in LDS
                                          (1, 1, 3, 4096, 4096)])    # every page, one full tile
def test_union_pages_long_streams_and_long_lists(B, Hkv, R, NP, k):
    """stc_union_pages on given lists (ascending, distinct per head): several tiles of pages,
    lists near the size limit, and an output that is the whole range of pages."""
    rng = np.random.default_rng(NP + k)
    lists = np.stack([np.sort(rng.choice(NP, size=k, replace=False)) for _ in range(B * Hkv * R)])
    lists = lists.reshape(B, Hkv * R, k).astype(np.int32)
    shape = stc.make_shape(B, Hkv * R, Hkv, 128, NP * 16, 8, NP * 16 * 8)
    U = min(NP, R * k)
    dev = "cuda:0"
    uidx = torch.full((B, Hkv, U), -5, dtype=torch.int32, device=dev)
    uheads = torch.full((B, Hkv, U), -1, dtype=torch.int16, device=dev)
    stc.stc_union_pages(shape, torch.from_numpy(lists).to(dev), k, uidx, uheads)
    torch.cuda.synchronize()
    gi, gh = uidx.cpu().numpy(), PT.host_u16(uheads)
    for b in range(B):
        for h in range(Hkv):
            pages, heads = O.union_pages(lists[b, h * R:(h + 1) * R], NP)
            n = len(pages)
            assert np.array_equal(gi[b, h, :n], pages) and np.array_equal(gh[b, h, :n], heads)
            assert (gi[b, h, n:] == -1).all() and (gh[b, h, n:] == 0).all()


@pytest.mark.parametrize("B,Hkv,N,dm,G,with_bias", [(2, 2, 301, 512, 8, True), (1, 3, 64, 128, 4, False),
                                                     (1, 1, 1000, 3584, 8, True),
                                                     (2, 1, 77, 256, 16, False), (1, 2, 50, 384, 1, True),
                                                     (1, 1, 130, 256, 2, True)])
def test_router_logits_bits_and_routing(B, Hkv, N, dm, G, with_bias):
    """The router's projection bit for bit (the order of its float additions is part of the
    definition), replicated over the KV heads; masks routed from it equal the oracle's."""
    rng = np.random.default_rng(110 + dm)
    h, Wr = randn_bf16(rng, (B, N, dm)), randn_bf16(rng, (G, dm))
    bias = rng.standard_normal(G).astype(np.float32) if with_bias else None
    dev = "cuda:0"
    logits = torch.full((B, Hkv, N, G), float("nan"), dtype=torch.float32, device=dev)
    stc.stc_router_logits(PT.to_dev_bf16(h), PT.to_dev_bf16(Wr),
                          None if bias is None else torch.from_numpy(bias).to(dev), logits, Hkv)
    torch.cuda.synchronize()
    got = logits.cpu().numpy()
    for b in range(B):
        want = O.router_logits(h[b], Wr, bias)
        for kvh in range(Hkv):
            assert np.array_equal(got[b, kvh].view(np.uint32), want.view(np.uint32))
    if G >= 4:                                      # logits -> global-budget masks, end to end
        D = 128
        K, V, q, _, _ = _rand_case(111, B, Hkv, Hkv, D, N, G)
        hip = PT.run_hip(K, V, q, G, 3, logits=got, global_k=2)
        for b in range(B):
            m = O.route_mask_global(O.router_logits(h[b], Wr, bias), 2 * N)
            for kvh in range(Hkv):
                assert np.array_equal(hip["mask"][b, kvh], m)


@pytest.mark.parametrize("B,Hkv,N,dm,G", [(3, 2, 203, 512, 8), (5, 1, 64, 128, 4), (2, 1, 130, 3584, 16)])
def test_router_logits_with_a_query_term_per_batch_element(B, Hkv, N, dm, G):
    """Query-conditioned router (Sec. 3.4; one linear map of the token state and the query
    summary, App. B.1): W_h h + (W_q s_Q + b).  The bracket comes from the same routine on the
    summaries (N = 1) and enters as one bias vector per batch element; both steps bit for bit."""
    rng = np.random.default_rng(120 + dm)
    h, sq = randn_bf16(rng, (B, N, dm)), randn_bf16(rng, (B, 1, dm))
    Wh, Wq = randn_bf16(rng, (G, dm)), randn_bf16(rng, (G, dm))
    b0 = rng.standard_normal(G).astype(np.float32)
    dev = "cuda:0"
    qterm = torch.full((B, 1, 1, G), float("nan"), dtype=torch.float32, device=dev)
    stc.stc_router_logits(PT.to_dev_bf16(sq), PT.to_dev_bf16(Wq), torch.from_numpy(b0).to(dev), qterm, 1)
    logits = torch.full((B, Hkv, N, G), float("nan"), dtype=torch.float32, device=dev)
    stc.stc_router_logits(PT.to_dev_bf16(h), PT.to_dev_bf16(Wh), qterm.view(B, G), logits, Hkv)
    torch.cuda.synchronize()
    got_q, got = qterm.cpu().numpy().reshape(B, G), logits.cpu().numpy()
    for b in range(B):
        want_q = O.router_logits(sq[b], Wq, b0)[0]
        assert np.array_equal(got_q[b].view(np.uint32), want_q.view(np.uint32))
        want = O.router_logits(h[b], Wh, want_q)
        for kvh in range(Hkv):
            assert np.array_equal(got[b, kvh].view(np.uint32), want.view(np.uint32))
    with pytest.raises(ValueError):
        stc.stc_router_logits(PT.to_dev_bf16(h), PT.to_dev_bf16(Wh), qterm.view(B * G, 1), logits, Hkv)


@pytest.mark.parametrize("mode", ["topk", "global", "mask"])
def test_routing_inputs_shared_by_the_kv_heads(mode):
    """One set of routing inputs per batch element (the paper's router gives one mask per token
    and layer), read by all KV heads: the cache equals the one built from replicated inputs and
    the oracle's; the router with Hkv = 1 writes the single copy."""
    rng = np.random.default_rng(500)
    B, Hq, Hkv, D, N, G, dm = 2, 8, 4, 128, 16 * 45 + 7, 8, 256
    K, V, q, _, _ = _rand_case(501, B, Hq, Hkv, D, N, G)
    h, Wr = randn_bf16(rng, (B, N, dm)), randn_bf16(rng, (G, dm))
    dev = "cuda:0"
    lg1 = torch.empty(B, 1, N, G, dtype=torch.float32, device=dev)
    stc.stc_router_logits(PT.to_dev_bf16(h), PT.to_dev_bf16(Wr), None, lg1, 1)
    torch.cuda.synchronize()
    logits1 = lg1.cpu().numpy()
    for b in range(B):
        assert np.array_equal(logits1[b, 0].view(np.uint32),
                              O.router_logits(h[b], Wr, None).view(np.uint32))
    kc1 = rng.integers(0, G + 1, size=(B, 1, N)).astype(np.uint8)
    m1 = rng.integers(0, 1 << G, size=(B, 1, N)).astype(np.uint16)
    kw = dict(topk=dict(logits=lg1, kcount=torch.from_numpy(kc1).to(dev)),
              mask=dict(mask_in=PT.to_dev_u16(m1)), **{"global": dict(logits=lg1, global_k=3)})[mode]
    c = stc.RoutedCache(B, Hq, Hkv, D, N, G, 9, device=dev)
    c.vpacked.view(torch.int16).fill_(0x7FC0)
    c.build(PT.to_dev_bf16(K), PT.to_dev_bf16(V), shared=True, **kw)
    c.step(PT.to_dev_bf16(q))
    torch.cuda.synchronize()
    assert int(c.dev_status.item()) == 0
    mask, off, vp = PT.host_u16(c.mask), c.tok_off.cpu().numpy().view(np.uint32), PT.host_bf16(c.vpacked)
    R = Hq // Hkv
    for b in range(B):
        if mode == "topk":
            m = O.route_mask(logits1[b, 0], kc1[b, 0])
        elif mode == "global":
            m = O.route_mask_global(logits1[b, 0], 3 * N)
        else:
            m = m1[b, 0] & np.uint16((1 << G) - 1)
        o = O.token_offsets(m, G)
        for hh in range(Hkv):
            assert np.array_equal(mask[b, hh], m) and np.array_equal(off[b, hh], o)
            assert np.array_equal(vp[b, hh, :int(o[-1])], O.pack_values(V[b, hh], m, o, G))
            qh = q[b, hh * R:(hh + 1) * R]
            idx = O.select_pages(O.page_scores(qh, O.page_bounds(K[b, hh])), 9)
            want = O.decode_attention(qh, K[b, hh], V[b, hh], m, idx, G)
            assert np.abs(c.out[b, hh * R:(hh + 1) * R].cpu().numpy() - want).max() < PT.TIGHT


def _plant_subnormals(rng, bits, frac=0.12):
    """bf16 bit patterns with a share of entries replaced by subnormal patterns of either sign."""
    out = bits.copy()
    hit = rng.random(bits.shape) < frac
    mant = rng.integers(1, 128, size=bits.shape).astype(np.uint16)
    sign = rng.integers(0, 2, size=bits.shape).astype(np.uint16) << np.uint16(15)
    out[hit] = (sign | mant)[hit]
    return out


@pytest.mark.parametrize("R,D,scale", [(7, 128, 1.0), (4, 64, 1.0), (9, 128, 1.0), (7, 128, 2.0 ** 90),
                                       (2, 128, 2.0 ** -70)])
def test_subnormal_inputs_count_as_zero_in_page_scores(R, D, scale):
    """Keys and queries that are subnormal as bf16 are zeros for the page scores (bounds keep
    their bit patterns): matrix-core kernel and the one-head-at-a-time kernel against the
    oracle, bit for bit.  With large queries the products of subnormal inputs would be ordinary
    floats, so a kernel that multiplied them would differ in many bits; with tiny queries the
    products of normal inputs lie in the subnormal float range and must come out exact."""
    rng = np.random.default_rng(400 + R + D)
    B, Hkv, N, G = 2, 2, 16 * 37 + 5, 8
    Hq = Hkv * R
    K = _plant_subnormals(rng, randn_bf16(rng, (B, Hkv, N, D), 1.0 if scale >= 1 else scale))
    q = _plant_subnormals(rng, randn_bf16(rng, (B, Hq, D), scale))
    V = randn_bf16(rng, (B, Hkv, N, D))
    dev = "cuda:0"
    c = stc.RoutedCache(B, Hq, Hkv, D, N, G, 5, device=dev)
    c.build(PT.to_dev_bf16(K), PT.to_dev_bf16(V), mask_in=PT.to_dev_u16(
        np.full((B, Hkv, N), 0xFF, dtype=np.uint16)))
    sc = torch.full((B, Hkv, c.NP), float("nan"), dtype=torch.float32, device=dev)
    c.score(PT.to_dev_bf16(q), sc)
    c.select(PT.to_dev_bf16(q))
    torch.cuda.synchronize()
    got, rows, idx = sc.cpu().numpy(), PT.host_bf16(c.bounds_rows()), c.page_idx.cpu().numpy()
    for b in range(B):
        for h in range(Hkv):
            bounds = O.page_bounds(K[b, h])
            assert np.array_equal(rows[b, h], bounds)          # subnormal patterns survive
            want = O.page_scores(q[b, h * R:(h + 1) * R], bounds)
            assert np.array_equal(got[b, h].view(np.uint32), want.view(np.uint32)), (b, h)
            assert np.array_equal(idx[b, h], O.select_pages(want, 5))


def test_subnormal_inputs_count_as_zero_in_router_logits():
    rng = np.random.default_rng(410)
    B, Hkv, N, dm, G = 2, 2, 300, 512, 8
    h = _plant_subnormals(rng, randn_bf16(rng, (B, N, dm), 2.0 ** 80))
    Wr = _plant_subnormals(rng, randn_bf16(rng, (G, dm)))
    dev = "cuda:0"
    logits = torch.full((B, Hkv, N, G), float("nan"), dtype=torch.float32, device=dev)
    stc.stc_router_logits(PT.to_dev_bf16(h), PT.to_dev_bf16(Wr), None, logits, Hkv)
    torch.cuda.synchronize()
    got = logits.cpu().numpy()
    for b in range(B):
        want = O.router_logits(h[b], Wr, None)
        assert np.array_equal(got[b, 1].view(np.uint32), want.view(np.uint32))


def _cache_equals_full_build(c, K_all, V_all, logits_all, kcount_all, G):
    """Every array of cache `c` (N tokens so far, capacity strides) against construction from
    scratch over the same N tokens by the oracle."""
    N = c.N
    bounds = PT.host_bf16(c.bounds_rows())
    mask = PT.host_u16(c.mask)[:, :, :N]
    off = c.tok_off.cpu().numpy().view(np.uint32)[:, :, :N + 1]
    vp = PT.host_bf16(c.vpacked)
    B, Hkv = K_all.shape[:2]
    for b in range(B):
        for h in range(Hkv):
            assert np.array_equal(bounds[b, h], O.page_bounds(K_all[b, h, :N]))
            m = O.route_mask(logits_all[b, h, :N], kcount_all[b, h, :N])
            o = O.token_offsets(m, G)
            assert np.array_equal(mask[b, h], m) and np.array_equal(off[b, h], o)
            assert np.array_equal(vp[b, h, :int(o[-1])], O.pack_values(V_all[b, h, :N], m, o, G))
    assert np.array_equal(PT.host_bf16(c.K)[:, :, :N], K_all[:, :, :N])


@pytest.mark.parametrize("D,G,Hq,Hkv,N0", [(128, 8, 14, 2, 600), (64, 4, 4, 4, 33), (128, 16, 3, 1, 1024)])
def test_flush_tail_into_the_cache_equals_full_build(D, G, Hq, Hkv, N0):
    """A decode loop with cache growth: append new tokens to the tail, attend, and from time to
    time move the oldest tail tokens into the compressed cache in place.  After every flush
    the cache equals construction from scratch over all its tokens, bit for bit; every decode
    step is checked against the oracle."""
    B, k, n_cap, tail_cap = 2, 12, N0 + 160, 48
    total = N0 + 150
    K_all, V_all, _, logits_all, kcount_all = _rand_case(120 + D + N0, B, Hq, Hkv, D, total, G,
                                                         outliers=True)
    rng = np.random.default_rng(121)
    dev = "cuda:0"
    c = stc.RoutedCache(B, Hq, Hkv, D, N0, G, k, device=dev, tail_cap=tail_cap, n_cap=n_cap)
    c.vpacked.view(torch.int16).fill_(0x7FC0)
    c.build(PT.to_dev_bf16(K_all[:, :, :N0]), PT.to_dev_bf16(V_all[:, :, :N0]),
            logits=torch.from_numpy(logits_all[:, :, :N0].copy()).to(dev),
            kcount=torch.from_numpy(kcount_all[:, :, :N0].copy()).to(dev))
    torch.cuda.synchronize()
    _cache_equals_full_build(c, K_all, V_all, logits_all, kcount_all, G)      # capacity strides
    R = Hq // Hkv
    seen = N0                      # tokens handed to the cache or its tail so far
    for step in range(150):
        c.append(PT.to_dev_bf16(K_all[:, :, seen]), PT.to_dev_bf16(V_all[:, :, seen]))
        seen += 1
        if c.n_tail == tail_cap or step in (6, 20):          # flush all but the newest few
            n = max(1, c.n_tail - int(rng.integers(0, 9)))
            lo = c.N
            c.flush(n, logits=torch.from_numpy(logits_all[:, :, lo:lo + n].copy()).to(dev),
                    kcount=torch.from_numpy(kcount_all[:, :, lo:lo + n].copy()).to(dev))
            torch.cuda.synchronize()
            assert int(c.dev_status.item()) == 0 and c.N == lo + n and c.N + c.n_tail == seen
            _cache_equals_full_build(c, K_all, V_all, logits_all, kcount_all, G)
        if step % 7 == 0 or c.n_tail == 0:
            qs = randn_bf16(rng, (B, Hq, D))
            c.step(PT.to_dev_bf16(qs))
            torch.cuda.synchronize()
            got, idx = c.out.cpu().numpy(), c.page_idx.cpu().numpy()
            b, h = step % B, step % Hkv
            Kc, Vc = K_all[b, h, :c.N], V_all[b, h, :c.N]
            m = O.route_mask(logits_all[b, h, :c.N], kcount_all[b, h, :c.N])
            sc = O.page_scores(qs[b, h * R:(h + 1) * R], O.page_bounds(Kc))
            want_idx = O.select_pages(sc, k)
            assert np.array_equal(idx[b, h], want_idx)
            want = O.decode_attention(qs[b, h * R:(h + 1) * R], Kc, Vc, m, want_idx, G,
                                      K_tail=K_all[b, h, c.N:seen], V_tail=V_all[b, h, c.N:seen])
            assert np.abs(got[b, h * R:(h + 1) * R] - want).max() < PT.TIGHT


def test_score_pages_alone_matches_oracle_bits():
    B, Hq, Hkv, D, N, G = 2, 14, 2, 128, 3000, 8
    K, V, q, logits, kcount = _rand_case(21, B, Hq, Hkv, D, N, G, outliers=True)
    hip = PT.run_hip(K, V, q, G, 20, logits=logits, kcount=kcount)
    c = hip["cache"]
    sc = torch.full_like(c.page_score, float("nan"))
    c.score(PT.to_dev_bf16(q), sc)
    torch.cuda.synchronize()
    got = sc.cpu().numpy()
    for b in range(B):
        for h in range(Hkv):
            want = O.page_scores(q[b, h * 7:(h + 1) * 7], O.page_bounds(K[b, h]))
            assert np.array_equal(got[b, h].view(np.uint32), want.view(np.uint32))
    assert np.array_equal(got.view(np.uint32), hip["page_score"].view(np.uint32))


def test_attention_closed_form_and_peaked():
    """q = 0 with integer values: weights are exactly 1/|T| (|T| = 128), so the
    output is an exact dyadic number; then a sharply peaked softmax."""
    rng = np.random.default_rng(6)
    B, Hq, Hkv, D, N, G = 1, 2, 1, 128, 512, 8
    gd = D // G
    K = randn_bf16(rng, (B, Hkv, N, D))
    Vi = rng.integers(-8, 9, size=(B, Hkv, N, D))
    V = f32_to_bf16_bits(Vi.astype(np.float32))
    mask_in = rng.integers(0, 1 << G, size=(B, Hkv, N)).astype(np.uint16)
    q0 = np.zeros((B, Hq, D), dtype=np.uint16)
    hip = PT.run_hip(K, V, q0, G, 8, mask_in=mask_in)
    assert list(hip["page_idx"][0, 0]) == list(range(8))
    keep = np.repeat((mask_in[0, 0, :128, None] >> np.arange(G)) & 1, gd, axis=1)
    want = (Vi[0, 0, :128] * keep).sum(axis=0) / 128.0
    assert np.abs(hip["out"][0, 0] - want).max() <= 1e-6
    # peaked: values encode (token, channel); a misplaced group or token is far off
    Vp = f32_to_bf16_bits(((np.arange(N)[:, None] % 64) + (np.arange(D)[None, :] % 32)).astype(
        np.float32))[None, None]
    qs = randn_bf16(rng, (B, Hq, D), 8.0)
    hip = PT.run_hip(K, Vp, qs, G, 8, mask_in=mask_in)
    ora = PT.run_oracle(K, Vp, qs, G, 8, mask_in=mask_in)
    assert PT.compare(hip, ora, Hq, Hkv) <= PT.TIGHT


def test_packed_store_overflow_is_flagged_not_written():
    B, Hq, Hkv, D, N, G = 1, 2, 2, 64, 600, 4
    K, V, q, logits, kcount = _rand_case(7, B, Hq, Hkv, D, N, G)
    kcount[:] = 3
    cap = 1000                                              # needs 1800 groups per stream
    hip = PT.run_hip(K, V, q, G, 4, logits=logits, kcount=kcount, cap=cap)
    assert hip["dev_status"] == 1
    for (b, h), o in PT.run_oracle(K, V, q, G, 4, logits=logits, kcount=kcount).items():
        assert np.array_equal(hip["mask"][b, h], o["mask"])
        assert np.array_equal(hip["tok_off"][b, h], o["tok_off"])
        assert np.array_equal(hip["vpacked"][b, h], o["vpacked"][:cap])
    assert np.all(np.isfinite(hip["out"]))


def test_attention_skips_invalid_page_entries_and_any_order():
    B, Hq, Hkv, D, N, G = 1, 7, 1, 128, 800, 8
    K, V, q, logits, kcount = _rand_case(8, B, Hq, Hkv, D, N, G)
    hip = PT.run_hip(K, V, q, G, 6, logits=logits, kcount=kcount)
    c = hip["cache"]
    listed = np.array([[[49, -1, 3, 50, 12, 7]]], dtype=np.int32)      # NP = 50: 50 and -1 skipped
    c.page_idx.copy_(torch.from_numpy(listed))
    c.attend(PT.to_dev_bf16(q))
    torch.cuda.synchronize()
    m = hip["mask"][0, 0]
    want = O.decode_attention(q[0], K[0, 0], V[0, 0], m, np.array([49, 3, 12, 7]), G)
    assert np.abs(c.out.cpu().numpy()[0] - want).max() <= PT.TIGHT


def test_compact_tokens():
    rng = np.random.default_rng(9)
    B, Hkv, Ns, D, nk = 2, 3, 40, 128, 11
    src = randn_bf16(rng, (B, Hkv, Ns, D))
    idx = np.sort(rng.choice(Ns, size=(B, nk)), axis=1).astype(np.int32)
    idx[1, 4] = Ns + 3                                       # out of range: zero row + flag
    d_src, d_idx = PT.to_dev_bf16(src), torch.from_numpy(idx).cuda()
    dst = torch.empty(B, Hkv, nk, D, dtype=torch.bfloat16, device="cuda")
    st = torch.zeros(1, dtype=torch.int32, device="cuda")
    stc.stc_compact_tokens(d_src, d_idx, dst, B, Hkv, Ns, nk, D, st)
    got = PT.host_bf16(dst)
    for b in range(B):
        for i in range(nk):
            want = src[b, :, idx[b, i]] if idx[b, i] < Ns else np.zeros((Hkv, D), np.uint16)
            assert np.array_equal(got[b, :, i], want)
    assert int(st.item()) == 1


# --------------------------------------------------------------------------- #
# The five workloads: reduced sizes element by element, full sizes on sampled streams
# --------------------------------------------------------------------------- #
def _run_workload(w, dev="cuda:0", layer=0, qscale=1.0):
    inp = W.make_cache_inputs(w, dev, layer)
    K, V = inp["K"], inp["V"]
    if w.routing == "vlm":                                  # token-level compaction first
        n_src = w.n_visual + w.n_text
        Kc = torch.empty(w.B, w.Hkv, w.N, w.D, dtype=torch.bfloat16, device=dev)
        Vc = torch.empty_like(Kc)
        stc.stc_compact_tokens(K, inp["token_idx"], Kc, w.B, w.Hkv, n_src, w.N, w.D)
        stc.stc_compact_tokens(V, inp["token_idx"], Vc, w.B, w.Hkv, n_src, w.N, w.D)
        ti = inp["token_idx"].long()
        gather = ti[:, None, :, None].expand(w.B, w.Hkv, w.N, w.D)
        assert torch.equal(Kc, torch.gather(K, 2, gather))
        K, V = Kc, Vc
    logits = inp["logits"]              # drawn per retained token: [B, Hkv, N, G]
    c = stc.RoutedCache(w.B, w.Hq, w.Hkv, w.D, w.N, w.G, w.k_pages, device=dev)
    c.build(K, V, logits=logits, kcount=inp["kcount"], mask_in=inp["mask_in"])
    q = W.make_query(w, 0, dev, layer, qscale)
    c.step(q)
    torch.cuda.synchronize()
    return c, dict(K=K, V=V, q=q, logits=logits, kcount=inp["kcount"], mask_in=inp["mask_in"])


def _check_streams(w, c, t, streams):
    """Oracle on the listed streams from the device tensors' bytes."""
    worst = 0.0
    R = w.R
    q = W.bf16_bits(t["q"])
    rows = c.bounds_rows()
    for (b, h) in streams:
        K, V = W.bf16_bits(t["K"][b, h]), W.bf16_bits(t["V"][b, h])
        if t["mask_in"] is not None:
            m = W.u16_numpy(t["mask_in"][b, h]) & np.uint16((1 << w.G) - 1)
        else:
            m = O.route_mask(t["logits"][b, h].cpu().numpy(), t["kcount"][b, h].cpu().numpy())
        off = O.token_offsets(m, w.G)
        assert np.array_equal(W.bf16_bits(rows[b, h]), O.page_bounds(K))
        assert np.array_equal(PT.host_u16(c.mask[b, h]), m)
        assert np.array_equal(c.tok_off[b, h].cpu().numpy().view(np.uint32), off)
        assert np.array_equal(W.bf16_bits(c.vpacked[b, h, :int(off[-1])]),
                              O.pack_values(V, m, off, w.G))
        qh = q[b, h * R:(h + 1) * R]
        if w.k_pages >= w.NP:
            idx = np.arange(w.NP, dtype=np.int32)
        else:
            score = O.page_scores(qh, O.page_bounds(K))
            assert np.array_equal(c.page_score[b, h].cpu().numpy().view(np.uint32),
                                  score.view(np.uint32))
            idx = O.select_pages(score, w.k_pages)
        assert np.array_equal(c.page_idx[b, h].cpu().numpy(), idx)
        out = O.decode_attention(qh, K, V, m, idx, w.G)
        err = float(np.abs(c.out[b, h * R:(h + 1) * R].cpu().numpy() - out).max())
        assert err <= PT.TOL, (b, h, err)
        worst = max(worst, err)
    return worst


REDUCED = {
    "tiny": {},                                                         # as specified
    "llama2_7b_4k": dict(B=1, Hq=4, Hkv=4, N=1200, k_pages=19),
    "qwen25_7b_32k": dict(B=2, Hq=14, Hkv=2, N=3000, k_pages=24),
    "llava15_7b_prefix": dict(B=3, Hq=4, Hkv=4),
    "qwen25_7b_128k": dict(B=1, Hq=14, Hkv=2, N=5000, k_pages=32),
}


@pytest.mark.parametrize("name", W.ORDER)
def test_workload_reduced_every_stream(name):
    w = W.shrink(W.WORKLOADS[name], **REDUCED[name])
    c, t = _run_workload(w)
    assert int(c.dev_status.item()) == 0
    worst = _check_streams(w, c, t, [(b, h) for b in range(w.B) for h in range(w.Hkv)])
    assert worst <= PT.TIGHT


@pytest.mark.parametrize("name", W.ORDER)
def test_workload_full_size_sampled_streams(name):
    """The full workload sizes, in the launch configuration the benchmark times."""
    w = W.WORKLOADS[name]
    c, t = _run_workload(w)
    assert int(c.dev_status.item()) == 0
    idx = c.page_idx.cpu().numpy()
    assert idx.min() >= 0 and idx.max() < w.NP
    assert np.all(np.diff(idx, axis=-1) > 0)                 # strictly ascending: no duplicates
    out = c.out.cpu().numpy()
    assert np.all(np.isfinite(out))
    tot = c.tok_off[..., -1].cpu().numpy().view(np.uint32).astype(np.int64)
    if t["kcount"] is not None:                               # offsets end at the sum of counts
        assert np.array_equal(tot, t["kcount"].sum(dim=-1, dtype=torch.int64).cpu().numpy())
    streams = sorted({(0, 0), (w.B - 1, w.Hkv - 1), (w.B // 2, w.Hkv // 3)})
    worst = _check_streams(w, c, t, streams)
    assert worst <= PT.TIGHT


@pytest.mark.parametrize("name", ["llama2_7b_4k", "qwen25_7b_32k"])
def test_workload_full_size_every_stream_selection(name):
    """Full size, the benchmark's launch configuration: page bounds, page-score bits and the
    selected page list of EVERY stream against the oracle; the attention output on 8 streams
    spread over the batch (the oracle's attention is the slow part)."""
    w = W.WORKLOADS[name]
    c, t = _run_workload(w)
    assert int(c.dev_status.item()) == 0
    q = W.bf16_bits(t["q"])
    rows = c.bounds_rows()
    got_idx = c.page_idx.cpu().numpy()
    got_score = c.page_score.cpu().numpy().view(np.uint32)
    R = w.R
    for b in range(w.B):
        Kb, rb = W.bf16_bits(t["K"][b]), W.bf16_bits(rows[b])
        for h in range(w.Hkv):
            bounds = O.page_bounds(Kb[h])
            assert np.array_equal(rb[h], bounds), (b, h)
            score = O.page_scores(q[b, h * R:(h + 1) * R], bounds)
            assert np.array_equal(got_score[b, h], score.view(np.uint32)), (b, h)
            assert np.array_equal(got_idx[b, h], O.select_pages(score, w.k_pages)), (b, h)
    streams = sorted({(i * w.B // 8, (3 * i) % w.Hkv) for i in range(8)})
    assert len(streams) == 8
    worst = _check_streams(w, c, t, streams)
    assert worst <= PT.TIGHT


@pytest.mark.parametrize("B,k_pages,tail_cap", [(8, 108, 128), (2, 60, 96)])
def test_tail_decode_across_the_launch_plan_switch(B, k_pages, tail_cap):
    """Buffers sized once for the full tail must serve every tail length: with few streams the
    attention launch changes its plan (wavefronts per workgroup, hence splits) while the tail
    grows.  The step is run at tail lengths on both sides of the switch, with one workspace."""
    Hq, Hkv, D, G, N = 28, 4, 128, 8, 16 * 140
    K, V, q, logits, kcount = _rand_case(300 + B, B, Hq, Hkv, D, N, G)
    rng = np.random.default_rng(301)
    Kt, Vt = randn_bf16(rng, (B, Hkv, tail_cap, D)), randn_bf16(rng, (B, Hkv, tail_cap, D))
    dev = "cuda:0"
    c = stc.RoutedCache(B, Hq, Hkv, D, N, G, k_pages, device=dev, tail_cap=tail_cap)
    c.build(PT.to_dev_bf16(K), PT.to_dev_bf16(V), logits=torch.from_numpy(logits).to(dev),
            kcount=torch.from_numpy(kcount).to(dev))
    c.K_tail.copy_(PT.to_dev_bf16(Kt))
    c.V_tail.copy_(PT.to_dev_bf16(Vt))
    R = Hq // Hkv
    for n_tail in (0, 1, 40, 64, 65, tail_cap):
        c.n_tail = n_tail
        for one_call in (True, False):
            c.out.fill_(float("nan"))
            c.step(PT.to_dev_bf16(q), one_call=one_call)
            torch.cuda.synchronize()
            got, idx = c.out.cpu().numpy(), c.page_idx.cpu().numpy()
            for (b, h) in [(0, 0), (B - 1, Hkv - 1)]:
                m = O.route_mask(logits[b, h], kcount[b, h])
                qh = q[b, h * R:(h + 1) * R]
                want_idx = O.select_pages(O.page_scores(qh, O.page_bounds(K[b, h])), k_pages)
                assert np.array_equal(idx[b, h], want_idx)
                want = O.decode_attention(qh, K[b, h], V[b, h], m, want_idx, G,
                                          K_tail=Kt[b, h, :n_tail], V_tail=Vt[b, h, :n_tail])
                err = np.abs(got[b, h * R:(h + 1) * R] - want).max()
                assert err < PT.TIGHT, (n_tail, one_call, b, h, err)


@pytest.mark.parametrize("NP,k_pages", [(2500, 40), (8192, 100)])
def test_long_streams_select_inside_the_attention_kernel_with_and_without_a_tail(NP, k_pages):
    """Few streams of more than 2048 pages: the one-call step selects inside the attention
    kernel with 16 keys per thread; with a tail, the workgroups that hold only tail pages skip
    the selection.  Page lists bit-exact, outputs within the tight bound, one call and two."""
    B, Hq, Hkv, D, G, N, tail_cap = 1, 14, 2, 128, 8, 16 * NP - 5, 48
    K, V, q, logits, kcount = _rand_case(420 + NP, B, Hq, Hkv, D, N, G)
    rng = np.random.default_rng(421)
    Kt, Vt = randn_bf16(rng, (B, Hkv, tail_cap, D)), randn_bf16(rng, (B, Hkv, tail_cap, D))
    dev = "cuda:0"
    c = stc.RoutedCache(B, Hq, Hkv, D, N, G, k_pages, device=dev, tail_cap=tail_cap)
    c.build(PT.to_dev_bf16(K), PT.to_dev_bf16(V), logits=torch.from_numpy(logits).to(dev),
            kcount=torch.from_numpy(kcount).to(dev))
    c.K_tail.copy_(PT.to_dev_bf16(Kt))
    c.V_tail.copy_(PT.to_dev_bf16(Vt))
    R = Hq // Hkv
    want_idx = [O.select_pages(O.page_scores(q[0, h * R:(h + 1) * R], O.page_bounds(K[0, h])),
                               k_pages) for h in range(Hkv)]
    masks = [O.route_mask(logits[0, h], kcount[0, h]) for h in range(Hkv)]
    for n_tail in (0, 17, tail_cap):
        c.n_tail = n_tail
        for one_call in (True, False):
            c.out.fill_(float("nan"))
            c.page_idx.fill_(-7)
            c.step(PT.to_dev_bf16(q), one_call=one_call)
            torch.cuda.synchronize()
            got, idx = c.out.cpu().numpy(), c.page_idx.cpu().numpy()
            for h in range(Hkv):
                assert np.array_equal(idx[0, h], want_idx[h]), (n_tail, one_call, h)
                want = O.decode_attention(q[0, h * R:(h + 1) * R], K[0, h], V[0, h], masks[h],
                                          want_idx[h], G, K_tail=Kt[0, h, :n_tail],
                                          V_tail=Vt[0, h, :n_tail])
                err = np.abs(got[0, h * R:(h + 1) * R] - want).max()
                assert err < PT.TIGHT, (n_tail, one_call, h, err)


def test_global_budget_at_full_llm_size():
    """The LLM-mode routing of the paper (budget N*K over the whole stream, K = 4 of 8) on
    the headline shape: exact budget on every stream, masks of sampled streams bit for bit,
    and the decode step over the resulting cache within the bar."""
    w = W.WORKLOADS["qwen25_7b_32k"]
    inp = W.make_cache_inputs(w, "cuda:0", 0)
    c = stc.RoutedCache(w.B, w.Hq, w.Hkv, w.D, w.N, w.G, w.k_pages, device="cuda:0")
    c.build(inp["K"], inp["V"], logits=inp["logits"], global_k=4)
    q = W.make_query(w, 0, "cuda:0")
    c.step(q)
    torch.cuda.synchronize()
    assert int(c.dev_status.item()) == 0
    tot = c.tok_off[..., -1].cpu().numpy().view(np.uint32)
    assert (tot == w.N * 4).all()
    qb = W.bf16_bits(q)
    for (b, h) in [(0, 0), (w.B - 1, w.Hkv - 1)]:
        m = O.route_mask_global(inp["logits"][b, h].cpu().numpy(), w.N * 4)
        assert np.array_equal(PT.host_u16(c.mask[b, h]), m)
        kept = O.popcount(m, w.G)
        assert kept.min() == 0 and kept.max() == w.G         # non-uniform allocation
        K, V = W.bf16_bits(inp["K"][b, h]), W.bf16_bits(inp["V"][b, h])
        off = O.token_offsets(m, w.G)
        assert np.array_equal(c.tok_off[b, h].cpu().numpy().view(np.uint32), off)
        assert np.array_equal(W.bf16_bits(c.vpacked[b, h, :int(off[-1])]),
                              O.pack_values(V, m, off, w.G))
        qh = qb[b, h * w.R:(h + 1) * w.R]
        idx = O.select_pages(O.page_scores(qh, O.page_bounds(K)), w.k_pages)
        assert np.array_equal(c.page_idx[b, h].cpu().numpy(), idx)
        want = O.decode_attention(qh, K, V, m, idx, w.G)
        got = c.out[b, h * w.R:(h + 1) * w.R].cpu().numpy()
        assert np.abs(got - want).max() <= PT.TIGHT


def test_router_at_full_llm_size_sampled_tokens():
    """The router's projection on the headline shape (16 x 32768 tokens of width 3584, 8 groups,
    as the benchmark times it): sampled tokens bit for bit, the copies for all KV heads equal."""
    dev = "cuda:0"
    B, N, dm, G, Hkv = 16, 32768, 3584, 8, 4
    g = torch.Generator(device=dev)
    g.manual_seed(3584)
    h = torch.randn(B, N, dm, device=dev, generator=g).bfloat16()
    Wr = (torch.randn(G, dm, device=dev, generator=g) / dm ** 0.5).bfloat16()
    bias = torch.randn(G, device=dev, generator=g)
    logits = torch.full((B, Hkv, N, G), float("nan"), dtype=torch.float32, device=dev)
    stc.stc_router_logits(h, Wr, bias, logits, Hkv)
    torch.cuda.synchronize()
    assert torch.equal(logits[:, 0], logits[:, Hkv - 1])
    rng = np.random.default_rng(5)
    Wb, bb = W.bf16_bits(Wr), bias.cpu().numpy()
    for b in (0, 7, B - 1):
        ts = np.concatenate([[0, N - 1], rng.integers(0, N, size=30)])
        want = O.router_logits(W.bf16_bits(h[b, ts]), Wb, bb)
        got = logits[b, 1, ts].cpu().numpy()
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


def test_decode_step_with_tail_at_full_llm_size_sampled_streams():
    """The headline shape with 100 recent tokens in the uncompressed tail, through the one-call
    step as the benchmark's --rows times it: sampled streams against the oracle."""
    w = W.WORKLOADS["qwen25_7b_32k"]
    dev = "cuda:0"
    inp = W.make_cache_inputs(w, dev, 0)
    c = stc.RoutedCache(w.B, w.Hq, w.Hkv, w.D, w.N, w.G, w.k_pages, device=dev, tail_cap=128)
    c.build(inp["K"], inp["V"], logits=inp["logits"], kcount=inp["kcount"])
    g = torch.Generator(device=dev)
    g.manual_seed(9)
    c.K_tail.copy_(torch.randn(c.K_tail.shape, device=dev, generator=g))
    c.V_tail.copy_(torch.randn(c.V_tail.shape, device=dev, generator=g))
    c.n_tail = 100
    q = W.make_query(w, 3, dev)
    c.step(q)
    torch.cuda.synchronize()
    qb = W.bf16_bits(q)
    for (b, h) in [(0, 0), (w.B - 1, w.Hkv - 1), (5, 2)]:
        K, V = W.bf16_bits(inp["K"][b, h]), W.bf16_bits(inp["V"][b, h])
        m = O.route_mask(inp["logits"][b, h].cpu().numpy(), inp["kcount"][b, h].cpu().numpy())
        qh = qb[b, h * w.R:(h + 1) * w.R]
        idx = O.select_pages(O.page_scores(qh, O.page_bounds(K)), w.k_pages)
        assert np.array_equal(c.page_idx[b, h].cpu().numpy(), idx)
        want = O.decode_attention(qh, K, V, m, idx, w.G, K_tail=W.bf16_bits(c.K_tail[b, h, :100]),
                                  V_tail=W.bf16_bits(c.V_tail[b, h, :100]))
        got = c.out[b, h * w.R:(h + 1) * w.R].cpu().numpy()
        assert np.abs(got - want).max() <= PT.TIGHT


def test_per_head_and_union_forms_at_full_llm_size_sampled_heads():
    """The headline shape with one page list per query head, and with the lists of a KV head
    merged: lists, union and outputs of sampled heads against the oracle; the two forms agree."""
    w = W.WORKLOADS["qwen25_7b_32k"]
    dev = "cuda:0"
    inp = W.make_cache_inputs(w, dev, 0)
    c = stc.RoutedCache(w.B, w.Hq, w.Hkv, w.D, w.N, w.G, w.k_pages, device=dev)
    c.build(inp["K"], inp["V"], logits=inp["logits"], kcount=inp["kcount"])
    q = W.make_query(w, 1, dev)
    k, R, NP = w.k_pages, w.R, w.NP

    def ws(which, kk):
        return torch.empty(max(16, stc.stc_workspace_bytes(c.shape, which, kk)), dtype=torch.uint8,
                           device=dev)
    idx = torch.full((w.B, w.Hq, k), -1, dtype=torch.int32, device=dev)
    out = torch.full((w.B, w.Hq, w.D), float("nan"), dtype=torch.float32, device=dev)
    stc.stc_select_pages_per_head(c.shape, q, c.bounds, k, idx, None,
                                  ws(stc.STC_WS_SELECT_PER_HEAD, k))
    stc.stc_decode_attention_per_head(c.shape, q, c.K, c.vpacked, c.mask, c.tok_off, idx, k, out,
                                      ws(stc.STC_WS_ATTENTION_PER_HEAD, k))
    U = min(NP, R * k)
    uidx = torch.full((w.B, w.Hkv, U), -5, dtype=torch.int32, device=dev)
    uheads = torch.full((w.B, w.Hkv, U), -1, dtype=torch.int16, device=dev)
    out_u = torch.full_like(out, float("nan"))
    stc.stc_union_pages(c.shape, idx, k, uidx, uheads)
    stc.stc_decode_attention_union(c.shape, q, c.K, c.vpacked, c.mask, c.tok_off, uidx, uheads,
                                   out_u, ws(stc.STC_WS_ATTENTION, U))
    torch.cuda.synchronize()
    assert float((out - out_u).abs().max()) <= 2 * PT.TIGHT
    qb = W.bf16_bits(q)
    for (b, h) in [(0, 0), (w.B - 1, w.Hkv - 1)]:
        K, V = W.bf16_bits(inp["K"][b, h]), W.bf16_bits(inp["V"][b, h])
        m = O.route_mask(inp["logits"][b, h].cpu().numpy(), inp["kcount"][b, h].cpu().numpy())
        bounds = O.page_bounds(K)
        lists = []
        for r in (0, R // 2, R - 1):
            j = h * R + r
            want_idx = O.select_pages(O.page_scores(qb[b, j:j + 1], bounds), k)
            assert np.array_equal(idx[b, j].cpu().numpy(), want_idx)
            want = O.decode_attention(qb[b, j:j + 1], K, V, m, want_idx, w.G)
            assert np.abs(out[b, j:j + 1].cpu().numpy() - want).max() <= PT.TIGHT
            assert np.abs(out_u[b, j:j + 1].cpu().numpy() - want).max() <= PT.TIGHT
        pages, heads = O.union_pages(idx[b, h * R:(h + 1) * R].cpu().numpy(), NP)
        n = len(pages)
        assert np.array_equal(uidx[b, h, :n].cpu().numpy(), pages)
        assert np.array_equal(PT.host_u16(uheads[b, h])[:n], heads)
        assert (uidx[b, h, n:] == -1).all()


def test_steps_are_deterministic():
    w = W.shrink(W.WORKLOADS["qwen25_7b_32k"], B=2, N=8192, k_pages=64)
    c, t = _run_workload(w)
    first = (c.page_idx.clone(), c.out.clone())
    for _ in range(3):
        c.step(t["q"])
    torch.cuda.synchronize()
    assert torch.equal(c.page_idx, first[0]) and torch.equal(c.out, first[1])


def test_decode_steps_replayed_from_a_hip_graph():
    """The step calls allocate nothing and clear nothing through the runtime, so a caller may
    capture them: three caches (selection inside the attention kernel, selection as its own
    launch, a cache with an uncompressed tail) captured into one graph, replayed four times
    with fresh queries and eager work in between; every replay gives the eager bits."""
    dev = "cuda:0"
    g = torch.Generator(device=dev)
    g.manual_seed(77)
    specs = [(4, 14, 2, 128, 5000, 8, 40, 0), (1, 8, 8, 64, 40000, 4, 300, 0),
             (2, 8, 2, 128, 3000, 8, 24, 40)]
    caches, qbufs = [], []
    for (B, Hq, Hkv, D, N, G, k, tail) in specs:
        K = torch.randn(B, Hkv, N, D, device=dev, generator=g).bfloat16()
        V = torch.randn(B, Hkv, N, D, device=dev, generator=g).bfloat16()
        lg = torch.randn(B, Hkv, N, G, device=dev, generator=g)
        c = stc.RoutedCache(B, Hq, Hkv, D, N, G, k, device=dev, tail_cap=tail)
        c.build(K, V, logits=lg, fixed_k=G // 2)
        if tail:
            c.K_tail.copy_(torch.randn(c.K_tail.shape, device=dev, generator=g))
            c.V_tail.copy_(torch.randn(c.V_tail.shape, device=dev, generator=g))
            c.n_tail = tail - 3
        caches.append(c)
        qbufs.append(torch.randn(B, Hq, D, device=dev, generator=g).bfloat16())
    for c, q in zip(caches, qbufs):            # eager first: one-time set-up of the launches
        c.step(q)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            for c, q in zip(caches, qbufs):
                c.step(q)
    torch.cuda.synchronize()
    for rep in range(4):
        want = []
        for c, q in zip(caches, qbufs):
            q.copy_(torch.randn(q.shape, device=dev, generator=g))
            c.step(q)                           # eager
            want.append((c.page_idx.clone(), c.out.clone()))
            c.page_idx.fill_(-1)
            c.out.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for c, (wi, wo) in zip(caches, want):
            assert torch.equal(c.page_idx, wi) and torch.equal(c.out, wo), rep


@pytest.mark.parametrize("N,k", [(3000, 20), (40000, 100)])
def test_workspaces_are_reusable_without_clearing(N, k):
    """Alternating two queries on one cache: nothing a call leaves in the selection or
    attention workspace (scores, split partials) reaches the next call's results, and
    workspaces may hold anything beforehand."""
    B, Hq, Hkv, D, G = 2, 8, 2, 128, 8
    K, V, q, logits, kcount = _rand_case(33, B, Hq, Hkv, D, N, G)
    hip = PT.run_hip(K, V, q, G, k, logits=logits, kcount=kcount)
    c = hip["cache"]
    assert c._ws_attn.numel() > 16                      # several splits: partials are merged
    for b in range(B):
        for h in range(Hkv):
            sc = O.page_scores(q[b, h * 4:(h + 1) * 4], O.page_bounds(K[b, h]))
            assert np.array_equal(hip["page_idx"][b, h], O.select_pages(sc, k))
    ora = PT.run_oracle(K, V, q, G, k, logits=logits, kcount=kcount, streams=[(1, 1)])
    assert np.abs(hip["out"][1, 4:8] - ora[(1, 1)]["out"]).max() < PT.TOL
    rng = np.random.default_rng(34)
    q2 = randn_bf16(rng, q.shape)
    hip2 = PT.run_hip(K, V, q2, G, k, logits=logits, kcount=kcount)
    assert not np.array_equal(hip2["page_idx"], hip["page_idx"])
    sc2 = O.page_scores(q2[0, 0:4], O.page_bounds(K[0, 0]))
    assert np.array_equal(hip2["page_idx"][0, 0], O.select_pages(sc2, k))
    dq, dq2 = PT.to_dev_bf16(q), PT.to_dev_bf16(q2)
    for i, fill in enumerate((0xFF, None, 0x00, None, None, None, 0x01, None)):
        if fill is not None:
            c._ws_select.fill_(fill)
            c._ws_attn.fill_(fill)
        c.page_idx.fill_(-7)
        c.out.fill_(float("nan"))
        c.step(dq2 if i % 2 else dq)
        torch.cuda.synchronize()
        ref = hip2 if i % 2 else hip
        assert np.array_equal(c.page_idx.cpu().numpy(), ref["page_idx"])
        assert np.array_equal(c.out.cpu().numpy(), ref["out"])
