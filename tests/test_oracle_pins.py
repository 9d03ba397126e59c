"""Pins of the CPU oracle to things other than itself: values the paper prints,
closed forms, brute force on tiny inputs, library routines it must reduce to.
All CPU; none of this touches the HIP path."""
import itertools
import math
import os
from decimal import ROUND_HALF_UP, Decimal

import numpy as np
import pytest

from oracle import stc_oracle as O
from tests.helpers import bits_to_f64, f32_to_bf16_bits, ints_bf16, randn_bf16

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# --------------------------------------------------------------------------- #
# Budgets: the percentages printed in the paper (Sec. 4.2, App. C.2, LLM table)
# --------------------------------------------------------------------------- #
def _budget_rows():
    rows = []
    with open(os.path.join(GOLDEN, "budgets.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            r, S, K, printed, where = line.split()
            rows.append((float(r), int(S), int(K), printed, where))
    return rows


@pytest.mark.parametrize("r,S,K,printed,where", _budget_rows())
def test_budget_matches_printed_percentage(r, S, K, printed, where):
    pct = Decimal(repr(O.rho_total(r, K, S) * 100.0))
    digits = len(printed.split(".")[1])
    got = pct.quantize(Decimal(1).scaleb(-digits), rounding=ROUND_HALF_UP)
    assert str(got) == printed, (where, got, printed)


@pytest.mark.parametrize("G,Kk", [(4, 1), (8, 2), (16, 4), (8, 7), (16, 12)])
def test_packed_store_bytes_equal_value_budget(G, Kk):
    """With K of S groups kept per token the packed store holds exactly K/S of
    V's bytes, so K plus packed V is (1+K/S)/2 of the cache (Sec. 3.3)."""
    rng = np.random.default_rng(1)
    N, D = 48, 64
    V = randn_bf16(rng, (N, D))
    logits = rng.standard_normal((N, G)).astype(np.float32)
    mask = O.route_mask(logits, Kk)
    off = O.token_offsets(mask, G)
    packed = O.pack_values(V, mask, off, G)
    assert packed.nbytes * G == V.nbytes * Kk
    kv_kept = (V.nbytes + packed.nbytes) / (2 * V.nbytes)   # K bytes == V bytes
    assert kv_kept == O.rho_total(1.0, Kk, G)


# --------------------------------------------------------------------------- #
# Page bounds
# --------------------------------------------------------------------------- #
def test_bounds_brute_force_with_ragged_tail():
    rng = np.random.default_rng(2)
    N, D, P = 37, 8, 16                     # last page has 5 tokens
    K = randn_bf16(rng, (N, D))
    got = O.page_bounds(K, P)
    Kf = bits_to_f64(K)
    assert got.shape == (3, 2, D)
    for p in range(3):
        for c in range(D):
            vals = [Kf[t, c] for t in range(p * P, min((p + 1) * P, N))]
            assert bits_to_f64(got[p, 0, c]) == min(vals)
            assert bits_to_f64(got[p, 1, c]) == max(vals)


def test_bounds_signed_zero_order():
    # one page, one channel per case: -0 sorts below +0 whatever the order.
    for col, mn, mx in [([0x0000, 0x8000], 0x8000, 0x0000),
                        ([0x8000, 0x0000], 0x8000, 0x0000),
                        ([0x8000, 0x8000], 0x8000, 0x8000),
                        ([0x0000, 0x0000], 0x0000, 0x0000),
                        ([0x8000, 0x3F80], 0x8000, 0x3F80),     # -0, 1
                        ([0x0000, 0xBF80], 0xBF80, 0x0000)]:    # +0, -1
        K = np.array(col, dtype=np.uint16).reshape(2, 1)
        b = O.page_bounds(K, 16)
        assert (int(b[0, 0, 0]), int(b[0, 1, 0])) == (mn, mx)


def test_score_is_upper_bound_of_every_token_logit():
    rng = np.random.default_rng(3)
    N, D, P, R = 160, 32, 16, 3
    K = randn_bf16(rng, (N, D), 2.0)
    q = randn_bf16(rng, (R, D))
    U = O.head_page_bounds_score(q, O.page_bounds(K, P)).astype(np.float64)
    logit = bits_to_f64(q) @ bits_to_f64(K).T          # [R, N]
    for p in range(N // P):
        top = logit[:, p * P:(p + 1) * P].max(axis=1)
        assert np.all(U[:, p] >= top - 1e-4 * np.abs(top) - 1e-5)


# --------------------------------------------------------------------------- #
# Routing mask, offsets, packing
# --------------------------------------------------------------------------- #
def test_route_mask_equals_argsort_topk_when_no_ties():
    rng = np.random.default_rng(4)
    N, G = 200, 8
    a = rng.standard_normal((N, G)).astype(np.float32)
    c = rng.integers(0, G + 1, size=N)
    got = O.route_mask(a, c)
    for t in range(N):
        top = np.argsort(-a[t].astype(np.float64), kind="stable")[:c[t]]
        assert int(got[t]) == sum(1 << int(g) for g in top)


def test_route_mask_ties_go_to_lowest_group_and_extremes():
    a = np.array([[1, 1, 1, 1], [0, 2, 2, 0], [5, 5, 7, 5]], dtype=np.float32)
    assert list(O.route_mask(a, 2)) == [0b0011, 0b0110, 0b0101]
    assert list(O.route_mask(a, 0)) == [0, 0, 0]
    assert list(O.route_mask(a, 4)) == [0b1111] * 3
    assert list(O.route_mask(a, np.array([1, 3, 4]))) == [0b0001, 0b0111, 0b1111]


def test_offsets_are_cumsum_of_popcounts():
    rng = np.random.default_rng(5)
    G = 16
    mask = rng.integers(0, 1 << G, size=300).astype(np.uint16)
    off = O.token_offsets(mask, G)
    pc = np.array([bin(int(m)).count("1") for m in mask])
    assert off.dtype == np.uint32 and off[0] == 0
    assert np.array_equal(off[1:], np.cumsum(pc))


@pytest.mark.parametrize("G", [1, 4, 8, 16])
def test_pack_round_trip_and_order(G):
    rng = np.random.default_rng(6)
    N, D = 75, 64
    gd = D // G
    V = randn_bf16(rng, (N, D))
    mask = rng.integers(0, 1 << G, size=N).astype(np.uint16)
    mask[3] = 0
    mask[4] = (1 << G) - 1
    off = O.token_offsets(mask, G)
    packed = O.pack_values(V, mask, off, G)
    keep = ((mask[:, None] >> np.arange(G)[None, :]) & 1).astype(bool)      # [N, G]
    # token order, then ascending group: row-major boolean selection
    assert np.array_equal(packed, V.reshape(N, G, gd)[keep])
    # unpack == mask * V, bit for bit (dropped groups are +0)
    un = np.zeros((N, G, gd), dtype=np.uint16)
    un[keep] = packed
    assert np.array_equal(un.reshape(N, D), np.where(np.repeat(keep, gd, axis=1), V, 0))


def test_pack_all_groups_kept_is_identity():
    rng = np.random.default_rng(7)
    N, D, G = 20, 32, 4
    V = randn_bf16(rng, (N, D))
    mask = O.route_mask(rng.standard_normal((N, G)).astype(np.float32), G)
    off = O.token_offsets(mask, G)
    assert np.array_equal(O.pack_values(V, mask, off, G).reshape(N, D), V)


# --------------------------------------------------------------------------- #
# Page score: value, summation order, sign handling, GQA rule
# --------------------------------------------------------------------------- #
def test_score_summation_order_is_adjacent_pair_tree():
    """terms 1, 1.5e, e, 3e with e = 2^-24, u = 2^-23 = ulp(1), all factors bf16.
    Adjacent pairs: (1+1.5e) -> 1+u (0.75u rounds up); (e+3e) = 2u; total 1+3u exact.
    A half-stride tree gives 1+2u ((1+e) ties to 1, then 1+2.25u -> 1+2u);
    a left-to-right sum gives 1+4u.  Only the adjacent tree yields 1+3u."""
    e = 2.0 ** -24
    t = np.array([1.0, 1.5 * e, e, 3 * e], dtype=np.float32)
    b = f32_to_bf16_bits(t)
    assert np.array_equal(bits_to_f64(b), t.astype(np.float64))
    bounds = np.stack([b, b])[None]                           # mn == mx
    q = f32_to_bf16_bits(np.ones((1, 4), dtype=np.float32))
    U = O.head_page_bounds_score(q, bounds)
    assert U.dtype == np.float32
    assert float(U[0, 0]) == 1.0 + 3 * 2.0 ** -23


def test_score_exact_on_small_integers():
    rng = np.random.default_rng(8)
    R, NP, D = 2, 9, 16
    q = ints_bf16(rng, (R, D), -4, 4)
    lo = rng.integers(-8, 8, size=(NP, D))
    hi = lo + rng.integers(0, 5, size=(NP, D))
    bounds = np.stack([f32_to_bf16_bits(lo.astype(np.float32)),
                       f32_to_bf16_bits(hi.astype(np.float32))], axis=1)
    U = O.head_page_bounds_score(q, bounds)
    qi = bits_to_f64(q).astype(int)
    for h, p in itertools.product(range(R), range(NP)):
        want = sum(max(int(qi[h, c]) * int(lo[p, c]), int(qi[h, c]) * int(hi[p, c]))
                   for c in range(D))
        assert float(U[h, p]) == float(want)


def test_score_close_to_float64_and_per_channel_max():
    rng = np.random.default_rng(9)
    R, N, D = 7, 256, 128
    K = randn_bf16(rng, (N, D), 3.0)
    q = randn_bf16(rng, (R, D))
    bounds = O.page_bounds(K)
    U = O.head_page_bounds_score(q, bounds).astype(np.float64)
    qf, bf = bits_to_f64(q), bits_to_f64(bounds)
    for h in range(R):
        for p in range(N // 16):
            terms = [max(qf[h, c] * bf[p, 0, c], qf[h, c] * bf[p, 1, c]) for c in range(D)]
            assert abs(U[h, p] - math.fsum(terms)) <= 1e-5 * math.fsum(abs(x) for x in terms)


def test_stream_score_is_max_over_group_heads_and_zero_is_positive():
    rng = np.random.default_rng(10)
    R, N, D = 4, 64, 16
    bounds = O.page_bounds(randn_bf16(rng, (N, D)))
    q = randn_bf16(rng, (R, D))
    per_head = np.stack([O.page_scores(q[h:h + 1], bounds) for h in range(R)])
    assert np.array_equal(O.page_scores(q, bounds), per_head.max(axis=0))
    zq = np.full((R, D), 0x8000, dtype=np.uint16)             # q = -0 everywhere
    s = O.page_scores(zq, bounds)
    assert np.array_equal(s.view(np.uint32), np.zeros(N // 16, dtype=np.uint32))


# --------------------------------------------------------------------------- #
# Selection
# --------------------------------------------------------------------------- #
def test_select_brute_force_with_ties():
    rng = np.random.default_rng(11)
    for trial in range(50):
        NP = int(rng.integers(1, 40))
        k = int(rng.integers(1, NP + 3))
        score = rng.integers(-3, 4, size=NP).astype(np.float32)      # many ties
        got = O.select_pages(score, k)
        # brute force: repeatedly take the best remaining (first of equals)
        left, want = list(range(NP)), []
        for _ in range(min(k, NP)):
            best = left[0]
            for p in left:
                if score[p] > score[best]:
                    best = p
            want.append(best)
            left.remove(best)
        assert got.dtype == np.int32
        assert list(got) == sorted(want)


def test_select_zero_query_takes_first_pages():
    rng = np.random.default_rng(12)
    bounds = O.page_bounds(randn_bf16(rng, (320, 32)))
    q = np.zeros((2, 32), dtype=np.uint16)
    assert list(O.select_pages(O.page_scores(q, bounds), 5)) == [0, 1, 2, 3, 4]


def test_select_on_constant_pages_is_topk_of_token_logits():
    """If every token of a page has the same key, min == max, so the page score
    is exactly that key's dot product with q and selection is a plain top-k."""
    rng = np.random.default_rng(13)
    NP, D, P, k = 24, 8, 16, 6
    page_key = ints_bf16(rng, (NP, D), -6, 6)
    K = np.repeat(page_key, P, axis=0)
    q = ints_bf16(rng, (1, D), -3, 3)
    idx = O.select_pages(O.page_scores(q, O.page_bounds(K, P)), k)
    logit = (bits_to_f64(page_key) @ bits_to_f64(q)[0])
    want = sorted(sorted(range(NP), key=lambda p: (-logit[p], p))[:k])
    assert list(idx) == want


def test_select_all_pages_when_k_at_least_np():
    s = np.array([3, 1, 2], dtype=np.float32)
    assert list(O.select_pages(s, 3)) == [0, 1, 2]
    assert list(O.select_pages(s, 10)) == [0, 1, 2]


# --------------------------------------------------------------------------- #
# Attention
# --------------------------------------------------------------------------- #
def _dense_attention_f64(q, K, V):
    """softmax(q K^T / sqrt(D)) V with library routines, float64."""
    from scipy.special import softmax
    D = q.shape[-1]
    return softmax(q @ K.T / np.sqrt(D), axis=-1) @ V


def test_attention_full_budget_all_groups_is_dense_attention():
    rng = np.random.default_rng(14)
    N, D, G, R = 96, 64, 4, 3
    q, K, V = randn_bf16(rng, (R, D)), randn_bf16(rng, (N, D)), randn_bf16(rng, (N, D))
    mask = np.full(N, (1 << G) - 1, dtype=np.uint16)
    got = O.decode_attention(q, K, V, mask, np.arange(N // 16), G)
    want = _dense_attention_f64(bits_to_f64(q), bits_to_f64(K), bits_to_f64(V))
    assert np.abs(got - want).max() <= 1e-6
    import torch
    tq = torch.from_numpy(bits_to_f64(q))[None, :, None, :]            # [1, R, 1, D]
    tk = torch.from_numpy(bits_to_f64(K))[None, None].expand(1, R, N, D)
    tv = torch.from_numpy(bits_to_f64(V))[None, None].expand(1, R, N, D)
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)[0, :, 0].numpy()
    assert np.abs(got - ref).max() <= 1e-6


def test_attention_masked_equals_dense_on_zero_filled_values():
    rng = np.random.default_rng(15)
    N, D, G, R, P = 100, 64, 8, 2, 16                   # ragged last page (4 tokens)
    gd = D // G
    q, K, V = randn_bf16(rng, (R, D), 4.0), randn_bf16(rng, (N, D)), randn_bf16(rng, (N, D))
    mask = rng.integers(0, 1 << G, size=N).astype(np.uint16)
    mask &= np.uint16(~(1 << 5) & 0xFFFF)               # nobody keeps group 5
    pages = np.array([0, 2, 3, 6], dtype=np.int32)      # page 6 is the ragged one
    got = O.decode_attention(q, K, V, mask, pages, G, P)
    toks = np.concatenate([np.arange(p * P, min((p + 1) * P, N)) for p in pages])
    keep = np.repeat(((mask[:, None] >> np.arange(G)) & 1), gd, axis=1)
    Vz = bits_to_f64(V) * keep
    want = _dense_attention_f64(bits_to_f64(q), bits_to_f64(K)[toks], Vz[toks])
    assert np.abs(got - want).max() <= 1e-6
    assert np.all(got[:, 5 * gd:6 * gd] == 0.0)         # dropped groups give exactly 0
    assert np.any(got[:, :gd] != 0.0)


def test_attention_closed_form_uniform_weights():
    """q = 0: every weight is 1/|T| (|T| = 64), so out = (sum of kept V)/64 exactly."""
    rng = np.random.default_rng(16)
    N, D, G, P = 128, 32, 4, 16
    gd = D // G
    K = randn_bf16(rng, (N, D))
    Vi = rng.integers(-8, 9, size=(N, D))
    V = f32_to_bf16_bits(Vi.astype(np.float32))
    mask = rng.integers(0, 1 << G, size=N).astype(np.uint16)
    pages = np.array([1, 3, 4, 7], dtype=np.int32)
    got = O.decode_attention(np.zeros((1, D), dtype=np.uint16), K, V, mask, pages, G, P)
    for c in range(D):
        tot = sum(int(Vi[t, c]) for p in pages for t in range(p * P, (p + 1) * P)
                  if (int(mask[t]) >> (c // gd)) & 1)
        assert float(got[0, c]) == tot / 64.0


def test_attention_token_without_groups_still_counts_in_denominator():
    D, G = 16, 2
    K = np.zeros((2, D), dtype=np.uint16)
    V = f32_to_bf16_bits(np.full((2, D), 6.0, dtype=np.float32))
    mask = np.array([0b11, 0b00], dtype=np.uint16)
    got = O.decode_attention(np.zeros((1, D), dtype=np.uint16), K, V, mask, np.array([0]), G)
    assert np.all(got == 3.0)


def test_single_group_is_token_level_quest():
    """G = 1 with every token kept: output is dense attention over the selected pages."""
    rng = np.random.default_rng(17)
    N, D, P, k = 256, 32, 16, 5
    q, K, V = randn_bf16(rng, (1, D), 3.0), randn_bf16(rng, (N, D)), randn_bf16(rng, (N, D))
    idx = O.select_pages(O.page_scores(q, O.page_bounds(K, P)), k)
    mask = np.ones(N, dtype=np.uint16)
    got = O.decode_attention(q, K, V, mask, idx, 1, P)
    toks = np.concatenate([np.arange(p * P, (p + 1) * P) for p in idx])
    want = _dense_attention_f64(bits_to_f64(q), bits_to_f64(K)[toks], bits_to_f64(V)[toks])
    assert np.abs(got - want).max() <= 1e-6


def test_attention_page_order_invariance_and_ones():
    rng = np.random.default_rng(18)
    N, D, G = 160, 32, 4
    q, K, V = randn_bf16(rng, (2, D)), randn_bf16(rng, (N, D)), randn_bf16(rng, (N, D))
    mask = rng.integers(0, 1 << G, size=N).astype(np.uint16)
    pages = np.array([0, 2, 5, 7, 9])
    a = O.decode_attention(q, K, V, mask, pages, G)
    b = O.decode_attention(q, K, V, mask, pages[::-1].copy(), G)
    assert np.abs(a - b).max() <= 1e-6
    ones = f32_to_bf16_bits(np.ones((N, D), dtype=np.float32))
    full = np.full(N, (1 << G) - 1, dtype=np.uint16)
    assert np.abs(O.decode_attention(q, K, ones, full, pages, G) - 1.0).max() <= 1e-6


def test_attention_peaked_softmax_picks_the_matching_token():
    """A query equal to 16x one key (all other keys orthogonal-ish small) puts
    essentially all weight on that token: out == its kept values."""
    N, D, G = 32, 16, 4
    gd = D // G
    K = np.zeros((N, D), dtype=np.float32)
    for t in range(N):
        K[t, t % D] = 1.0 + (t // D)                    # token 21: K[21, 5] = 2
    q = np.zeros((1, D), dtype=np.float32)
    q[0, 5] = 200.0
    V = np.arange(N * D, dtype=np.float32).reshape(N, D) % 97
    mask = np.full(N, 0b1011, dtype=np.uint16)
    got = O.decode_attention(f32_to_bf16_bits(q), f32_to_bf16_bits(K), f32_to_bf16_bits(V),
                             mask, np.array([0, 1]), G)
    want = V[21].copy()
    want[2 * gd:3 * gd] = 0.0
    assert np.abs(got[0] - want).max() <= 1e-6


def test_all_wrappers_use_gqa_head_layout_of_sdpa():
    """Query head j reads KV head j // (Hq/Hkv), the usual GQA convention
    (checked against torch SDPA on K, V repeated per query head)."""
    import torch
    rng = np.random.default_rng(19)
    B, Hq, Hkv, N, D, G = 2, 6, 2, 64, 32, 4
    q = randn_bf16(rng, (B, Hq, D))
    K = randn_bf16(rng, (B, Hkv, N, D))
    V = randn_bf16(rng, (B, Hkv, N, D))
    mask = np.full((B, Hkv, N), (1 << G) - 1, dtype=np.uint16)
    bounds = O.build_page_bounds_all(K)
    idx, score = O.select_pages_all(q, bounds, N // 16)
    assert np.array_equal(idx, np.broadcast_to(np.arange(N // 16, dtype=np.int32), idx.shape))
    got = O.decode_attention_all(q, K, V, mask, idx, G)
    R = Hq // Hkv
    tq = torch.from_numpy(bits_to_f64(q))[:, :, None, :]
    tk = torch.from_numpy(bits_to_f64(K)).repeat_interleave(R, dim=1)
    tv = torch.from_numpy(bits_to_f64(V)).repeat_interleave(R, dim=1)
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)[:, :, 0].numpy()
    assert np.abs(got - ref).max() <= 1e-6


def test_route_and_pack_all_modes_agree():
    rng = np.random.default_rng(20)
    B, Hkv, N, D, G = 2, 2, 40, 32, 8
    V = randn_bf16(rng, (B, Hkv, N, D))
    logits = rng.standard_normal((B, Hkv, N, G)).astype(np.float32)
    kc = rng.integers(0, G + 1, size=(B, Hkv, N)).astype(np.uint8)
    m1, o1, p1 = O.route_and_pack_all(V, G, logits=logits, kcount=kc)
    m2, o2, p2 = O.route_and_pack_all(V, G, mask_in=m1 | np.uint16(0xFF00))
    assert np.array_equal(m1, m2) and np.array_equal(o1, o2)
    assert all(np.array_equal(a, b) for a, b in zip(p1, p2))
    assert np.array_equal(o1[..., -1], np.array(kc, dtype=np.int64).sum(axis=-1))


# --- global token-group budget (Sec. 3.4; App. B.1: M = N*K of the N x S pairs) -----------

def test_global_budget_brute_force_with_ties():
    """Plain Python: rank every (token, group) pair by (logit descending, flat index
    ascending) and keep the first M; logits drawn from few values so ties are everywhere,
    including -0 against +0."""
    rng = np.random.default_rng(50)
    for N, G, M in ((7, 4, 9), (5, 8, 17), (9, 2, 0), (3, 16, 48), (6, 4, 1)):
        a = rng.choice(np.array([-1.5, -0.0, 0.0, 0.25, 2.0], dtype=np.float32), size=(N, G))
        pairs = [(t, g) for t in range(N) for g in range(G)]
        ranked = sorted(pairs, key=lambda tg: (-float(a[tg]), tg[0] * G + tg[1]))
        want = np.zeros(N, dtype=np.uint16)
        for (t, g) in ranked[:M]:
            want[t] |= np.uint16(1 << g)
        got = O.route_mask_global(a, M)
        assert np.array_equal(got, want)
        assert int(O.popcount(got, G).sum()) == M


def test_global_budget_keeps_exactly_m_above_a_threshold():
    rng = np.random.default_rng(51)
    N, G, K = 500, 8, 3
    a = rng.standard_normal((N, G)).astype(np.float32)
    m = O.route_mask_global(a, N * K)
    bits = (m[:, None] >> np.arange(G)) & 1
    assert int(bits.sum()) == N * K                       # the budget is met exactly
    assert a[bits == 1].min() > a[bits == 0].max()         # no ties here: a clean threshold
    assert np.array_equal(O.route_mask_global(a, 0), np.zeros(N, dtype=np.uint16))
    assert np.array_equal(O.route_mask_global(a, N * G), np.full(N, (1 << G) - 1, dtype=np.uint16))
    with pytest.raises(ValueError):
        O.route_mask_global(a, N * G + 1)


def test_global_budget_equals_per_token_topk_when_tokens_share_one_value_set():
    """Every token's logits are a permutation of the same G distinct values, so the N*K
    largest pairs of the grid are exactly every token's own top K (App. B.1's fixed-K mode)."""
    rng = np.random.default_rng(52)
    N, G = 64, 8
    vals = np.arange(G, dtype=np.float32) * 0.5 - 1.0
    a = np.stack([rng.permutation(vals) for _ in range(N)])
    for K in (1, 3, 8):
        assert np.array_equal(O.route_mask_global(a, N * K), O.route_mask(a, K))


def test_global_budget_all_equal_logits_fill_in_token_order():
    N, G, M = 10, 4, 14
    m = O.route_mask_global(np.zeros((N, G), dtype=np.float32), M)
    assert list(m[:5]) == [15, 15, 15, 3, 0] and not m[5:].any()


def test_global_budget_allocation_is_non_uniform_as_in_the_diagnostic_figure():
    """Fig. 1 caption: S = 4, average budget 1.0 per token; some tokens get no group, some
    all four, many a partial allocation.  For iid continuous logits the threshold sits at
    the 3/4 quantile, so P(no group) -> (3/4)^4 and P(all four) -> (1/4)^4."""
    rng = np.random.default_rng(53)
    N, S = 40000, 4
    a = rng.standard_normal((N, S)).astype(np.float32)
    kept = O.popcount(O.route_mask_global(a, N * 1), S)
    assert kept.sum() == N and kept.mean() == 1.0
    assert abs((kept == 0).mean() - 0.75 ** 4) < 0.01
    assert abs((kept == 4).mean() - 0.25 ** 4) < 0.002
    assert (kept == 1).any() and (kept == 2).any() and (kept == 3).any()


def test_route_and_pack_all_global_mode():
    rng = np.random.default_rng(54)
    B, Hkv, N, D, G = 2, 2, 40, 64, 4
    V = randn_bf16(rng, (B, Hkv, N, D))
    logits = rng.standard_normal((B, Hkv, N, G)).astype(np.float32)
    mask, off, packed = O.route_and_pack_all(V, G, logits=logits, global_k=2)
    for b in range(B):
        for h in range(Hkv):
            assert np.array_equal(mask[b, h], O.route_mask_global(logits[b, h], 2 * N))
            assert int(off[b, h, -1]) == 2 * N == packed[b * Hkv + h].shape[0]


# --- uncompressed recent tail (Sec. 3.4 exempts the query region from compression) --------

def test_attention_with_tail_is_dense_attention_over_both_sets():
    """Definition written out: one softmax over the selected cached tokens (routed values)
    and every tail token (full values), against numpy float64 and torch SDPA float64."""
    import torch
    rng = np.random.default_rng(60)
    N, D, G, R, nt = 96, 64, 4, 3, 21
    gd = D // G
    K, V = randn_bf16(rng, (N, D)), randn_bf16(rng, (N, D))
    Kt, Vt = randn_bf16(rng, (nt, D)), randn_bf16(rng, (nt, D))
    q = randn_bf16(rng, (R, D))
    mask = rng.integers(0, 1 << G, size=N).astype(np.uint16)
    pages = [1, 4, 5]
    got = O.decode_attention(q, K, V, mask, pages, G, K_tail=Kt, V_tail=Vt)
    toks = np.concatenate([np.arange(p * 16, p * 16 + 16) for p in pages])
    keep = np.repeat((mask[toks, None] >> np.arange(G)) & 1, gd, axis=1)
    Kall = np.concatenate([bits_to_f64(K)[toks], bits_to_f64(Kt)])
    Vall = np.concatenate([bits_to_f64(V)[toks] * keep, bits_to_f64(Vt)])
    s = bits_to_f64(q) @ Kall.T / math.sqrt(D)
    w = np.exp(s - s.max(axis=1, keepdims=True))
    want = (w / w.sum(axis=1, keepdims=True)) @ Vall
    assert np.abs(got - want).max() < 1e-6
    sd = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(bits_to_f64(q))[None], torch.from_numpy(Kall)[None],
        torch.from_numpy(Vall)[None]).numpy()[0]
    assert np.abs(got - sd).max() < 1e-6


def test_attention_tail_special_cases():
    rng = np.random.default_rng(61)
    N, D, G, R = 64, 64, 4, 2
    K, V = randn_bf16(rng, (N, D)), randn_bf16(rng, (N, D))
    q = randn_bf16(rng, (R, D))
    mask = rng.integers(0, 1 << G, size=N).astype(np.uint16)
    base = O.decode_attention(q, K, V, mask, [0, 2], G)
    # an empty tail changes nothing
    empty = np.zeros((0, D), dtype=np.uint16)
    assert np.array_equal(O.decode_attention(q, K, V, mask, [0, 2], G, K_tail=empty, V_tail=empty),
                          base)
    # moving a fully kept page from the cache into the tail gives the same output
    full = mask.copy()
    full[48:64] = (1 << G) - 1
    a = O.decode_attention(q, K, V, full, [0, 2, 3], G)
    b = O.decode_attention(q, K, V, full, [0, 2], G, K_tail=K[48:64], V_tail=V[48:64])
    assert np.abs(a - b).max() < 1e-6
    # a tail token whose key matches the query dominates: the output is its full value row
    Kt = f32_to_bf16_bits(bits_to_f64(q[:1]).astype(np.float32) * 6.0)
    Vt = ints_bf16(rng, (1, D), -8, 9)
    o = O.decode_attention(q[:1], K, V, np.zeros(N, dtype=np.uint16), [0, 1, 2, 3], G,
                           K_tail=Kt, V_tail=Vt)
    assert np.abs(o[0] - bits_to_f64(Vt)[0]).max() < 1e-3


# --- per-query-head page selection (the other reading of Quest under GQA) -----------------

def test_per_head_selection_is_each_heads_own_topk():
    """Constant pages: bounds collapse (min = max), a head's page score is exactly its logit
    with any token of the page, so each head's selection is the textbook top-k of ITS logits,
    and heads of one group choose different pages."""
    rng = np.random.default_rng(70)
    B, Hq, Hkv, D, NP, k = 1, 4, 2, 64, 12, 4
    page_rows = ints_bf16(rng, (B, Hkv, NP, D), -3, 3)
    K = np.repeat(page_rows, 16, axis=2)                     # [B, Hkv, NP*16, D]
    q = ints_bf16(rng, (B, Hq, D), -3, 3)
    bounds = O.build_page_bounds_all(K)
    idx, score = O.select_pages_per_head_all(q, bounds, k)
    assert idx.shape == (B, Hq, k) and score.shape == (B, Hq, NP)
    for j in range(Hq):
        logit = bits_to_f64(page_rows[0, j // 2]) @ bits_to_f64(q[0, j])
        assert np.array_equal(score[0, j].astype(np.float64), logit)
        want = sorted(sorted(range(NP), key=lambda p: (-logit[p], p))[:k])
        assert list(idx[0, j]) == want
    assert not np.array_equal(idx[0, 0], idx[0, 1])          # same KV head, different pages


def test_per_head_equals_shared_selection_for_mha_and_for_identical_heads():
    rng = np.random.default_rng(71)
    B, Hkv, D, N, k = 2, 2, 64, 160, 3
    K = randn_bf16(rng, (B, Hkv, N, D))
    bounds = O.build_page_bounds_all(K)
    q = randn_bf16(rng, (B, Hkv, D))                          # MHA: one head per KV head
    a, sa = O.select_pages_per_head_all(q, bounds, k)
    b_, sb = O.select_pages_all(q, bounds, k)
    assert np.array_equal(a, b_) and np.array_equal(sa.view(np.uint32), sb.view(np.uint32))
    q3 = np.repeat(q, 3, axis=1)                              # 3 identical heads per KV head
    c, _ = O.select_pages_per_head_all(q3, bounds, k)
    assert np.array_equal(c, np.repeat(b_, 3, axis=1))


def test_per_head_attention_wrapper_uses_each_heads_pages():
    rng = np.random.default_rng(72)
    B, Hq, Hkv, D, N, G, k = 1, 4, 2, 64, 96, 4, 2
    K, V = randn_bf16(rng, (B, Hkv, N, D)), randn_bf16(rng, (B, Hkv, N, D))
    q = randn_bf16(rng, (B, Hq, D))
    mask = rng.integers(0, 1 << G, size=(B, Hkv, N)).astype(np.uint16)
    idx, _ = O.select_pages_per_head_all(q, O.build_page_bounds_all(K), k)
    out = O.decode_attention_per_head_all(q, K, V, mask, idx, G)
    for j in range(Hq):
        want = O.decode_attention(q[0, j:j + 1], K[0, j // 2], V[0, j // 2], mask[0, j // 2],
                                  idx[0, j], G)
        assert np.array_equal(out[0, j:j + 1], want)


# --- router logits (App. B.1: one linear projection from the hidden state to S logits) -----

def test_router_logits_exact_on_small_integers_and_close_to_float64():
    rng = np.random.default_rng(80)
    N, dm, G = 37, 384, 8
    h, W = ints_bf16(rng, (N, dm), -4, 4), ints_bf16(rng, (G, dm), -4, 4)
    bias = rng.integers(-5, 6, size=G).astype(np.float32)
    got = O.router_logits(h, W, bias)
    want = bits_to_f64(h) @ bits_to_f64(W).T + bias            # integers: exact in any order
    assert got.dtype == np.float32 and np.array_equal(got.astype(np.float64), want)
    h, W = randn_bf16(rng, (N, dm)), randn_bf16(rng, (G, dm))
    got = O.router_logits(h, W)
    want = bits_to_f64(h) @ bits_to_f64(W).T
    assert np.abs(got - want).max() < 1e-4 * np.abs(want).max()
    # transposed operands or a dropped chunk would not survive this
    assert np.abs(O.router_logits(h[:, :128], W[:, :128]) - want).max() > 1.0


def test_router_logits_summation_order():
    """Within a chunk of 128 channels: balanced adjacent-pair tree.  Across chunks: left to
    right.  With e = 2^-24 (half an ulp of 1.0f) the two orders round differently."""
    e = 2.0 ** -24
    one = f32_to_bf16_bits(np.float32(1.0))
    def row(vals, dm):
        r = np.zeros(dm, dtype=np.float32)
        for i, v in vals.items():
            r[i] = v
        return f32_to_bf16_bits(r)
    W = np.full((1, 256), one, dtype=np.uint16)
    # chunk sums 1, e... : terms (1, 1.5e, e, 3e) at channels 0..3 of chunk 0, as in the page
    # score pin: tree gives (1 + 1.5e) + (e + 3e) = (1 + 2e) + 4e = 1 + 6e -> 1 + 3u (u = 2e)
    h = row({0: 1.0, 1: 1.5 * e, 2: e, 3: 3 * e}, 256)[None]
    assert float(O.router_logits(h, W)[0, 0]) == 1.0 + 6 * e
    # left to right over the four terms would give ((1 + 1.5e) + e) + 3e = (1+2e) + e -> 1+2e, +3e
    assert float(np.float32(np.float32(np.float32(np.float32(1.0) + np.float32(1.5 * e))
                                       + np.float32(e)) + np.float32(3 * e))) != 1.0 + 6 * e
    # across chunks: chunk sums (1, e, e): left to right (1 + e) + e = 1 (ties to even, twice);
    # a tree over the chunks would give 1 + (e + e) = 1 + 2e
    W3 = np.full((1, 384), one, dtype=np.uint16)
    h3 = row({0: 1.0, 128: e, 256: e}, 384)[None]
    assert float(O.router_logits(h3, W3)[0, 0]) == 1.0
    # the bias is added after the last chunk
    assert float(O.router_logits(h3, W3, np.array([2 * e], dtype=np.float32))[0, 0]) == 1.0 + 2 * e


def test_router_then_routing_pipeline():
    rng = np.random.default_rng(81)
    N, dm, G = 50, 256, 4
    h, W = randn_bf16(rng, (N, dm)), randn_bf16(rng, (G, dm))
    a = O.router_logits(h, W)
    m = O.route_mask(a, 2)
    top2 = np.argsort(-a, axis=1, kind="stable")[:, :2]
    want = (1 << top2[:, 0]) | (1 << top2[:, 1])
    assert np.array_equal(m, want.astype(np.uint16))


def test_union_pages_is_the_set_union_with_membership():
    rng = np.random.default_rng(73)
    NP, R, k = 40, 5, 7
    lists = np.stack([np.sort(rng.choice(NP, k, replace=False)) for _ in range(R)]).astype(np.int32)
    lists[2, 3] = -1                                         # ignored entry
    pages, heads = O.union_pages(lists, NP)
    want = sorted(set(int(p) for row in lists for p in row if p >= 0))
    assert list(pages) == want
    for p, m in zip(pages, heads):
        assert int(m) == sum(1 << r for r in range(R) if p in lists[r])
    # attending the union with membership = attending each head's own list
    D, G, N = 64, 4, NP * 16
    K, V = randn_bf16(rng, (N, D)), randn_bf16(rng, (N, D))
    q = randn_bf16(rng, (R, D))
    mask = rng.integers(0, 1 << G, size=N).astype(np.uint16)
    for r in range(R):
        own = O.decode_attention(q[r:r + 1], K, V, mask, [p for p in lists[r] if p >= 0], G)
        via = O.decode_attention(q[r:r + 1], K, V, mask, pages[(heads >> r) & 1 == 1], G)
        assert np.abs(own - via).max() < 1e-6


# --------------------------------------------------------------------------- #
# Subnormal bf16 inputs of the two multiply-and-sum routines count as zero
# --------------------------------------------------------------------------- #
def _with_subnormals(rng, bits, frac=0.15):
    """A copy of bf16 bit patterns with a share of entries replaced by subnormal patterns
    (exponent field 0, non-zero mantissa, either sign), and the same copy with zeros there."""
    sub = bits.copy()
    zero = bits.copy()
    hit = rng.random(bits.shape) < frac
    mant = rng.integers(1, 128, size=bits.shape).astype(np.uint16)
    sign = (rng.integers(0, 2, size=bits.shape).astype(np.uint16) << np.uint16(15))
    sub[hit] = (sign | mant)[hit]
    zero[hit] = 0
    return sub, zero


def test_subnormal_inputs_are_zeros_for_page_scores():
    """Closed form of the reading: scores with subnormal queries/bounds equal the scores of the
    inputs with those entries set to zero; normal inputs are untouched (the float32 widening of
    a subnormal bf16 is itself non-zero, so a dropped flush would change low-order bits when
    the partner is large)."""
    rng = np.random.default_rng(77)
    K = randn_bf16(rng, (160, 64))
    bounds = O.page_bounds(K)
    q = randn_bf16(rng, (3, 64), 2.0 ** 100)              # large queries: sub * q is a normal float
    b_sub, b_zero = _with_subnormals(rng, bounds)
    q_sub, q_zero = _with_subnormals(rng, q)
    want = O.head_page_bounds_score(q_zero, b_zero)
    got = O.head_page_bounds_score(q_sub, b_sub)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    # the flush matters: plain IEEE arithmetic on the same bits gives other scores
    plain_q, plain_b = bits_to_f64(q_sub), bits_to_f64(b_sub)
    ieee = np.maximum(plain_q[:, None, :] * plain_b[None, :, 0, :],
                      plain_q[:, None, :] * plain_b[None, :, 1, :]).sum(-1)
    assert np.abs(ieee - want.astype(np.float64)).max() > 0
    # the smallest normal bf16 is not flushed
    one_q = np.zeros((1, 64), np.uint16)
    one_q[0, 5] = 0x3F80                                   # 1.0
    one_b = np.zeros((1, 2, 64), np.uint16)
    one_b[0, :, 5] = 0x0080                                # 2^-126 in both bounds
    assert O.head_page_bounds_score(one_q, one_b)[0, 0] == np.float32(2.0 ** -126)
    one_b[0, :, 5] = 0x007F                                # largest subnormal
    assert O.head_page_bounds_score(one_q, one_b)[0, 0] == 0.0


def test_subnormal_inputs_are_zeros_for_router_logits():
    rng = np.random.default_rng(78)
    h = randn_bf16(rng, (40, 256), 2.0 ** 90)
    Wb = randn_bf16(rng, (8, 256))
    h_sub, h_zero = _with_subnormals(rng, h)
    W_sub, W_zero = _with_subnormals(rng, Wb)
    got, want = O.router_logits(h_sub, W_sub), O.router_logits(h_zero, W_zero)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    assert not np.array_equal(want, O.router_logits(h_zero, Wb))      # the zeros do change it


# --------------------------------------------------------------------------- #
# Router: the fixed float32 order decides the same masks as the exact product
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("dm,G", [(512, 8), (3584, 8), (1024, 16)])
def test_masks_from_float32_router_logits_equal_masks_from_the_exact_product(dm, G):
    """Validity of fixing a float32 summation order for the router: wherever the exact
    (float64) logits separate the kept groups from the dropped ones by more than the float32
    summation error can move them, top-K routing of the chunked float32 logits gives the mask
    of the exact logits.  Bound used: 1e-5 * sum_c |h_c W_gc| per logit (float32 tree and chain
    sums of d_model terms stay well inside it)."""
    rng = np.random.default_rng(dm + G)
    N = 600
    h = randn_bf16(rng, (N, dm))
    Wb = randn_bf16(rng, (G, dm), 1.0 / math.sqrt(dm))
    bias = rng.standard_normal(G).astype(np.float32)
    lg32 = O.router_logits(h, Wb, bias)
    hf, Wf = bits_to_f64(h), bits_to_f64(Wb)
    lg64 = hf @ Wf.T + bias.astype(np.float64)
    slack = 1e-5 * (np.abs(hf) @ np.abs(Wf).T + np.abs(bias)[None, :])      # [N, G]
    assert np.all(np.abs(lg32 - lg64) <= slack)
    kcount = rng.integers(1, G, size=N).astype(np.uint8)                    # 1 .. G-1 kept
    m32 = O.route_mask(lg32, kcount)
    order = np.argsort(-lg64, axis=1, kind="stable")
    m64 = np.zeros(N, dtype=np.uint16)                       # top-K of the exact logits
    for t in range(N):
        for g in order[t, :kcount[t]]:
            m64[t] |= np.uint16(1 << int(g))
    srt = np.take_along_axis(lg64, order, axis=1)
    cut = kcount.astype(np.int64)
    gap = srt[np.arange(N), cut - 1] - srt[np.arange(N), cut]               # margin at the cut
    clear = gap > 2 * slack.max(axis=1)
    assert clear.mean() > 0.9                                               # the check has teeth
    assert np.array_equal(m32[clear], m64[clear])
