"""CPU oracle for decode attention over a Quest-selected, group-packed KV cache.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the HIP
kernels are compared against.  Only tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py may import it; the product package never does and
shares no code with it.  It depends on numpy alone.

What each routine follows (paper = "Sub-Token Routing for KV Cache Compression"):

  page_bounds       Stage I of the paper (Sec. 3.2) delegates token-level
                    reduction to Quest with chunk size 16 (App. C.1, LLM
                    training-config table).  Quest's page summary is the
                    per-page, per-channel min and max of the cached keys.
  router_logits     App. B.1 (the router's architecture): the S group logits of a
                    token are one matrix-vector product of a learned S x d_model
                    matrix with the token's hidden state at the layer input.
  route_mask        Sec. 3.3 "Routing mask": the top-K of the S group logits of
                    a token give a binary mask m[i,j]; App. B.1 gives the fixed
                    per-token K used for VLMs.  Here the count may differ per
                    token (Sec. 3.4 allows K_i to vary by token).
  route_mask_global Sec. 3.4 "global token-group budget" and App. B.1: for a
                    retained sequence of N tokens and nominal budget K the
                    router keeps the M = N*K token-group pairs of largest logit
                    over the whole N x S grid, so the kept count varies by
                    token (0..S).
  token_offsets,    the group-packed store: an encoding of the routed value
  pack_values       vector of Sec. 3.3 (tilde v = m * v per group) that stores
                    kept groups only.
  page_scores,      Quest's query-aware upper bound sum_c max(q_c*min_c,
  select_pages      q_c*max_c) and its top-k pages.
  decode_attention  Sec. 3.3 attention equation: softmax(q K^T / sqrt(d_h))
                    applied to the routed (zero-filled) value matrix; softmax
                    uses q and K only, dropped groups contribute nothing.  An
                    optional tail of recent tokens is attended uncompressed
                    (Sec. 3.4 exempts the tokens of the query region from compression).
  rho_total         Sec. 3.3 "Compression ratio" and App. C.2:
                    rho_total = r * (1 + K/S) / 2.

Readings where the paper is silent:
  * bf16 tensors are passed as uint16 bit patterns; widening to float is exact.
  * min/max of +0 and -0: -0 orders below +0, so the result does not depend on
    the order in which a page is reduced.
  * page score arithmetic: every product is formed in float32 (exact for two
    bf16 factors), the D terms are summed in float32 by a balanced tree over
    adjacent channels (c0+c1), (c2+c3), ... repeated until one value is left.
  * router logits: float32; products of two bf16 factors are exact; the d_model
    terms are summed in chunks of 128 adjacent channels, each chunk by the
    balanced adjacent-pair tree, the chunk sums accumulated left to right; an
    optional float32 bias is added last.  (Masks are integer decisions taken on
    these logits, so the order is part of the definition.)
  * page scores and router logits take a bf16 input that is subnormal (exponent
    field 0, |x| < 2^-126) as a zero: the paper fixes no arithmetic, the library
    forms these products on matrix cores that read such inputs as zero, and a
    key, query or hidden-state channel of that magnitude carries no signal.
    Page bounds, masks and packed values keep subnormal bit patterns as they
    are (they are compared and copied, never multiplied).
  * GQA: one page set per KV head; its score is the max over the query heads of
    that group.  Ties in every top-k go to the lowest index.  A zero score is +0.
  * the selected pages are listed in ascending page order.
  * attention: float64 accumulation, result rounded to float32.
  * the softmax denominator runs over every selected token, whether or not any
    of its value groups were kept.

parity unpinned: the GQA rule (max over the group's heads, or one page list per
query head), the absence of forced "window" pages, keeping recent tokens in an
always-attended uncompressed tail, applying the global budget at cache build
to all cached tokens, and the router as a plain linear map without a query
summary are this build's readings; the paper gives nothing to check them
against.  The arithmetic of each of them is pinned by the tests.
"""
import math

import numpy as np


# --------------------------------------------------------------------------- #
# bf16 helpers
# --------------------------------------------------------------------------- #
def bf16_to_f32(bits):
    """uint16 bf16 bit patterns -> float32 (exact)."""
    bits = np.asarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_to_f32_daz(bits):
    """bf16 bit patterns -> float32 with subnormal inputs read as zero."""
    b = np.asarray(bits, dtype=np.uint16)
    x = bf16_to_f32(b)
    return np.where((b & np.uint16(0x7F80)) == 0, np.float32(0.0), x).astype(np.float32)


def _f32_to_bf16_bits_exact(x):
    """float32 values that are exactly representable in bf16 -> bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    assert not np.any(u & np.uint32(0xFFFF)), "value is not a bf16"
    return (u >> np.uint32(16)).astype(np.uint16)


# --------------------------------------------------------------------------- #
# Budget accounting  (Sec. 3.3 "Compression ratio"; App. C.2)
# --------------------------------------------------------------------------- #
def rho_total(r, K, S):
    """Total retained KV fraction: token keep ratio r times (1 + K/S)/2."""
    return r * (1.0 + K / S) / 2.0


# --------------------------------------------------------------------------- #
# Page bounds (Quest page summary; chunk size 16, App. C.1)
# --------------------------------------------------------------------------- #
def page_bounds(K_bits, P=16):
    """K_bits[N, D] -> bounds[NP, 2, D] (row 0 = min, row 1 = max) as bf16 bits.

    A last page with fewer than P tokens is reduced over its valid tokens only.
    """
    K_bits = np.asarray(K_bits, dtype=np.uint16)
    N, D = K_bits.shape
    NP = (N + P - 1) // P
    out = np.zeros((NP, 2, D), dtype=np.uint16)
    Kf = bf16_to_f32(K_bits)
    for p in range(NP):
        rows = Kf[p * P:min((p + 1) * P, N)]
        rbits = K_bits[p * P:min((p + 1) * P, N)]
        mn = rows.min(axis=0)
        mx = rows.max(axis=0)
        mn_bits = _f32_to_bf16_bits_exact(mn)
        mx_bits = _f32_to_bf16_bits_exact(mx)
        # +0 and -0 compare equal as floats: order -0 below +0.
        has_neg0 = np.any(rbits == 0x8000, axis=0)
        has_pos0 = np.any(rbits == 0x0000, axis=0)
        mn_bits = np.where(mn == 0.0, np.where(has_neg0, 0x8000, 0x0000), mn_bits)
        mx_bits = np.where(mx == 0.0, np.where(has_pos0, 0x0000, 0x8000), mx_bits)
        out[p, 0] = mn_bits
        out[p, 1] = mx_bits
    return out


# --------------------------------------------------------------------------- #
# Routing mask, offsets, packing (Sec. 3.3)
# --------------------------------------------------------------------------- #
def router_logits(h_bits, W_bits, bias=None):
    """h_bits[N, d_model], W_bits[G, d_model] (bf16 bits), bias[G] float32 or None
    -> logits[N, G] float32 = h W^T (+ bias), in the order stated in the header."""
    h = bf16_to_f32_daz(h_bits)                               # [N, dm]
    W = bf16_to_f32_daz(W_bits)                               # [G, dm]
    N, dm = h.shape
    G = W.shape[0]
    assert dm % 128 == 0, "d_model must be a multiple of 128"
    nc = dm // 128
    acc = np.zeros((N, G), dtype=np.float32)
    for c in range(nc):
        sl = slice(c * 128, (c + 1) * 128)
        term = (h[:, None, sl] * W[None, :, sl]).astype(np.float32)   # exact products
        while term.shape[-1] > 1:
            term = (term[..., 0::2] + term[..., 1::2]).astype(np.float32)
        acc = (acc + term[..., 0]).astype(np.float32)
    if bias is not None:
        acc = (acc + np.asarray(bias, dtype=np.float32)[None, :]).astype(np.float32)
    return acc


def route_mask(logits, kcount):
    """logits[N, G] float32, kcount[N] -> mask[N] uint16.

    Bit g of mask[t] is set iff group g is among the kcount[t] largest logits
    of token t; equal logits are ranked by ascending group index.
    """
    a = np.asarray(logits, dtype=np.float32)
    N, G = a.shape
    c = np.broadcast_to(np.asarray(kcount, dtype=np.int64), (N,))
    mask = np.zeros(N, dtype=np.uint16)
    for g in range(G):
        # number of groups that rank ahead of g
        ahead = np.zeros(N, dtype=np.int64)
        for g2 in range(G):
            if g2 == g:
                continue
            wins = a[:, g2] > a[:, g]
            if g2 < g:
                wins = wins | (a[:, g2] == a[:, g])
            ahead += wins
        mask |= ((ahead < c).astype(np.uint16) << np.uint16(g))
    return mask


def route_mask_global(logits, budget):
    """logits[N, G] float32, budget M (0..N*G) -> mask[N] uint16.

    The M token-group pairs of largest logit over the whole grid are kept (paper:
    M = N*K).  Equal logits (IEEE comparison, so -0 == +0) are ranked by
    ascending (token, group), i.e. by flat index t*G + g.
    """
    a = np.asarray(logits, dtype=np.float32)
    N, G = a.shape
    M = int(budget)
    if not 0 <= M <= N * G:
        raise ValueError("budget out of range")
    flat = a.reshape(-1)
    # primary key: logit descending; secondary: flat index ascending
    order = np.lexsort((np.arange(N * G), -flat.astype(np.float64)))
    keep = order[:M]
    mask = np.zeros(N, dtype=np.uint16)
    np.bitwise_or.at(mask, keep // G, (1 << (keep % G)).astype(np.uint16))
    return mask


def popcount(m, G):
    m = np.asarray(m).astype(np.int64)
    n = np.zeros(m.shape, dtype=np.int64)
    for g in range(G):
        n += (m >> g) & 1
    return n


def token_offsets(mask, G):
    """tok_off[0] = 0, tok_off[t+1] = tok_off[t] + popcount(mask[t]) (group units)."""
    cnt = popcount(mask, G)
    off = np.zeros(len(cnt) + 1, dtype=np.uint32)
    run = 0
    for t in range(len(cnt)):
        off[t] = run
        run += int(cnt[t])
    off[len(cnt)] = run
    return off


def pack_values(V_bits, mask, tok_off, G):
    """V_bits[N, D] -> vpacked[tok_off[N], D/G]: kept groups, token order then
    ascending group index; group g of token t goes to slot
    tok_off[t] + (number of kept groups of t below g)."""
    V_bits = np.asarray(V_bits, dtype=np.uint16)
    N, D = V_bits.shape
    gd = D // G
    out = np.zeros((int(tok_off[N]), gd), dtype=np.uint16)
    for t in range(N):
        m = int(mask[t])
        below = 0
        for g in range(G):
            if (m >> g) & 1:
                out[int(tok_off[t]) + below] = V_bits[t, g * gd:(g + 1) * gd]
                below += 1
    return out


# --------------------------------------------------------------------------- #
# Page scores and selection (Quest)
# --------------------------------------------------------------------------- #
def head_page_bounds_score(q_bits, bounds_bits):
    """q_bits[R, D], bounds_bits[NP, 2, D] -> U[R, NP] float32.

    U_h[p] = sum_c max(q_h[c]*mn[p,c], q_h[c]*mx[p,c]); float32 terms summed by
    the balanced adjacent-pair tree.  D must be a power of two.
    """
    q = bf16_to_f32_daz(q_bits)                   # [R, D]
    b = bf16_to_f32_daz(bounds_bits)              # [NP, 2, D]
    mn, mx = b[:, 0, :], b[:, 1, :]
    term = np.maximum(q[:, None, :] * mn[None, :, :],
                      q[:, None, :] * mx[None, :, :]).astype(np.float32)
    D = term.shape[-1]
    assert D & (D - 1) == 0, "D must be a power of two"
    while term.shape[-1] > 1:
        term = (term[..., 0::2] + term[..., 1::2]).astype(np.float32)
    return term[..., 0]


def page_scores(q_bits, bounds_bits):
    """Stream score: max over the R query heads of the group; zero is +0."""
    U = head_page_bounds_score(q_bits, bounds_bits)
    s = U.max(axis=0).astype(np.float32)
    s[s == 0.0] = 0.0                              # -0 -> +0
    return s


def select_pages(score, k):
    """Indices of the min(k, NP) largest scores (ties: lowest index), ascending."""
    score = np.asarray(score, dtype=np.float32)
    NP = score.shape[0]
    k_eff = min(int(k), NP)
    order = sorted(range(NP), key=lambda p: (-float(score[p]), p))
    return np.array(sorted(order[:k_eff]), dtype=np.int32)


# --------------------------------------------------------------------------- #
# Routed attention (Sec. 3.3 attention equation)
# --------------------------------------------------------------------------- #
def decode_attention(q_bits, K_bits, V_bits, mask, page_idx, G, P=16, K_tail=None, V_tail=None):
    """q_bits[R, D]; K_bits, V_bits [N, D]; mask[N]; page_idx ascending or not.

    Tokens attended: every t < N of every listed page, and, when a tail is given
    (K_tail, V_tail [n_tail, D]), every tail token with its full value vector: the
    recent tokens, which the paper exempts from compression (Sec. 3.4, end of the LLM routing
    subsection).  One softmax runs over both sets.  Returns float32 [R, D].
    """
    q = bf16_to_f32(q_bits).astype(np.float64)
    N, D = np.asarray(K_bits).shape
    gd = D // G
    toks = []
    for p in page_idx:
        for t in range(int(p) * P, min((int(p) + 1) * P, N)):
            toks.append(t)
    toks = np.array(toks, dtype=np.int64)
    Kt = bf16_to_f32(np.asarray(K_bits)[toks]).astype(np.float64)      # [T, D]
    Vt = bf16_to_f32(np.asarray(V_bits)[toks]).astype(np.float64)      # [T, D]
    mt = np.asarray(mask)[toks].astype(np.int64)
    if K_tail is not None and len(K_tail):
        Kt = np.concatenate([Kt, bf16_to_f32(np.asarray(K_tail)).astype(np.float64)])
        Vt = np.concatenate([Vt, bf16_to_f32(np.asarray(V_tail)).astype(np.float64)])
        mt = np.concatenate([mt, np.full(len(K_tail), (1 << G) - 1, dtype=np.int64)])
    # routed (zero-filled) values: tilde v = m * v per group
    keep = np.zeros((len(mt), D), dtype=np.float64)
    for g in range(G):
        keep[:, g * gd:(g + 1) * gd] = ((mt >> g) & 1)[:, None]
    Vr = Vt * keep
    R = q.shape[0]
    out = np.zeros((R, D), dtype=np.float64)
    for h in range(R):
        s = (Kt * q[h][None, :]).sum(axis=1) / math.sqrt(D)
        w = np.exp(s - s.max())
        out[h] = (w[:, None] * Vr).sum(axis=0) / w.sum()
    return out.astype(np.float32)


# --------------------------------------------------------------------------- #
# Whole tensors: loops over (batch, kv head) streams
# --------------------------------------------------------------------------- #
def build_page_bounds_all(K_bits, P=16):
    """K_bits[B, Hkv, N, D] -> bounds[B, Hkv, NP, 2, D]."""
    B, Hkv, N, D = K_bits.shape
    NP = (N + P - 1) // P
    out = np.zeros((B, Hkv, NP, 2, D), dtype=np.uint16)
    for b in range(B):
        for h in range(Hkv):
            out[b, h] = page_bounds(K_bits[b, h], P)
    return out


def route_and_pack_all(V_bits, G, logits=None, kcount=None, mask_in=None, global_k=None):
    """V_bits[B, Hkv, N, D] plus either (logits[B,Hkv,N,G], kcount[B,Hkv,N] or
    scalar), or (logits, global_k: per-stream budget N*global_k), or
    mask_in[B,Hkv,N] -> (mask, tok_off[B,Hkv,N+1], list of packed arrays per
    stream in (b, h) order)."""
    B, Hkv, N, D = V_bits.shape
    mask = np.zeros((B, Hkv, N), dtype=np.uint16)
    off = np.zeros((B, Hkv, N + 1), dtype=np.uint32)
    packed = []
    for b in range(B):
        for h in range(Hkv):
            if mask_in is not None:
                m = np.asarray(mask_in[b, h], dtype=np.uint16) & np.uint16((1 << G) - 1)
            elif global_k is not None:
                m = route_mask_global(logits[b, h], N * int(global_k))
            else:
                kc = kcount if np.isscalar(kcount) else kcount[b, h]
                m = route_mask(logits[b, h], kc)
            mask[b, h] = m
            off[b, h] = token_offsets(m, G)
            packed.append(pack_values(V_bits[b, h], m, off[b, h], G))
    return mask, off, packed


def select_pages_all(q_bits, bounds_bits, k):
    """q_bits[B, Hq, D], bounds[B, Hkv, NP, 2, D] ->
    (page_idx[B, Hkv, min(k,NP)] int32, page_score[B, Hkv, NP] float32)."""
    B, Hq, D = q_bits.shape
    _, Hkv, NP = bounds_bits.shape[:3]
    R = Hq // Hkv
    k_eff = min(int(k), NP)
    idx = np.zeros((B, Hkv, k_eff), dtype=np.int32)
    score = np.zeros((B, Hkv, NP), dtype=np.float32)
    for b in range(B):
        for h in range(Hkv):
            score[b, h] = page_scores(q_bits[b, h * R:(h + 1) * R], bounds_bits[b, h])
            idx[b, h] = select_pages(score[b, h], k_eff)
    return idx, score


def select_pages_per_head_all(q_bits, bounds_bits, k):
    """The other reading of Quest under GQA: every query head selects its own pages from its
    own upper-bound score (no maximum over the group).
    q_bits[B, Hq, D], bounds[B, Hkv, NP, 2, D] ->
    (page_idx[B, Hq, min(k,NP)] int32, page_score[B, Hq, NP] float32)."""
    B, Hq, D = q_bits.shape
    _, Hkv, NP = bounds_bits.shape[:3]
    R = Hq // Hkv
    k_eff = min(int(k), NP)
    idx = np.zeros((B, Hq, k_eff), dtype=np.int32)
    score = np.zeros((B, Hq, NP), dtype=np.float32)
    for b in range(B):
        for j in range(Hq):
            score[b, j] = page_scores(q_bits[b, j:j + 1], bounds_bits[b, j // R])
            idx[b, j] = select_pages(score[b, j], k_eff)
    return idx, score


def union_pages(page_idx_group, NP):
    """page_idx_group[R, k]: the page lists of the R query heads of one KV head ->
    (pages[U] ascending, heads[U] uint16): every page some head selected, once, with bit r of
    heads[i] set iff head r selected pages[i].  An encoding that lets the group's heads share
    one pass over the keys and values; entries outside [0, NP) are ignored."""
    masks = np.zeros(NP, dtype=np.uint16)
    for r, row in enumerate(np.asarray(page_idx_group)):
        for p in row:
            if 0 <= int(p) < NP:
                masks[int(p)] |= np.uint16(1 << r)
    pages = np.nonzero(masks)[0].astype(np.int32)
    return pages, masks[pages]


def decode_attention_per_head_all(q_bits, K_bits, V_bits, mask, page_idx, G, P=16):
    """page_idx[B, Hq, k]: query head j attends its own pages of KV head j // (Hq/Hkv).
    -> out[B, Hq, D] float32."""
    B, Hq, D = q_bits.shape
    Hkv = K_bits.shape[1]
    R = Hq // Hkv
    out = np.zeros((B, Hq, D), dtype=np.float32)
    for b in range(B):
        for j in range(Hq):
            out[b, j:j + 1] = decode_attention(q_bits[b, j:j + 1], K_bits[b, j // R],
                                               V_bits[b, j // R], mask[b, j // R],
                                               page_idx[b, j], G, P)
    return out


def decode_attention_all(q_bits, K_bits, V_bits, mask, page_idx, G, P=16, K_tail=None,
                         V_tail=None):
    """-> out[B, Hq, D] float32; query head j belongs to KV head j // (Hq/Hkv).
    K_tail, V_tail [B, Hkv, n_tail, D]: uncompressed recent tokens, always attended."""
    B, Hq, D = q_bits.shape
    Hkv = K_bits.shape[1]
    R = Hq // Hkv
    out = np.zeros((B, Hq, D), dtype=np.float32)
    for b in range(B):
        for h in range(Hkv):
            out[b, h * R:(h + 1) * R] = decode_attention(
                q_bits[b, h * R:(h + 1) * R], K_bits[b, h], V_bits[b, h],
                mask[b, h], page_idx[b, h], G, P,
                None if K_tail is None else K_tail[b, h], None if V_tail is None else V_tail[b, h])
    return out
