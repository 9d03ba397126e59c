"""Seeded synthetic inputs shaped like the paper's workloads.

This module only draws inputs (keys, values, queries, router logits, kept-group
counts, retained-token index sets).  It holds none of the method's arithmetic:
no bounds, masks, offsets, packing, scores, selection or attention.  Both the
HIP path and the CPU oracle are fed the bytes produced here.

Generator: counter based.  Element i of the tensor with tag T under seed S is a
function of (S, T, i) alone (an integer mixer, two uniforms, Box-Muller), so a
tensor can be drawn in pieces, on the CPU or on the GPU.  Transcendental
functions may differ in the last bit between devices, so a tensor is drawn
once, on one device, and copied as bytes to wherever else it is needed.
"""
import math
from dataclasses import dataclass, replace

import torch

_M32 = 0xFFFFFFFF
_MUL = 0x45D9F3B          # odd, < 2^31: 32-bit value times it stays below 2^63

# tensor tags
TAG_K, TAG_V, TAG_LOGITS, TAG_KCOUNT, TAG_MASKBITS, TAG_MASKFIX = 1, 2, 3, 4, 5, 6
TAG_OUTLIER, TAG_RETAIN, TAG_Q0 = 7, 8, 1000


def _mix32(x):
    """Integer mixer on int64 tensors holding 32-bit values."""
    x = ((x >> 16) ^ x) * _MUL & _M32
    x = ((x >> 16) ^ x) * _MUL & _M32
    x = (x >> 16) ^ x
    return x


def _hash2(seed, tag, idx):
    """Two independent 32-bit words per element index (int64 tensor)."""
    lo = idx & _M32
    hi = (idx >> 32) & _M32
    key = _mix32(torch.full_like(lo, (seed * 0x9E3779B1 + tag * 0x85EBCA77 + 0x1234567) & _M32))
    h = _mix32(lo ^ key)
    h = _mix32(h ^ hi ^ 0x5BD1E995)
    a = _mix32(h ^ 0x2545F491)
    b = _mix32(h ^ 0x68E31DA4)
    return a, b


def uniform(seed, tag, n, device="cpu", offset=0):
    """n uniforms in [0, 1), float64."""
    idx = torch.arange(offset, offset + n, dtype=torch.int64, device=device)
    a, b = _hash2(seed, tag, idx)
    return (a.to(torch.float64) * 4294967296.0 + b.to(torch.float64)) / 18446744073709551616.0


def normal(seed, tag, n, device="cpu", offset=0):
    """n standard normals, float32 (Box-Muller on two hashed uniforms)."""
    idx = torch.arange(offset, offset + n, dtype=torch.int64, device=device)
    a, b = _hash2(seed, tag, idx)
    u1 = (a.to(torch.float32) + 1.0) * (1.0 / 4294967296.0)
    u1 = torch.clamp(u1, min=2.0 ** -32, max=1.0)
    u2 = b.to(torch.float32) * (1.0 / 4294967296.0)
    return torch.sqrt(-2.0 * torch.log(u1)) * torch.cos((2.0 * math.pi) * u2)


def normal_tensor(seed, tag, shape, device="cpu", dtype=torch.float32, chunk=1 << 24):
    n = 1
    for s in shape:
        n *= int(s)
    out = torch.empty(n, dtype=dtype, device=device)
    for o in range(0, n, chunk):
        m = min(chunk, n - o)
        out[o:o + m] = normal(seed, tag, m, device, o).to(dtype)
    return out.view(*shape)


def counts_from_pmf(seed, tag, shape, pmf, device="cpu"):
    """Integers 1..len(pmf) drawn with the given probabilities (inverse CDF)."""
    n = 1
    for s in shape:
        n *= int(s)
    tot = float(sum(pmf))
    cdf, run = [], 0.0
    for p in pmf[:-1]:
        run += p / tot
        cdf.append(run)
    edges = torch.tensor(cdf, dtype=torch.float64, device=device)
    u = uniform(seed, tag, n, device)
    return (torch.bucketize(u, edges, right=True) + 1).to(torch.uint8).view(*shape)


@dataclass(frozen=True)
class Workload:
    """One synthetic cache shape.  k_pages = Quest token budget / page size."""
    name: str
    B: int
    Hq: int
    Hkv: int
    D: int
    N: int
    G: int
    k_pages: int
    seed: int
    routing: str            # "bernoulli" | "uniform" | "geometric" | "binomial" | "vlm"
    outliers: bool = False  # four K channels per KV head scaled by 8
    layers: int = 1         # independent caches walked per decode step
    steps: int = 1          # decode queries over one static cache
    P: int = 16
    # VLM prefix only: source cache and how much of it a token-level method keeps
    n_visual: int = 0
    n_text: int = 0
    visual_keep: float = 1.0
    visual_groups: int = 0

    @property
    def NP(self):
        return (self.N + self.P - 1) // self.P

    @property
    def R(self):
        return self.Hq // self.Hkv

    @property
    def streams(self):
        return self.B * self.Hkv


def _vlm_n(nv, nt, keep):
    return int(round(nv * keep)) + nt


WORKLOADS = {
    # 1 layer, 8 MHA heads of 64, 1024 tokens, top 16 pages, G = 4, ~50 % random keep-mask
    "tiny": Workload("tiny", B=1, Hq=8, Hkv=8, D=64, N=1024, G=4, k_pages=16, seed=0,
                     routing="bernoulli"),
    # LLaMA-2-7B-shaped layer: 32 MHA heads of 128, batch 8, context 4096, budget 1024 tokens
    "llama2_7b_4k": Workload("llama2_7b_4k", B=8, Hq=32, Hkv=32, D=128, N=4096, G=8, k_pages=64,
                             seed=1, routing="uniform", outliers=True),
    # Qwen2.5-7B-shaped layer: 28 query / 4 KV heads, batch 16, context 32768, budget 2048 tokens
    "qwen25_7b_32k": Workload("qwen25_7b_32k", B=16, Hq=28, Hkv=4, D=128, N=32768, G=8,
                              k_pages=128, seed=2, routing="geometric", outliers=True),
    # LLaVA-1.5-7B-shaped prefix: 576 visual + 64 text tokens, 25 % of the visual tokens kept
    "llava15_7b_prefix": Workload("llava15_7b_prefix", B=64, Hq=32, Hkv=32, D=128,
                                  N=_vlm_n(576, 64, 0.25), G=8,
                                  k_pages=(_vlm_n(576, 64, 0.25) + 15) // 16, seed=3, routing="vlm",
                                  steps=128, n_visual=576, n_text=64, visual_keep=0.25,
                                  visual_groups=3),
    # long context: Qwen2.5-7B shapes, batch 1, context 131072, budget 4096 tokens, 28 layers
    "qwen25_7b_128k": Workload("qwen25_7b_128k", B=1, Hq=28, Hkv=4, D=128, N=131072, G=16,
                               k_pages=256, seed=4, routing="binomial", outliers=True, layers=28),
}
ORDER = ["tiny", "llama2_7b_4k", "qwen25_7b_32k", "llava15_7b_prefix", "qwen25_7b_128k"]


def shrink(w, **kw):
    """A smaller workload of the same structure (for parity tests)."""
    return replace(w, **kw)


def _pmf(w):
    if w.routing == "uniform":                      # counts uniform on 1..G
        return [1.0] * w.G
    if w.routing == "geometric":                    # P(c) ~ 0.91^(c-1): mean ~4 of 8
        return [0.91 ** c for c in range(w.G)]
    if w.routing == "binomial":                     # 1 + Binomial(G-1, 0.2): mean 4 of 16
        n, p = w.G - 1, 0.2
        return [math.comb(n, c) * p ** c * (1 - p) ** (n - c) for c in range(n + 1)]
    raise ValueError(w.routing)


def outlier_scale(w, layer, device):
    """[Hkv, D] multiplier: four channels per KV head (from the seed) are 8, others 1."""
    u = uniform(w.seed, TAG_OUTLIER + 100 * layer, w.Hkv * w.D, device).view(w.Hkv, w.D)
    idx = torch.argsort(u, dim=1)[:, :4]
    scale = torch.ones(w.Hkv, w.D, dtype=torch.float32, device=device)
    scale.scatter_(1, idx, 8.0)
    return scale


def make_cache_inputs(w, device="cpu", layer=0):
    """Inputs of cache construction for one layer's cache.

    Returns a dict of tensors on `device`:
      K, V            [B, Hkv, N, D] bfloat16
      logits          [B, Hkv, N, G] float32 (routing by top-k), or None
      kcount          [B, Hkv, N] uint8, or None
      mask_in         [B, Hkv, N] int16 holding uint16 bit masks ("bernoulli" only), or None
    For the VLM prefix, K/V are the source cache [B, Hkv, n_visual+n_text, D],
      token_idx       [B, N] int32 lists the retained tokens (visual ascending, then text),
    and logits / kcount are per retained token (N of them), in that order.
    """
    tagoff = 100 * layer
    n_src = w.n_visual + w.n_text if w.routing == "vlm" else w.N
    shape = (w.B, w.Hkv, n_src, w.D)
    K = normal_tensor(w.seed, TAG_K + tagoff, shape, device)
    if w.outliers:
        K = K * outlier_scale(w, layer, device)[None, :, None, :]
    K = K.to(torch.bfloat16)
    V = normal_tensor(w.seed, TAG_V + tagoff, shape, device).to(torch.bfloat16)
    out = {"K": K, "V": V, "logits": None, "kcount": None, "mask_in": None, "token_idx": None}
    if w.routing == "bernoulli":
        n = w.B * w.Hkv * w.N
        bits = uniform(w.seed, TAG_MASKBITS + tagoff, n * w.G, device).view(n, w.G) < 0.5
        m = (bits.to(torch.int64) << torch.arange(w.G, device=device)).sum(dim=1)
        fix = (uniform(w.seed, TAG_MASKFIX + tagoff, n, device) * w.G).to(torch.int64)
        m = torch.where(m == 0, torch.ones_like(m) << fix, m)       # at least one group
        out["mask_in"] = m.to(torch.int16).view(w.B, w.Hkv, w.N)
        return out
    out["logits"] = normal_tensor(w.seed, TAG_LOGITS + tagoff, (w.B, w.Hkv, w.N, w.G), device)
    if w.routing == "vlm":
        nk = int(round(w.n_visual * w.visual_keep))
        u = uniform(w.seed, TAG_RETAIN + tagoff, w.B * w.n_visual, device).view(w.B, w.n_visual)
        vis = torch.sort(torch.argsort(u, dim=1)[:, :nk], dim=1).values
        txt = torch.arange(w.n_visual, w.n_visual + w.n_text, device=device)[None].expand(w.B, -1)
        out["token_idx"] = torch.cat([vis, txt], dim=1).to(torch.int32).contiguous()
        kc = torch.cat([torch.full((nk,), w.visual_groups), torch.full((w.n_text,), w.G)])
        out["kcount"] = kc.to(torch.uint8).to(device)[None, None].expand(w.B, w.Hkv, -1).contiguous()
    else:
        out["kcount"] = counts_from_pmf(w.seed, TAG_KCOUNT + tagoff, (w.B, w.Hkv, w.N), _pmf(w),
                                        device)
    return out


def make_query(w, step=0, device="cpu", layer=0, scale=1.0):
    """Decode query [B, Hq, D] bfloat16 for decode step `step`."""
    q = normal_tensor(w.seed, TAG_Q0 + step + 100000 * layer, (w.B, w.Hq, w.D), device)
    return (q * scale).to(torch.bfloat16)


def bf16_bits(t):
    """bfloat16 tensor -> numpy uint16 bit patterns on the host."""
    import numpy as np
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def u16_numpy(t):
    """int16-typed tensor holding uint16 values -> numpy uint16 on the host."""
    import numpy as np
    return t.contiguous().cpu().numpy().view(np.uint16)
