// Device helpers shared by the cache-construction kernels and the kernel that appends tokens
// to a built cache.
#pragma once
#include "stc_common.hpp"

namespace stc {

// The G logits of one token (16-byte loads when G is a multiple of 4: the row is then
// 16-byte aligned).
template <int G>
__device__ __forceinline__ void load_token_logits(const float* __restrict__ lp, float (&a)[G]) {
  if constexpr ((G & 3) == 0) {
#pragma unroll
    for (int q = 0; q < G / 4; ++q) {
      const float4 v = *(const float4*)(lp + 4 * q);
      a[4 * q] = v.x, a[4 * q + 1] = v.y, a[4 * q + 2] = v.z, a[4 * q + 3] = v.w;
    }
  } else {
#pragma unroll
    for (int g = 0; g < G; ++g) a[g] = lp[g];
  }
}

// Routing mask of one token: bit g set iff group g is among the c largest of its G logits
// (equal logits: the lower group first).
template <int G>
__device__ __forceinline__ uint32_t rank_mask_g(const float* __restrict__ lp, int c) {
  float a[G];
  load_token_logits<G>(lp, a);
  uint32_t m = 0;
#pragma unroll
  for (int g = 0; g < G; ++g) {
    int ahead = 0;  // groups ranked before g: larger logit, or equal with lower index
#pragma unroll
    for (int g2 = 0; g2 < G; ++g2)
      if (g2 != g) ahead += (a[g2] > a[g]) || (g2 < g && a[g2] == a[g]);
    if (ahead < c) m |= 1u << g;
  }
  return m;
}

// The same for a group count known at run time (a power of two up to 16, uniform over the
// launch: the switch is a scalar branch).
__device__ __forceinline__ uint32_t rank_mask(const float* __restrict__ lp, int c, int G) {
  switch (G) {
    case 1: return rank_mask_g<1>(lp, c);
    case 2: return rank_mask_g<2>(lp, c);
    case 4: return rank_mask_g<4>(lp, c);
    case 8: return rank_mask_g<8>(lp, c);
    case 16: return rank_mask_g<16>(lp, c);
    default: return 0u;
  }
}

// Minimum and maximum of 8 adjacent channels over `ntok` token rows (row stride D*2 bytes,
// `row` points at the 16-byte piece of the first row); w[i] = min | max << 16 as bf16 bits,
// -0 ordered below +0.  ntok <= 0 gives zeros.
template <int D>
__device__ __forceinline__ void page_bounds_words(const uint4* row, int ntok,
                                                  uint32_t (&w)[8]) {
  constexpr int LPP = D / 8;
  int mn[8], mx[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    mn[i] = 0x7fffffff;
    mx[i] = (int)0x80000000;
  }
#pragma unroll 4
  for (int t = 0; t < ntok; ++t, row += LPP) {
    const uint4 v = *row;
    const uint32_t x[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int a = bf16_order(x[i] & 0xffffu);
      const int b = bf16_order(x[i] >> 16);
      mn[2 * i] = min(mn[2 * i], a);
      mx[2 * i] = max(mx[2 * i], a);
      mn[2 * i + 1] = min(mn[2 * i + 1], b);
      mx[2 * i + 1] = max(mx[2 * i + 1], b);
    }
  }
#pragma unroll
  for (int i = 0; i < 8; ++i)
    w[i] = ntok > 0 ? (bf16_unorder(mn[i]) | (bf16_unorder(mx[i]) << 16)) : 0u;
}

// The two 16-byte units of channels 8*sub .. 8*sub+7 of page `page` in the tiled bounds layout.
template <int D>
__device__ __forceinline__ void store_bounds_units(uint4* __restrict__ stream_tiles, int page,
                                                   int sub, const uint32_t (&w)[8]) {
  uint4* tile = stream_tiles + (size_t)(page / kBoundsTilePages) * (bounds_tile_dwords(D) / 4);
  const int pt = page % kBoundsTilePages;
  tile[bounds_tile_unit(D, pt, 8 * sub)] = make_uint4(w[0], w[1], w[2], w[3]);
  tile[bounds_tile_unit(D, pt, 8 * sub + 4)] = make_uint4(w[4], w[5], w[6], w[7]);
}

}  // namespace stc
