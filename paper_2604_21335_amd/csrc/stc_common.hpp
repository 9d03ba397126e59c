// Shared device helpers for the libstc kernels (gfx950 only, 64-wide wavefronts).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "stc_kernels.hpp"

namespace stc {

// Compile-time loop: f(integral_constant<int, I>) for I in [B, E).  Register arrays
// indexed through it have constant indices from the start, so they never land in
// scratch memory.
template <int I>
struct IC {
  static constexpr int value = I;
  constexpr operator int() const { return I; }
};
template <int B, int E, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (B < E) {
    f(IC<B>{});
    static_for<B + 1, E>(f);
  }
}

constexpr int kWave = 64;
constexpr int kPage = 16;

// Page bounds are stored in tiles of 8 pages.  A tile is D/32 rows of 64 units of 16 bytes;
// a unit holds 4 adjacent channels of one page, each as a dword (bf16 minimum in the low
// half, bf16 maximum in the high half).  With CH = D/8 channels per chunk, channel c of page
// pt of the tile sits in row (c % CH) / 4, unit (pt % 4) + 4 * (c / CH) + 32 * (pt / 4),
// dword c % 4.  (The unit number is the lane of the wavefront that scores it.)
__host__ __device__ constexpr int bounds_tile_dwords(int D) { return kBoundsTilePages * D; }
__host__ __device__ constexpr int bounds_tile_unit(int D, int pt, int c) {
  return ((c % (D / 8)) / 4) * 64 + (pt % 4) + 4 * (c / (D / 8)) + 32 * (pt / 4);
}

// bf16 pair in one dword: element 2i in the low half, 2i+1 in the high half.
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// DPP lane move inside a row of 16 lanes (control codes of the gfx9 DPP encoding; lanes
// without a source read 0).
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float x) {
  return __int_as_float(
      __builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, true));
}

// Rows 0,1 and rows 2,3 (of 16 lanes) exchange values: every lane gets the sum of its own
// and the partner row's value.
__device__ __forceinline__ float row_pair_sum(float u) {
  const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(u), __float_as_uint(u), false,
                                                  false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Sum over the 8 lanes that share lane bits 0, 1 and 5 (lane bits 2, 3, 4 count the chunks of
// a page, or the pieces of a token's channel chunk), continuing the balanced tree: chunks
// (0,1)(2,3).. first.  row_ror:n makes lane i read lane i-n of its row, so after the
// two rotations the lanes with bit 2 set hold ((c0+c1)+(c2+c3)) of their row; the row
// exchange adds chunks 4..7.  Valid in lanes with (lane & 0x1c) == 4.
__device__ __forceinline__ float chunk_tree_sum(float u) {
  u += dpp_f32<0x124>(u);  // row_ror:4
  u += dpp_f32<0x128>(u);  // row_ror:8
  return row_pair_sum(u);
}
constexpr int kChunkSumLanes = 4;  // (lane & 0x1c) of the lanes that hold the sum

// Order-preserving map of float bits to unsigned keys (finite inputs).
__device__ __forceinline__ uint32_t float_key(float f) {
  uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Total order on bf16 bit patterns as signed integers: -0 sorts below +0.
__device__ __forceinline__ int bf16_order(uint32_t bits16) {
  int s = (int)(bits16 << 16);
  return s ^ ((s >> 31) & 0x7fffffff);
}
__device__ __forceinline__ uint32_t bf16_unorder(int k) {
  int s = k ^ ((k >> 31) & 0x7fffffff);
  return ((uint32_t)s) >> 16;
}

}  // namespace stc
