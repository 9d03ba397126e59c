// Quest page summary: per-page, per-channel min and max of the cached keys
// (token-level stage of the paper, Sec. 3.2; chunk size 16 from App. C.1).
#include "stc_common.hpp"
#include "stc_kernels.hpp"

namespace stc {

// One thread owns 8 adjacent channels (one 128-bit load per token row) of one
// page and walks the page's tokens.  D/8 neighbouring threads cover a row, so a
// wavefront reads 64/(D/8) whole rows of 2*D bytes per load instruction.  The result goes
// into the tiled layout the scoring kernel reads (two 16-byte units per thread); pages
// past the last one of a stream's last tile are written as zeros.
template <int D>
__global__ __launch_bounds__(256) void bounds_kernel(const uint4* __restrict__ K,
                                                     uint4* __restrict__ bounds, int N, int NP) {
  constexpr int LPP = D / 8;  // threads per page
  const int stream = blockIdx.y;
  const int sub = threadIdx.x % LPP;
  const int page = blockIdx.x * (256 / LPP) + threadIdx.x / LPP;
  const int ntiles = (NP + kBoundsTilePages - 1) / kBoundsTilePages;
  if (page >= ntiles * kBoundsTilePages) return;
  const int t0 = page * kPage;
  const int t1 = min(t0 + kPage, N);  // t1 <= t0 for a padding page
  const uint4* row = K + ((size_t)stream * N + t0) * LPP + sub;
  int mn[8], mx[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    mn[i] = 0x7fffffff;
    mx[i] = (int)0x80000000;
  }
#pragma unroll 4
  for (int t = t0; t < t1; ++t, row += LPP) {
    const uint4 v = *row;
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int a = bf16_order(w[i] & 0xffffu);
      const int b = bf16_order(w[i] >> 16);
      mn[2 * i] = min(mn[2 * i], a);
      mx[2 * i] = max(mx[2 * i], a);
      mn[2 * i + 1] = min(mn[2 * i + 1], b);
      mx[2 * i + 1] = max(mx[2 * i + 1], b);
    }
  }
  uint32_t w[8];  // per channel: minimum | maximum << 16
#pragma unroll
  for (int i = 0; i < 8; ++i)
    w[i] = page < NP ? (bf16_unorder(mn[i]) | (bf16_unorder(mx[i]) << 16)) : 0u;
  uint4* tile = bounds + ((size_t)stream * ntiles + page / kBoundsTilePages) *
                             (bounds_tile_dwords(D) / 4);
  const int pt = page % kBoundsTilePages;
  tile[bounds_tile_unit(D, pt, 8 * sub)] = make_uint4(w[0], w[1], w[2], w[3]);
  tile[bounds_tile_unit(D, pt, 8 * sub + 4)] = make_uint4(w[4], w[5], w[6], w[7]);
}

int launch_bounds(const stc_shape_t& s, const void* K, void* bounds, hipStream_t st) {
  const int NP = (s.N + kPage - 1) / kPage;
  const int streams = s.B * s.Hkv;
  const int pages_per_block = 256 / (s.D / 8);
  const int pages = (NP + kBoundsTilePages - 1) / kBoundsTilePages * kBoundsTilePages;
  dim3 grid((pages + pages_per_block - 1) / pages_per_block, streams);
  if (s.D == 128)
    bounds_kernel<128><<<grid, 256, 0, st>>>((const uint4*)K, (uint4*)bounds, s.N, NP);
  else
    bounds_kernel<64><<<grid, 256, 0, st>>>((const uint4*)K, (uint4*)bounds, s.N, NP);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

}  // namespace stc
