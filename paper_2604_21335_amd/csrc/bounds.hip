// Quest page summary: per-page, per-channel min and max of the cached keys
// (token-level stage of the paper, Sec. 3.2; chunk size 16 from App. C.1).
#include "build_helpers.hpp"
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
                                                     uint4* __restrict__ bounds, int N, int NP,
                                                     int Ncap) {
  constexpr int LPP = D / 8;  // threads per page
  const int stream = blockIdx.y;
  const int sub = threadIdx.x % LPP;
  const int page = blockIdx.x * (256 / LPP) + threadIdx.x / LPP;
  const int ntiles = (NP + kBoundsTilePages - 1) / kBoundsTilePages;
  if (page >= ntiles * kBoundsTilePages) return;
  const int t0 = page * kPage;
  const int t1 = min(t0 + kPage, N);  // t1 <= t0 for a padding page: zeros
  uint32_t w[8];  // per channel: minimum | maximum << 16
  page_bounds_words<D>(K + ((size_t)stream * Ncap + t0) * LPP + sub, t1 - t0, w);
  store_bounds_units<D>(
      bounds + (size_t)stream * bounds_tiles(Ncap) * (bounds_tile_dwords(D) / 4), page, sub, w);
}

int launch_bounds(const stc_shape_t& s, const void* K, void* bounds, hipStream_t st) {
  const int NP = (s.N + kPage - 1) / kPage;
  const int streams = s.B * s.Hkv;
  const int pages_per_block = 256 / (s.D / 8);
  const int pages = (NP + kBoundsTilePages - 1) / kBoundsTilePages * kBoundsTilePages;
  dim3 grid((pages + pages_per_block - 1) / pages_per_block, streams);
  if (s.D == 128)
    bounds_kernel<128><<<grid, 256, 0, st>>>((const uint4*)K, (uint4*)bounds, s.N, NP,
                                          token_cap(s));
  else
    bounds_kernel<64><<<grid, 256, 0, st>>>((const uint4*)K, (uint4*)bounds, s.N, NP,
                                         token_cap(s));
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

}  // namespace stc
