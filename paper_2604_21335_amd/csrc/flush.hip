// Appending tokens to a built cache: the oldest n tokens of the uncompressed tail become
// tokens N .. N+n-1 of the compressed cache.  Their keys are copied, their values are routed
// (given masks, or per-token top-K of given logits) and packed behind the stream's packed
// store, the offsets are continued from tok_off[N], and the bounds of every page that holds
// one of them are recomputed (the first such page may already hold older tokens).  The
// result is, bit for bit, the cache that construction from scratch over all N+n tokens gives.
// The rows that stay in the tail are then moved to its front.
#include "build_helpers.hpp"
#include "stc_common.hpp"
#include "stc_kernels.hpp"

namespace stc {

// One 256-thread workgroup per stream (cache construction, not the decode path).
template <int D>
__global__ __launch_bounds__(256) void flush_tail_kernel(
    uint4* K_tail, uint4* V_tail, int n, int n_tail, int tail_cap,
    int mode, const float* __restrict__ logits, const uint8_t* __restrict__ kcount, int fixed_k,
    const uint16_t* __restrict__ mask_in, uint4* K, uint4* __restrict__ bounds,
    uint16_t* __restrict__ mask, uint32_t* __restrict__ tok_off, uint4* __restrict__ vpacked,
    int32_t* dev_status, int N, int Ncap, int G, long long cap) {
  constexpr int PPT = D / 8;  // 16-byte pieces per token row
  __shared__ int waves[4];
  __shared__ uint32_t s_off[256];
  __shared__ uint32_t s_mask[256];
  const int stream = blockIdx.x;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  uint4* Ks = K + (size_t)stream * Ncap * PPT;
  uint4* Kt = K_tail + (size_t)stream * tail_cap * PPT;
  uint4* Vt = V_tail + (size_t)stream * tail_cap * PPT;
  uint16_t* mk = mask + (size_t)stream * Ncap;
  uint32_t* off = tok_off + (size_t)stream * (Ncap + 1);
  const int ppg = PPT / G;  // 16-byte pieces per group
  uint4* dst = vpacked + (size_t)stream * (size_t)cap * ppg;

  uint32_t carry = off[N];  // kept groups of the stream so far = offset of token N
  for (int i0 = 0; i0 < n; i0 += 256) {
    const int i = i0 + tid;
    uint32_t m = 0;
    if (i < n) {
      const size_t tok = (size_t)stream * n + i;  // dense per-token inputs of the new tokens
      if (mode == STC_ROUTE_MASK) {
        m = mask_in[tok] & ((1u << G) - 1u);
      } else {
        const int c = kcount ? (int)kcount[tok] : fixed_k;
        m = rank_mask(logits + tok * G, min(c, G), G);
      }
      mk[N + i] = (uint16_t)m;
    }
    // exclusive scan of the kept-group counts over the tile
    int inc = __popc(m);
    for (int d = 1; d < 64; d <<= 1) {
      const int o = __shfl_up(inc, d);
      if (lane >= d) inc += o;
    }
    if (lane == 63) waves[wave] = inc;
    __syncthreads();
    uint32_t base = carry, tot = 0;
    for (int w = 0; w < 4; ++w) {
      if (w < wave) base += waves[w];
      tot += waves[w];
    }
    const uint32_t my_off = base + inc - __popc(m);
    if (i < n) off[N + i + 1] = my_off + __popc(m);
    s_off[tid] = my_off;
    s_mask[tid] = m;
    __syncthreads();
    // key rows and kept value groups of the tile, 16 bytes per work item
    const int ntok = min(256, n - i0);
    for (int e = tid; e < ntok * PPT; e += 256) {
      const int tk = e / PPT, pc = e % PPT;
      Ks[(size_t)(N + i0 + tk) * PPT + pc] = Kt[(size_t)(i0 + tk) * PPT + pc];
      const int g = pc / ppg, within = pc % ppg;
      const uint32_t mm = s_mask[tk];
      if ((mm >> g) & 1u) {
        const long long slot = (long long)s_off[tk] + __popc(mm & ((1u << g) - 1u));
        if (slot < cap) dst[slot * ppg + within] = Vt[(size_t)(i0 + tk) * PPT + pc];
      }
    }
    carry += tot;
    __syncthreads();
  }
  if (tid == 0 && dev_status && (long long)carry > cap) *dev_status = 1;

  // bounds of the pages that hold a new token, from the key rows now in the cache
  __threadfence_block();
  __syncthreads();
  const int N1 = N + n;
  const int p_first = N / kPage, p_last = (N1 - 1) / kPage;
  uint4* tiles = bounds + (size_t)stream * bounds_tiles(Ncap) * (bounds_tile_dwords(D) / 4);
  for (int w = tid; w < (p_last - p_first + 1) * PPT; w += 256) {
    const int page = p_first + w / PPT, sub = w % PPT;
    const int t0 = page * kPage, t1 = min(t0 + kPage, N1);
    uint32_t words[8];
    page_bounds_words<D>(Ks + (size_t)t0 * PPT + sub, t1 - t0, words);
    store_bounds_units<D>(tiles, page, sub, words);
  }
  // pages of the last tile past the last token hold zeros (they may never have been written)
  const int pad0 = p_last + 1, pad1 = (p_last / kBoundsTilePages + 1) * kBoundsTilePages;
  for (int w = tid; w < (pad1 - pad0) * PPT; w += 256) {
    const uint32_t zeros[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    store_bounds_units<D>(tiles, pad0 + w / PPT, w % PPT, zeros);
  }

  // The rows that stay in the tail (n .. n_tail-1) move to its front, 16 bytes per work item.
  // Source and destination overlap, so the rows go in ascending chunks, each read completely
  // before any of it is written: a chunk's destination holds sources of this and of earlier
  // chunks only (the rows moved into the cache above have been read: barrier above).
  constexpr int U = 4;
  const int total = (n_tail - n) * PPT, shift = n * PPT;
  for (int base = 0; base < total; base += 256 * U) {
    uint4 kv[U], vv[U];
#pragma unroll
    for (int j = 0; j < U; ++j) {
      const int e = base + j * 256 + tid;
      if (e < total) kv[j] = Kt[e + shift], vv[j] = Vt[e + shift];
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < U; ++j) {
      const int e = base + j * 256 + tid;
      if (e < total) Kt[e] = kv[j], Vt[e] = vv[j];
    }
    __syncthreads();
  }
}

int launch_flush_tail(const stc_shape_t& s, void* K_tail, void* V_tail, int n, int n_tail,
                      int tail_cap, int mode, const float* logits, const uint8_t* kcount,
                      int fixed_k, const uint16_t* mask_in, void* K, void* bounds, uint16_t* mask,
                      uint32_t* tok_off, void* vpacked, int32_t* dev_status, hipStream_t st) {
  const int streams = s.B * s.Hkv;
#define STC_FLUSH(DD)                                                                           \
  flush_tail_kernel<DD><<<streams, 256, 0, st>>>(                                               \
      (uint4*)K_tail, (uint4*)V_tail, n, n_tail, tail_cap, mode, logits, kcount, fixed_k,   \
      mask_in, (uint4*)K, (uint4*)bounds, mask, tok_off, (uint4*)vpacked, dev_status, s.N,      \
      token_cap(s), s.G, (long long)s.v_cap_groups)
  if (s.D == 128)
    STC_FLUSH(128);
  else
    STC_FLUSH(64);
#undef STC_FLUSH
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

}  // namespace stc
