// Sub-token value-group routing at cache-build time (paper Sec. 3.3): top-k
// routing mask per token (or, for the LLM setting of Sec. 3.4 / App. B.1, the N*K
// best token-group pairs of the whole stream), per-token offsets into the
// group-packed store, and the packed copy of the kept value groups.
#include "build_helpers.hpp"
#include "stc_common.hpp"
#include "stc_kernels.hpp"

namespace stc {

constexpr int kChunk = 256;  // tokens per workgroup in the route / pack kernels

__device__ __forceinline__ int block_sum_256(int v, int* lds4) {
  // sum over a 256-thread block; every thread gets the total
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d);
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) lds4[wave] = v;
  __syncthreads();
  const int tot = lds4[0] + lds4[1] + lds4[2] + lds4[3];
  __syncthreads();
  return tot;
}

// Exclusive prefix sum over a 256-thread block (in thread order).
__device__ __forceinline__ int block_exscan_256(int v, int* lds4, int* total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int inc = v;
  for (int d = 1; d < 64; d <<= 1) {
    const int o = __shfl_up(inc, d);
    if (lane >= d) inc += o;
  }
  if (lane == 63) lds4[wave] = inc;
  __syncthreads();
  int base = 0;
  for (int w = 0; w < wave; ++w) base += lds4[w];
  if (total) *total = lds4[0] + lds4[1] + lds4[2] + lds4[3];
  __syncthreads();
  return base + inc - v;
}

// Step 1: routing mask of every token and the number of kept groups per chunk.
__global__ __launch_bounds__(kChunk) void route_mask_kernel(
    int mode, const float* __restrict__ logits, const uint8_t* __restrict__ kcount, int fixed_k,
    const uint16_t* mask_in, uint16_t* mask, uint32_t* __restrict__ chunk_sum, int N, int G,
    int nchunks, int Ncap, int mask_in_stride) {
  __shared__ int red[4];
  const int stream = blockIdx.y;
  const int t = blockIdx.x * kChunk + threadIdx.x;
  uint32_t m = 0;
  if (t < N) {
    const size_t tok = (size_t)stream * N + t;  // dense inputs: logits, kcount
    if (mode == STC_ROUTE_MASK) {
      m = mask_in[(size_t)stream * mask_in_stride + t] & ((1u << G) - 1u);
    } else {
      int c = kcount ? (int)kcount[tok] : fixed_k;
      m = rank_mask(logits + tok * G, min(c, G), G);
    }
    mask[(size_t)stream * Ncap + t] = (uint16_t)m;
  }
  const int tot = block_sum_256(__popc(m), red);
  if (threadIdx.x == 0) chunk_sum[(size_t)stream * nchunks + blockIdx.x] = (uint32_t)tot;
}

// ---------------------------------------------------------------------------
// Global token-group budget (Sec. 3.4; App. B.1: M = N*K of the N x S pairs): one
// 1024-thread workgroup per stream finds the key of the M-th largest logit by a radix
// select over the stream's N*G logits (12 + 10 + 10 bits; the wide first digit spreads
// logits that share sign and exponent over many bins), then walks the tokens in order and
// keeps every pair above that key plus the first `remaining` pairs equal to it.
// ---------------------------------------------------------------------------
constexpr int kGlobalThreads = 1024;
constexpr int kGlobalBins = 4096;

// Order-preserving key of a finite float with -0 and +0 mapped to one key.
__device__ __forceinline__ uint32_t logit_key(float f) {
  uint32_t u = __float_as_uint(f);
  if (u == 0x80000000u) u = 0u;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Exclusive prefix sum over a 1024-thread block (thread order); *total = block sum.
__device__ __forceinline__ uint32_t block_exscan_1024(uint32_t v, uint32_t* lds16,
                                                      uint32_t* total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  uint32_t inc = v;
  for (int d = 1; d < 64; d <<= 1) {
    const uint32_t o = __shfl_up(inc, d);
    if (lane >= d) inc += o;
  }
  if (lane == 63) lds16[wave] = inc;
  __syncthreads();
  uint32_t base = 0, tot = 0;
  for (int w = 0; w < kGlobalThreads / 64; ++w) {
    if (w < wave) base += lds16[w];
    tot += lds16[w];
  }
  *total = tot;
  __syncthreads();
  return base + inc - v;
}

__global__ __launch_bounds__(kGlobalThreads) void route_global_kernel(
    const float* __restrict__ logits, uint16_t* __restrict__ mask, int N, int G,
    uint32_t budget, int Ncap) {
  __shared__ uint32_t hist[kGlobalBins];
  __shared__ uint32_t waves[kGlobalThreads / 64];
  __shared__ uint32_t s_prefix, s_remaining;
  const int stream = blockIdx.x;
  const int tid = threadIdx.x;
  const uint32_t n = (uint32_t)N * (uint32_t)G;
  const float* a = logits + (size_t)stream * n;
  uint16_t* mk = mask + (size_t)stream * Ncap;

  uint32_t prefix = 0, decided = 0, remaining = budget;
  if (budget > 0) {
    // digits from the top: bits 31..20, 19..10, 9..0
    for (int pass = 0; pass < 3; ++pass) {
      const int shift = pass == 0 ? 20 : (pass == 1 ? 10 : 0);
      const uint32_t bins = pass == 0 ? 4096u : 1024u;
      for (uint32_t i = tid; i < kGlobalBins; i += kGlobalThreads) hist[i] = 0;
      __syncthreads();
      for (uint32_t i = tid; i < n; i += kGlobalThreads) {
        const uint32_t key = logit_key(a[i]);
        if ((key & decided) == prefix) atomicAdd(&hist[(key >> shift) & (bins - 1)], 1u);
      }
      __syncthreads();
      // thread t owns the 4 adjacent digits 4095-4t .. 4092-4t (descending order)
      uint32_t c[4], own = 0;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint32_t d = kGlobalBins - 1 - (4 * tid + j);
        c[j] = d < bins ? hist[d] : 0u;
        own += c[j];
      }
      uint32_t tot;
      uint32_t above = block_exscan_1024(own, waves, &tot);  // pairs with a larger digit
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (above < remaining && remaining <= above + c[j]) {
          s_prefix = prefix | ((uint32_t)(kGlobalBins - 1 - (4 * tid + j)) << shift);
          s_remaining = remaining - above;
        }
        above += c[j];
      }
      __syncthreads();
      prefix = s_prefix;
      remaining = s_remaining;
      decided |= (bins - 1) << shift;
      __syncthreads();
    }
  }
  // prefix = key of the budget-th largest logit; `remaining` of the pairs equal to it are
  // kept, lowest (token, group) first.  budget == 0 keeps nothing.
  uint32_t carry = 0;  // pairs equal to the key in earlier tiles
  for (int t0 = 0; t0 < N; t0 += kGlobalThreads) {
    const int t = t0 + tid;
    uint32_t key[16];
    uint32_t eq = 0;
#pragma unroll
    for (int g = 0; g < 16; ++g) {
      key[g] = (g < G && t < N) ? logit_key(a[(size_t)t * G + g]) : 0u;
      eq += (g < G && t < N && budget > 0) && key[g] == prefix;
    }
    uint32_t tot;
    uint32_t e = carry + block_exscan_1024(eq, waves, &tot);
    uint32_t m = 0;
    if (budget > 0) {
#pragma unroll
      for (int g = 0; g < 16; ++g) {
        if (g < G && t < N) {
          if (key[g] > prefix) m |= 1u << g;
          else if (key[g] == prefix && e++ < remaining) m |= 1u << g;
        }
      }
    }
    if (t < N) mk[t] = (uint16_t)m;
    carry += tot;
  }
}

// Step 2: per stream, exclusive scan of the chunk sums (in place); writes the
// stream total to tok_off[N] and flags a packed store that is too small.
__global__ __launch_bounds__(256) void scan_chunks_kernel(uint32_t* chunk_sum, uint32_t* tok_off,
                                                          int32_t* dev_status, int N, int nchunks,
                                                          long long cap, int Ncap) {
  __shared__ int red[4];
  const int stream = blockIdx.x;
  uint32_t* cs = chunk_sum + (size_t)stream * nchunks;
  int carry = 0;
  for (int base = 0; base < nchunks; base += 256) {
    const int i = base + threadIdx.x;
    const int v = i < nchunks ? (int)cs[i] : 0;
    int tot;
    const int ex = block_exscan_256(v, red, &tot);
    if (i < nchunks) cs[i] = (uint32_t)(carry + ex);
    carry += tot;
  }
  if (threadIdx.x == 0) {
    tok_off[(size_t)stream * (Ncap + 1) + N] = (uint32_t)carry;
    if (dev_status && (long long)carry > cap) *dev_status = 1;
  }
}

// Step 3: per-token offsets, then the packed copy.  Work items are 16-byte
// pieces of V in memory order, so reads are coalesced and the writes of kept
// neighbours are adjacent.
template <int D>
__global__ __launch_bounds__(kChunk) void pack_kernel(const uint4* __restrict__ V,
                                                      const uint16_t* __restrict__ mask,
                                                      const uint32_t* __restrict__ chunk_off,
                                                      uint32_t* __restrict__ tok_off,
                                                      uint4* __restrict__ vpacked, int N, int G,
                                                      int nchunks, long long cap, int Ncap) {
  __shared__ int red[4];
  __shared__ uint32_t s_off[kChunk];
  __shared__ uint32_t s_mask[kChunk];
  constexpr int PPT = D / 8;  // 16-byte pieces per token row
  const int stream = blockIdx.y;
  const int t0 = blockIdx.x * kChunk;
  const int t = t0 + threadIdx.x;
  uint32_t m = 0;
  if (t < N) m = mask[(size_t)stream * Ncap + t];
  const int ex = block_exscan_256(__popc(m), red, nullptr);
  const uint32_t off = chunk_off[(size_t)stream * nchunks + blockIdx.x] + (uint32_t)ex;
  if (t < N) tok_off[(size_t)stream * (Ncap + 1) + t] = off;
  s_off[threadIdx.x] = off;
  s_mask[threadIdx.x] = m;
  __syncthreads();
  const int ppg = PPT / G;  // pieces per group (gd*2/16)
  const int ntok = min(kChunk, N - t0);
  const uint4* src = V + ((size_t)stream * N + t0) * PPT;
  uint4* dst = vpacked + (size_t)stream * (size_t)cap * ppg;
  for (int e = threadIdx.x; e < ntok * PPT; e += kChunk) {
    const int tok = e / PPT, pc = e % PPT;
    const int g = pc / ppg, within = pc % ppg;
    const uint32_t mk = s_mask[tok];
    if ((mk >> g) & 1u) {
      const long long slot = (long long)s_off[tok] + __popc(mk & ((1u << g) - 1u));
      if (slot < cap) dst[slot * ppg + within] = src[e];
    }
  }
}

// Row gather used to compact a cache to the tokens a token-level method kept.
template <int D>
__global__ __launch_bounds__(256) void compact_kernel(const uint4* __restrict__ src,
                                                      const int32_t* __restrict__ token_idx,
                                                      uint4* __restrict__ dst, int Hkv, int N_src,
                                                      int n_keep, int32_t* dev_status) {
  constexpr int PPT = D / 8;
  const int stream = blockIdx.y, b = stream / Hkv;
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= n_keep * PPT) return;
  const int i = e / PPT, pc = e % PPT;
  const int t = token_idx[(size_t)b * n_keep + i];
  uint4 v = make_uint4(0, 0, 0, 0);
  if (t >= 0 && t < N_src) {
    v = src[((size_t)stream * N_src + t) * PPT + pc];
  } else if (dev_status && pc == 0) {
    *dev_status = 1;
  }
  dst[((size_t)stream * n_keep + i) * PPT + pc] = v;
}

size_t route_ws_bytes(const stc_shape_t& s) {
  const size_t nchunks = (s.N + kChunk - 1) / kChunk;
  return (size_t)s.B * s.Hkv * nchunks * sizeof(uint32_t);
}

int launch_route_pack(const stc_shape_t& s, int mode, const void* V, const float* logits,
                      const uint8_t* kcount, int fixed_k, const uint16_t* mask_in, uint16_t* mask,
                      uint32_t* tok_off, void* vpacked, int32_t* dev_status, void* ws,
                      hipStream_t st) {
  const int streams = s.B * s.Hkv;
  const int nchunks = (s.N + kChunk - 1) / kChunk;
  const int Ncap = token_cap(s);  // stride of mask and tok_off; V, logits, kcount are dense
  int mask_in_stride = s.N;
  uint32_t* chunk = (uint32_t*)ws;
  dim3 grid(nchunks, streams);
  if (mode == STC_ROUTE_GLOBAL) {
    // the mask of the whole stream first, then the common path with that mask as given
    route_global_kernel<<<streams, kGlobalThreads, 0, st>>>(
        logits, mask, s.N, s.G, (uint32_t)((long long)s.N * fixed_k), Ncap);
    if (hipGetLastError() != hipSuccess) return -1;
    mode = STC_ROUTE_MASK;
    mask_in = mask;
    mask_in_stride = Ncap;
  }
  route_mask_kernel<<<grid, kChunk, 0, st>>>(mode, logits, kcount, fixed_k, mask_in, mask, chunk,
                                             s.N, s.G, nchunks, Ncap, mask_in_stride);
  if (hipGetLastError() != hipSuccess) return -1;
  scan_chunks_kernel<<<streams, 256, 0, st>>>(chunk, tok_off, dev_status, s.N, nchunks,
                                              (long long)s.v_cap_groups, Ncap);
  if (hipGetLastError() != hipSuccess) return -1;
  if (s.D == 128)
    pack_kernel<128><<<grid, kChunk, 0, st>>>((const uint4*)V, mask, chunk, tok_off,
                                              (uint4*)vpacked, s.N, s.G, nchunks,
                                              (long long)s.v_cap_groups, Ncap);
  else
    pack_kernel<64><<<grid, kChunk, 0, st>>>((const uint4*)V, mask, chunk, tok_off,
                                             (uint4*)vpacked, s.N, s.G, nchunks,
                                             (long long)s.v_cap_groups, Ncap);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

int launch_compact(const void* src, const int32_t* token_idx, void* dst, int B, int Hkv, int N_src,
                   int n_keep, int D, int32_t* dev_status, hipStream_t st) {
  const int per_stream = n_keep * (D / 8);
  dim3 grid((per_stream + 255) / 256, B * Hkv);
  if (D == 128)
    compact_kernel<128><<<grid, 256, 0, st>>>((const uint4*)src, token_idx, (uint4*)dst, Hkv, N_src,
                                              n_keep, dev_status);
  else
    compact_kernel<64><<<grid, 256, 0, st>>>((const uint4*)src, token_idx, (uint4*)dst, Hkv, N_src,
                                             n_keep, dev_status);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

}  // namespace stc
