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
    int nchunks, int Ncap, int mask_in_stride, int share) {
  __shared__ int red[4];
  const int stream = blockIdx.y;
  const int src = stream / share;  // the routing inputs of `share` streams are one set
  const int t = blockIdx.x * kChunk + threadIdx.x;
  uint32_t m = 0;
  if (t < N) {
    const size_t tok = (size_t)src * N + t;  // dense inputs: logits, kcount
    if (mode == STC_ROUTE_MASK) {
      m = mask_in[(size_t)src * mask_in_stride + t] & ((1u << G) - 1u);
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
// Global token-group budget (Sec. 3.4; App. B.1: M = N*K of the N x S pairs): the key of the
// M-th largest of a stream's N*G logits by a radix select (12 + 10 + 10 bits; the wide first
// digit spreads logits that share sign and exponent over many bins), then every pair above
// that key is kept plus the first `remaining` pairs equal to it in (token, group) order.
// Every pass over the logits is spread over the whole chip: many workgroups per stream build
// the digit histogram (shared memory first, then one atomic per non-empty bin), one workgroup
// per stream picks the digit.  Per-stream state lives in the workspace.
// ---------------------------------------------------------------------------
constexpr int kGlobalThreads = 1024;
constexpr int kGlobalBins = 4096;
constexpr int kHistThreads = 256;
constexpr int kHistSlice = 16384;  // logits per histogram workgroup

struct GlobalState {
  uint32_t prefix;     // key bits fixed so far
  uint32_t decided;    // mask of those bits
  uint32_t remaining;  // rank of the wanted key among the keys that share the prefix
  uint32_t take_all;   // after the last pass: every pair equal to the key is kept
};

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

__device__ __forceinline__ int global_shift(int pass) { return pass == 0 ? 20 : (pass == 1 ? 10 : 0); }
__device__ __forceinline__ uint32_t global_bins(int pass) { return pass == 0 ? 4096u : 1024u; }

// Start of a selection: empty histograms, nothing decided, rank = budget.
__global__ __launch_bounds__(256) void global_init_kernel(uint32_t* __restrict__ hist,
                                                          GlobalState* __restrict__ state,
                                                          int streams, uint32_t budget) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < streams * kGlobalBins) hist[i] = 0u;
  if (i < streams) state[i] = GlobalState{0u, 0u, budget, 0u};
}

// Histogram of digit `pass` over the keys that share the stream's prefix; workgroup
// blockIdx.x covers logits [blockIdx.x * slice, +slice) of stream blockIdx.y.
__global__ __launch_bounds__(kHistThreads) void global_hist_kernel(
    const float* __restrict__ logits, uint32_t* __restrict__ hist,
    const GlobalState* __restrict__ state, uint32_t n, uint32_t slice, int pass, int share) {
  __shared__ uint32_t lh[kGlobalBins];
  const int stream = blockIdx.y;
  const int tid = threadIdx.x;
  const int shift = global_shift(pass);
  const uint32_t bins = global_bins(pass);
  const uint32_t prefix = state[stream].prefix, decided = state[stream].decided;
  for (uint32_t i = tid; i < bins; i += kHistThreads) lh[i] = 0u;
  __syncthreads();
  const float* a = logits + (size_t)(stream / share) * n;
  const uint32_t lo = blockIdx.x * slice, hi = n - lo < slice ? n : lo + slice;
  auto count = [&](float f) {
    const uint32_t key = logit_key(f);
    if ((key & decided) == prefix) atomicAdd(&lh[(key >> shift) & (bins - 1)], 1u);
  };
  if ((n & 3u) == 0) {  // every stream and slice starts on a 16-byte boundary
    for (uint32_t i = lo + 4 * tid; i < hi; i += 4 * kHistThreads) {
      const float4 v = *(const float4*)(a + i);
      count(v.x), count(v.y), count(v.z), count(v.w);
    }
  } else {
    for (uint32_t i = lo + tid; i < hi; i += kHistThreads) count(a[i]);
  }
  __syncthreads();
  uint32_t* gh = hist + (size_t)stream * kGlobalBins;
  for (uint32_t i = tid; i < bins; i += kHistThreads) {
    const uint32_t c = lh[i];
    if (c) atomicAdd(&gh[i], c);
  }
}

// The digit that holds the wanted key: block scan over the stream's histogram in descending
// digit order.  Leaves the histogram empty for the next pass.
__global__ __launch_bounds__(kGlobalThreads) void global_pick_kernel(
    uint32_t* __restrict__ hist, GlobalState* __restrict__ state, int pass) {
  __shared__ uint32_t waves[kGlobalThreads / 64];
  const int stream = blockIdx.x;
  const int tid = threadIdx.x;
  const int shift = global_shift(pass);
  const uint32_t bins = global_bins(pass);
  uint32_t* gh = hist + (size_t)stream * kGlobalBins;
  const GlobalState st = state[stream];
  // thread t owns the 4 adjacent digits 4095-4t .. 4092-4t (descending order)
  uint32_t c[4], own = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const uint32_t d = kGlobalBins - 1 - (4 * tid + j);
    c[j] = d < bins ? gh[d] : 0u;
    if (d < bins) gh[d] = 0u;
    own += c[j];
  }
  uint32_t tot;
  uint32_t above = block_exscan_1024(own, waves, &tot);  // pairs with a larger digit
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    if (above < st.remaining && st.remaining <= above + c[j]) {
      GlobalState nx;
      nx.prefix = st.prefix | ((uint32_t)(kGlobalBins - 1 - (4 * tid + j)) << shift);
      nx.decided = st.decided | ((bins - 1) << shift);
      nx.remaining = st.remaining - above;
      nx.take_all = nx.remaining == c[j] ? 1u : 0u;
      state[stream] = nx;
    }
    above += c[j];
  }
}

// Pairs equal to the stream's key per chunk of 256 tokens (the chunks of the mask kernel).
__global__ __launch_bounds__(kChunk) void global_eq_kernel(const float* __restrict__ logits,
                                                           const GlobalState* __restrict__ state,
                                                           uint32_t* __restrict__ chunk_eq, int N,
                                                           int G, int nchunks, int share) {
  __shared__ int red[4];
  const int stream = blockIdx.y;
  if (state[stream].take_all) return;  // no ranks among equal pairs needed
  const uint32_t key = state[stream].prefix;
  const uint32_t n = (uint32_t)N * (uint32_t)G;
  const float* a = logits + (size_t)(stream / share) * n;
  const uint32_t lo = (uint32_t)blockIdx.x * kChunk * G;
  const uint32_t hi = n - lo < (uint32_t)kChunk * G ? n : lo + (uint32_t)kChunk * G;
  int eq = 0;
  for (uint32_t i = lo + threadIdx.x; i < hi; i += kChunk) eq += logit_key(a[i]) == key;
  const int tot = block_sum_256(eq, red);
  if (threadIdx.x == 0) chunk_eq[(size_t)stream * nchunks + blockIdx.x] = (uint32_t)tot;
}

// Exclusive scan of a stream's per-chunk counts, in place.
__global__ __launch_bounds__(256) void global_eq_scan_kernel(uint32_t* chunk_eq,
                                                             const GlobalState* __restrict__ state,
                                                             int nchunks) {
  __shared__ int red[4];
  if (state[blockIdx.x].take_all) return;
  uint32_t* cs = chunk_eq + (size_t)blockIdx.x * nchunks;
  int carry = 0;
  for (int base = 0; base < nchunks; base += 256) {
    const int i = base + threadIdx.x;
    const int v = i < nchunks ? (int)cs[i] : 0;
    int tot;
    const int ex = block_exscan_256(v, red, &tot);
    if (i < nchunks) cs[i] = (uint32_t)(carry + ex);
    carry += tot;
  }
}

// Masks of a chunk of 256 tokens from the stream's key: pairs above it, and the first
// `remaining` pairs equal to it in (token, group) order.  Also the chunk's number of kept
// groups, as route_mask_kernel writes it.  budget == 0 keeps nothing.
template <int G>
__global__ __launch_bounds__(kChunk) void global_mask_kernel(
    const float* __restrict__ logits, const GlobalState* __restrict__ state,
    const uint32_t* __restrict__ chunk_eq, uint16_t* __restrict__ mask,
    uint32_t* __restrict__ chunk_sum, int N, int nchunks, int Ncap, uint32_t budget, int share) {
  __shared__ int red[4];
  const int stream = blockIdx.y;
  const int t = blockIdx.x * kChunk + threadIdx.x;
  const GlobalState gs = state[stream];
  const uint32_t prefix = gs.prefix, remaining = gs.remaining;
  const bool ranked = budget > 0 && !gs.take_all;  // equal pairs are taken in order
  float lg[G];
  load_token_logits<G>(logits + ((size_t)(stream / share) * N + min(t, N - 1)) * G, lg);
  uint32_t key[G];
  int eq = 0;
#pragma unroll
  for (int g = 0; g < G; ++g) {
    key[g] = t < N ? logit_key(lg[g]) : 0u;
    eq += (t < N && ranked) && key[g] == prefix;
  }
  uint32_t e = (ranked ? chunk_eq[(size_t)stream * nchunks + blockIdx.x] : 0u) +
               (uint32_t)block_exscan_256(eq, red, nullptr);
  uint32_t m = 0;
  if (budget > 0 && t < N) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      if (key[g] > prefix) m |= 1u << g;
      else if (key[g] == prefix && (!ranked || e++ < remaining)) m |= 1u << g;
    }
  }
  if (t < N) mask[(size_t)stream * Ncap + t] = (uint16_t)m;
  const int tot = block_sum_256(__popc(m), red);
  if (threadIdx.x == 0) chunk_sum[(size_t)stream * nchunks + blockIdx.x] = (uint32_t)tot;
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

namespace {

// Workspace: kept groups per chunk, then (global budget only) equal-key counts per chunk,
// the per-stream digit histograms and the per-stream selection state.
struct RouteWs {
  size_t chunk_sum, chunk_eq, hist, state, total;
};

RouteWs route_ws_layout(const stc_shape_t& s) {
  const size_t streams = (size_t)s.B * s.Hkv;
  const size_t nchunks = (s.N + kChunk - 1) / kChunk;
  auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
  RouteWs w;
  w.chunk_sum = 0;
  w.chunk_eq = up(streams * nchunks * sizeof(uint32_t));
  w.hist = w.chunk_eq + up(streams * nchunks * sizeof(uint32_t));
  w.state = w.hist + up(streams * kGlobalBins * sizeof(uint32_t));
  w.total = w.state + up(streams * sizeof(GlobalState));
  return w;
}

}  // namespace

size_t route_ws_bytes(const stc_shape_t& s) { return route_ws_layout(s).total; }

int launch_route_pack(const stc_shape_t& s, int mode, const void* V, const float* logits,
                      const uint8_t* kcount, int fixed_k, const uint16_t* mask_in, uint16_t* mask,
                      uint32_t* tok_off, void* vpacked, int32_t* dev_status, void* ws,
                      hipStream_t st) {
  // STC_ROUTE_SHARED: one set of routing inputs per batch element, read by all its KV heads
  const int share = (mode & STC_ROUTE_SHARED) ? s.Hkv : 1;
  mode &= ~STC_ROUTE_SHARED;
  const int streams = s.B * s.Hkv;
  const int nchunks = (s.N + kChunk - 1) / kChunk;
  const int Ncap = token_cap(s);  // stride of mask and tok_off; V, logits, kcount are dense
  const RouteWs lay = route_ws_layout(s);
  uint32_t* chunk = (uint32_t*)((char*)ws + lay.chunk_sum);
  dim3 grid(nchunks, streams);
  if (mode == STC_ROUTE_GLOBAL) {
    uint32_t* chunk_eq = (uint32_t*)((char*)ws + lay.chunk_eq);
    uint32_t* hist = (uint32_t*)((char*)ws + lay.hist);
    GlobalState* state = (GlobalState*)((char*)ws + lay.state);
    const uint32_t budget = (uint32_t)((long long)s.N * fixed_k);
    const uint32_t n = (uint32_t)s.N * (uint32_t)s.G;
    global_init_kernel<<<(streams * kGlobalBins + 255) / 256, 256, 0, st>>>(hist, state, streams,
                                                                            budget);
    if (budget > 0) {
      dim3 hgrid((unsigned)(((unsigned long long)n + kHistSlice - 1) / kHistSlice), streams);
      for (int pass = 0; pass < 3; ++pass) {
        global_hist_kernel<<<hgrid, kHistThreads, 0, st>>>(logits, hist, state, n, kHistSlice,
                                                           pass, share);
        global_pick_kernel<<<streams, kGlobalThreads, 0, st>>>(hist, state, pass);
      }
      global_eq_kernel<<<grid, kChunk, 0, st>>>(logits, state, chunk_eq, s.N, s.G, nchunks,
                                                share);
      global_eq_scan_kernel<<<streams, 256, 0, st>>>(chunk_eq, state, nchunks);
    }
#define STC_GLOBAL_MASK(GG)                                                                   \
  case GG:                                                                                    \
    global_mask_kernel<GG><<<grid, kChunk, 0, st>>>(logits, state, chunk_eq, mask, chunk, s.N, \
                                                    nchunks, Ncap, budget, share);            \
    break;
    switch (s.G) {
      STC_GLOBAL_MASK(1)
      STC_GLOBAL_MASK(2)
      STC_GLOBAL_MASK(4)
      STC_GLOBAL_MASK(8)
      STC_GLOBAL_MASK(16)
      default:
        return -1;
    }
#undef STC_GLOBAL_MASK
  } else {
    route_mask_kernel<<<grid, kChunk, 0, st>>>(mode, logits, kcount, fixed_k, mask_in, mask, chunk,
                                               s.N, s.G, nchunks, Ncap, s.N, share);
  }
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
