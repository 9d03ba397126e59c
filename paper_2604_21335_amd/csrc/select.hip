// Query-aware page selection (Quest, Sec. 3.2): the k pages of largest upper-bound score
// of each stream (the scores come from score.hip).
#include "stc_common.hpp"
#include "stc_kernels.hpp"
#include "topk_block.hpp"

namespace stc {

// ---------------------------------------------------------------------------
// Top-k pages of a stream: radix select of the k-th largest key (4 passes of 8
// bits), then an order-preserving compaction.  Equal scores are taken in
// ascending page order; the output is ascending in page index.
// ---------------------------------------------------------------------------
constexpr int kSelThreads = 1024;

__global__ __launch_bounds__(kSelThreads) void topk_kernel(const float* __restrict__ score,
                                                           int32_t* __restrict__ page_idx, int NP,
                                                           int k) {
  __shared__ int hist[256];
  __shared__ int waves[kSelThreads / 64];
  __shared__ uint32_t s_prefix;
  __shared__ int s_remaining;
  const int stream = blockIdx.x;
  const float* sc = score + (size_t)stream * NP;
  int32_t* out = page_idx + (size_t)stream * k;
  const int tid = threadIdx.x;

  uint32_t prefix = 0;  // leading bits of the k-th largest key found so far
  int remaining = k;    // rank of that key among the keys sharing the prefix
  for (int shift = 24; shift >= 0; shift -= 8) {
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    for (int i = tid; i < NP; i += kSelThreads) {
      const uint32_t key = float_key(sc[i]);
      const bool in = shift == 24 || (key >> (shift + 8)) == (prefix >> (shift + 8));
      if (in) atomicAdd(&hist[(key >> shift) & 255u], 1);
    }
    __syncthreads();
    // digits in descending order: thread t looks at digit 255 - t
    const int cnt = tid < 256 ? hist[255 - tid] : 0;
    int tot;
    const int above = block_exscan(cnt, waves, &tot);  // keys with a larger digit
    if (tid < 256 && above < remaining && remaining <= above + cnt) {
      s_prefix = prefix | ((uint32_t)(255 - tid) << shift);
      s_remaining = remaining - above;
    }
    __syncthreads();
    prefix = s_prefix;
    remaining = s_remaining;
    __syncthreads();
  }
  // prefix = key of the k-th largest score; `remaining` of the pages equal to
  // it are taken, lowest page index first.
  const int per = (NP + kSelThreads - 1) / kSelThreads;
  const int i0 = min(tid * per, NP), i1 = min(i0 + per, NP);
  int eq = 0;
  for (int i = i0; i < i1; ++i) eq += float_key(sc[i]) == prefix;
  int tot;
  int eq_before = block_exscan(eq, waves, &tot);
  int sel = 0;
  {
    int e = eq_before;
    for (int i = i0; i < i1; ++i) {
      const uint32_t key = float_key(sc[i]);
      if (key > prefix) ++sel;
      else if (key == prefix) sel += (e++ < remaining);
    }
  }
  int pos = block_exscan(sel, waves, &tot);
  for (int i = i0; i < i1; ++i) {
    const uint32_t key = float_key(sc[i]);
    bool take = key > prefix;
    if (key == prefix) take = eq_before++ < remaining;
    if (take && pos < k) out[pos++] = i;
  }
}

// Stand-alone selection: one workgroup per stream.
template <int IPT, int THREADS>
__global__ __launch_bounds__(THREADS) void topk_reg_kernel(const float* __restrict__ score,
                                                           int32_t* __restrict__ page_idx, int NP,
                                                           int k) {
  int32_t* out = page_idx + (size_t)blockIdx.x * k;
  topk_block<IPT, THREADS>(score + (size_t)blockIdx.x * NP, NP, k,
                           [out](int pos, int page) { out[pos] = page; });
}

__global__ void iota_pages_kernel(int32_t* __restrict__ page_idx, int NP, int total) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < total) page_idx[i] = i % NP;
}

int launch_select(const stc_shape_t& s, const void* q, const void* bounds, int k_pages,
                  int32_t* page_idx, float* score, bool per_head, hipStream_t st) {
  const int NP = (s.N + kPage - 1) / kPage;
  const int streams = s.B * (per_head ? s.Hq : s.Hkv);  // page lists to produce
  if (k_pages >= NP) {
    const int total = streams * NP;
    iota_pages_kernel<<<(total + 255) / 256, 256, 0, st>>>(page_idx, NP, total);
    return hipGetLastError() == hipSuccess ? 0 : -1;
  }
  if (!per_head && score_can_select(s, k_pages))
    return launch_score_select(s, q, bounds, score, page_idx, k_pages, st);
  if (launch_score(s, q, bounds, score, per_head, st)) return -1;
  // keys per thread; streams of more than 1024 pages use 512 threads (measured: faster than
  // both 256 threads with more keys each and 1024 threads with longer barriers)
#define STC_TOPK(IPT, TH) \
  topk_reg_kernel<IPT, TH><<<streams, TH, 0, st>>>(score, page_idx, NP, k_pages)
  if (NP <= 256) STC_TOPK(1, 256);
  else if (NP <= 512) STC_TOPK(2, 256);
  else if (NP <= 1024) STC_TOPK(4, 256);
  else if (NP <= 2048) STC_TOPK(4, 512);
  else if (NP <= 4096) STC_TOPK(8, 512);
  else if (NP <= 8192) STC_TOPK(16, 512);
  else topk_kernel<<<streams, kSelThreads, 0, st>>>(score, page_idx, NP, k_pages);
#undef STC_TOPK
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

// Union of the R page lists of a KV head's query heads, one workgroup per KV head.  The lists
// (R*k entries) sit in LDS.  Pages are walked in tiles of kUnionTile: every list entry that
// falls into the tile ORs its head's bit into the tile's array of head sets, then thread t
// takes the tile's pages 16t .. 16t+15 in order and a block scan compacts the pages with a
// non-empty set.  Unused output slots get page -1.
constexpr int kUnionTile = 4096;

__global__ __launch_bounds__(256) void union_pages_kernel(const int32_t* __restrict__ lists,
                                                          int32_t* __restrict__ union_idx,
                                                          uint16_t* __restrict__ union_heads,
                                                          int NP, int R, int k, int U) {
  extern __shared__ int32_t s_list[];  // [R * k]
  __shared__ uint32_t s_set[kUnionTile];
  __shared__ int waves[4];
  constexpr int PPT = kUnionTile / 256;  // pages per thread and tile
  const int stream = blockIdx.x;
  const int tid = threadIdx.x;
  const int n = R * k;
  for (int i = tid; i < n; i += 256) s_list[i] = lists[(size_t)stream * n + i];
  int32_t* out_idx = union_idx + (size_t)stream * U;
  uint16_t* out_heads = union_heads + (size_t)stream * U;
  int base = 0;  // union entries written so far (pages below the current tile)
  for (int p0 = 0; p0 < NP; p0 += kUnionTile) {
    for (int i = tid; i < kUnionTile; i += 256) s_set[i] = 0u;
    __syncthreads();  // also: the lists are in LDS
    const int p1 = min(p0 + kUnionTile, NP);
    for (int i = tid; i < n; i += 256) {
      const int p = s_list[i];
      if (p >= p0 && p < p1) atomicOr(&s_set[p - p0], 1u << (i / k));
    }
    __syncthreads();
    uint32_t m[PPT];
    int cnt = 0;
#pragma unroll
    for (int j = 0; j < PPT; ++j) {
      m[j] = s_set[tid * PPT + j];
      cnt += m[j] != 0;
    }
    int tot;
    int pos = base + block_exscan(cnt, waves, &tot);  // ends with a barrier: s_set may be reused
#pragma unroll
    for (int j = 0; j < PPT; ++j) {
      if (m[j] != 0 && pos < U) {
        out_idx[pos] = p0 + tid * PPT + j;
        out_heads[pos] = (uint16_t)m[j];
      }
      pos += m[j] != 0;
    }
    base += tot;
  }
  for (int i = min(base, U) + tid; i < U; i += 256) {
    out_idx[i] = -1;
    out_heads[i] = 0;
  }
}

int launch_union_pages(const stc_shape_t& s, const int32_t* page_idx_per_head, int k_pages,
                       int32_t* union_idx, uint16_t* union_heads, int U, hipStream_t st) {
  const int NP = (s.N + kPage - 1) / kPage;
  const int R = s.Hq / s.Hkv;
  const size_t lds = (size_t)R * k_pages * sizeof(int32_t);
  // up to 64 KiB of lists next to the 16 KiB of head sets: beyond the default LDS limit
  static std::atomic<uint64_t> allowed{0};
  if (!allow_dynamic_lds((const void*)union_pages_kernel, 65536, allowed)) return -1;
  union_pages_kernel<<<s.B * s.Hkv, 256, lds, st>>>(page_idx_per_head, union_idx, union_heads, NP,
                                                    R, k_pages, U);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

}  // namespace stc
