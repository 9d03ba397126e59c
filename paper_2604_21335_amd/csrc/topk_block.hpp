// Top-k pages of one stream by one workgroup: shared by the stand-alone selection kernel and
// by the attention kernel whose workgroups select their own pages.
#pragma once
#include "stc_common.hpp"

namespace stc {

// One step of a wavefront scan on the data-parallel-primitive path (no LDS traffic): lanes
// whose source lies outside the row, or whose row is masked off, combine with `ident`.
#define STC_DPP_STEP(v, op, ident, ctrl, row_mask) \
  v = op(v, (uint32_t)__builtin_amdgcn_update_dpp((int)(ident), (int)(v), ctrl, row_mask, 0xf, false))

struct OpAdd {
  __device__ __forceinline__ uint32_t operator()(uint32_t a, uint32_t b) const { return a + b; }
};
struct OpMin {
  __device__ __forceinline__ uint32_t operator()(uint32_t a, uint32_t b) const { return min(a, b); }
};
struct OpMax {
  __device__ __forceinline__ uint32_t operator()(uint32_t a, uint32_t b) const { return max(a, b); }
};

// Inclusive scan over the 64 lanes: shifts by 1, 2, 4, 8 inside each row of 16 lanes, then
// lane 15 of rows 0 and 2 into rows 1 and 3, then lane 31 into rows 2 and 3.
template <class Op>
__device__ __forceinline__ uint32_t wave_scan(uint32_t v, Op op, uint32_t ident) {
  STC_DPP_STEP(v, op, ident, 0x111, 0xf);  // row_shr:1
  STC_DPP_STEP(v, op, ident, 0x112, 0xf);  // row_shr:2
  STC_DPP_STEP(v, op, ident, 0x114, 0xf);  // row_shr:4
  STC_DPP_STEP(v, op, ident, 0x118, 0xf);  // row_shr:8
  STC_DPP_STEP(v, op, ident, 0x142, 0xa);  // row_bcast:15 into rows 1 and 3
  STC_DPP_STEP(v, op, ident, 0x143, 0xc);  // row_bcast:31 into rows 2 and 3
  return v;
}
#undef STC_DPP_STEP

// Reduction over the 64 lanes, in a scalar register.
template <class Op>
__device__ __forceinline__ uint32_t wave_reduce(uint32_t v, Op op, uint32_t ident) {
  return (uint32_t)__builtin_amdgcn_readlane((int)wave_scan(v, op, ident), 63);
}

__device__ __forceinline__ int wave_incl_scan(int v, int /*lane*/) {
  return (int)wave_scan((uint32_t)v, OpAdd{}, 0u);
}

// Exclusive scan over the block (thread order); *total = block sum.
__device__ __forceinline__ int block_exscan(int v, int* lds_waves, int* total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nw = blockDim.x >> 6;
  const int inc = wave_incl_scan(v, lane);
  if (lane == 63) lds_waves[wave] = inc;
  __syncthreads();
  int base = 0, tot = 0;
  for (int w = 0; w < nw; ++w) {
    const int x = lds_waves[w];
    if (w < wave) base += x;
    tot += x;
  }
  *total = tot;
  __syncthreads();
  return base + inc - v;
}

// The same scan for callers that keep two buffers of per-wavefront sums and alternate
// between them: a buffer is written again two barriers after it was last read at the
// earliest, so the barrier behind the reads can go.
template <int NW>
__device__ __forceinline__ uint32_t block_exscan_once(uint32_t v, uint32_t* lds_waves,
                                                      uint32_t* total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint32_t inc = wave_scan(v, OpAdd{}, 0u);
  if (lane == 63) lds_waves[wave] = inc;
  __syncthreads();
  uint32_t base = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < NW; ++w) {
    const uint32_t x = lds_waves[w];
    if (w < wave) base += x;
    tot += x;
  }
  *total = tot;
  return base + inc - v;
}

// Top-k pages of a stream by one workgroup of THREADS threads with the keys held in
// registers: thread t owns the IPT adjacent pages t*IPT .. (NP <= THREADS * IPT <= 65535).
// The selected pages are handed to emit(position in the ascending list, page).  Each radix
// pass is a shared-memory histogram of one key byte, which every wavefront then scans for
// itself (digits in descending order) to find the digit that holds the k-th largest key: no
// broadcast and no second barrier.  The usual case (one pass, then at most 64 candidates
// ranked directly) crosses five workgroup barriers.
template <int IPT, int THREADS, class Emit>
__device__ __forceinline__ void topk_block(const float* __restrict__ sc, int NP, int k,
                                           Emit emit) {
  constexpr int NW = THREADS / 64;
  __shared__ __align__(16) int hist[256];
  __shared__ uint32_t waves[NW];  // per-wavefront sums of the final scan
  __shared__ uint32_t s_min[NW], s_max[NW];
  __shared__ int s_ncand;
  __shared__ uint32_t cand[64];
  __shared__ int s_gt[64], s_ge[64];  // per candidate: candidates above it / not below it
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int i0 = tid * IPT;

  // keys of absent pages (index >= NP) are 0, below the key of any finite float
  uint32_t key[IPT];
  if constexpr (IPT >= 4) {
    if (i0 + IPT <= NP && (NP % 4) == 0) {
#pragma unroll
      for (int j = 0; j < IPT; j += 4) {
        const float4 v = *(const float4*)(sc + i0 + j);
        key[j] = float_key(v.x), key[j + 1] = float_key(v.y);
        key[j + 2] = float_key(v.z), key[j + 3] = float_key(v.w);
      }
    } else {
#pragma unroll
      for (int j = 0; j < IPT; ++j) key[j] = i0 + j < NP ? float_key(sc[i0 + j]) : 0u;
    }
  } else {
#pragma unroll
    for (int j = 0; j < IPT; ++j) key[j] = i0 + j < NP ? float_key(sc[i0 + j]) : 0u;
  }
  if (tid < 256) hist[tid] = 0;
  if (tid < 64) s_gt[tid] = 0, s_ge[tid] = 0;
  if (tid == 0) s_ncand = 0;

  // Bits above the highest bit in which two keys differ are common to all keys and
  // need no pass; starting at that bit also spreads the first histogram over many
  // bins (page scores share their sign and most exponent bits).
  uint32_t kmin = 0xffffffffu, kmax = 0u;
#pragma unroll
  for (int j = 0; j < IPT; ++j)
    if (i0 + j < NP) kmin = min(kmin, key[j]), kmax = max(kmax, key[j]);
  kmin = wave_reduce(kmin, OpMin{}, 0xffffffffu);
  kmax = wave_reduce(kmax, OpMax{}, 0u);
  if ((tid & 63) == 0) s_min[tid >> 6] = kmin, s_max[tid >> 6] = kmax;
  __syncthreads();
#pragma unroll
  for (int w = 0; w < NW; ++w) kmin = min(kmin, s_min[w]), kmax = max(kmax, s_max[w]);
  const uint32_t diff = kmin ^ kmax;
  const int top = diff ? 31 - __clz(diff) : 0;  // highest differing bit
  int shift = max(top - 7, 0);
  uint32_t decided = shift + 8 < 32 ? ~((1u << (shift + 8)) - 1u) : 0u;  // key bits fixed so far
  uint32_t prefix = kmax & decided;
  int remaining = k;  // rank of the k-th largest key among the keys sharing the prefix
  // The last window may overlap bits that are already fixed; keys are filtered on all
  // fixed bits, so the digit found repeats them.  The histogram is zero on entry to every
  // pass.
  for (;; shift = max(shift - 8, 0)) {
#pragma unroll
    for (int j = 0; j < IPT; ++j) {
      const bool in = (key[j] & decided) == prefix;
      if (in && i0 + j < NP) atomicAdd(&hist[(key[j] >> shift) & 255u], 1);
    }
    __syncthreads();
    // Every wavefront finds the digit for itself (no broadcast, no second barrier): lane l
    // looks at digits 255-4l .. 252-4l, a wavefront scan gives the keys with a larger digit.
    const int4 h4 = *(const int4*)&hist[252 - 4 * lane];
    const int c4[4] = {h4.w, h4.z, h4.y, h4.x};
    const int mine4 = c4[0] + c4[1] + c4[2] + c4[3];
    int above = (int)wave_scan((uint32_t)mine4, OpAdd{}, 0u) - mine4;
    int f_digit = 0, f_above = 0, f_cnt = 0;
    bool found = false;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const bool hit = above < remaining && remaining <= above + c4[j];
      if (hit) f_digit = 255 - 4 * lane - j, f_above = above, f_cnt = c4[j];
      found |= hit;
      above += c4[j];
    }
    const int src = __builtin_amdgcn_readfirstlane(__ffsll((long long)__ballot(found)) - 1);
    const int digit = __builtin_amdgcn_readlane(f_digit, src);
    const int c = __builtin_amdgcn_readlane(f_cnt, src);  // keys that share the new prefix
    remaining -= __builtin_amdgcn_readlane(f_above, src);
    prefix = (prefix & ~(255u << shift)) | ((uint32_t)digit << shift);
    decided = ~((1u << shift) - 1u);
    if (shift == 0) break;
    if (c <= 64) {
      // Few keys are left: list them and rank them directly.
#pragma unroll
      for (int j = 0; j < IPT; ++j)
        if (i0 + j < NP && (key[j] & decided) == prefix) cand[atomicAdd(&s_ncand, 1)] = key[j];
      __syncthreads();
      // rank of every candidate among the candidates: wavefront w compares all of them with
      // its share of the list, the partial counts meet in shared memory
      {
        constexpr int PER = (64 + NW - 1) / NW;
        const int ci = tid & 63, j0 = (tid >> 6) * PER;
        if (ci < c && j0 < c) {
          const uint32_t mine = cand[ci];
          int gt = 0, ge = 0;
#pragma unroll
          for (int j = 0; j < PER; ++j) {
            const uint32_t o = cand[min(j0 + j, 63)];
            const bool in = j0 + j < c;
            gt += in && o > mine;
            ge += in && o >= mine;
          }
          if (gt) atomicAdd(&s_gt[ci], gt);
          if (ge) atomicAdd(&s_ge[ci], ge);
        }
      }
      __syncthreads();
      {  // every wavefront picks the k-th key itself: lane i looks at candidate i
        const int ci = min(lane, c - 1);
        const int gt = s_gt[ci], ge = s_ge[ci];
        const uint32_t mine = cand[ci];
        const bool kth = gt < remaining && remaining <= ge;  // equal keys agree
        const int s2 = __builtin_amdgcn_readfirstlane(__ffsll((long long)__ballot(kth)) - 1);
        prefix = (uint32_t)__builtin_amdgcn_readlane((int)mine, s2);
        remaining -= __builtin_amdgcn_readlane(gt, s2);
      }
      break;
    }
    // another pass: the histogram is cleared once every wavefront has read it
    __syncthreads();
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
  }
  // prefix = key of the k-th largest score; `remaining` of the pages equal to it are
  // taken, lowest page index first.  One scan carries both counts of a thread: pages above
  // the key in the low half, pages equal to it in the high half.
  uint32_t both = 0;
#pragma unroll
  for (int j = 0; j < IPT; ++j)
    if (i0 + j < NP) both += (key[j] > prefix ? 1u : 0u) + (key[j] == prefix ? 0x10000u : 0u);
  uint32_t tot;
  const uint32_t before = block_exscan_once<NW>(both, waves, &tot);
  int e = (int)(before >> 16);                           // equal pages in front of this thread
  int pos = (int)(before & 0xffffu) + min(e, remaining);  // selected pages in front of it
#pragma unroll
  for (int j = 0; j < IPT; ++j) {
    if (i0 + j < NP) {
      bool t = key[j] > prefix;
      if (key[j] == prefix) t = e++ < remaining;
      if (t && pos < k) emit(pos++, i0 + j);
    }
  }
}

}  // namespace stc
