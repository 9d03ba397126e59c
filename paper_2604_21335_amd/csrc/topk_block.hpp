// Top-k pages of one stream by one workgroup: shared by the stand-alone selection kernel and
// by the attention kernel whose workgroups select their own pages.
#pragma once
#include "stc_common.hpp"

namespace stc {

__device__ __forceinline__ int wave_incl_scan(int v, int lane) {
  for (int d = 1; d < 64; d <<= 1) {
    const int o = __shfl_up(v, d);
    if (lane >= d) v += o;
  }
  return v;
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

// Top-k pages of a stream by one workgroup of THREADS threads with the keys held in
// registers: thread t owns the IPT adjacent pages t*IPT .. (NP <= THREADS * IPT).  The selected
// pages are handed to emit(position in the ascending list, page).  Each radix pass is a
// shared-memory histogram of one key byte, a block scan over the digits in descending
// order and a broadcast of the digit that holds the k-th largest key.
template <int IPT, int THREADS, class Emit>
__device__ __forceinline__ void topk_block(const float* __restrict__ sc, int NP, int k,
                                           Emit emit) {
  __shared__ int hist[256];
  __shared__ int waves[THREADS / 64];
  __shared__ uint32_t s_prefix;
  __shared__ int s_remaining, s_cand, s_ncand;
  __shared__ uint32_t cand[64];
  const int tid = threadIdx.x;
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

  // Bits above the highest bit in which two keys differ are common to all keys and
  // need no pass; starting at that bit also spreads the first histogram over many
  // bins (page scores share their sign and most exponent bits).
  uint32_t kmin = 0xffffffffu, kmax = 0u;
#pragma unroll
  for (int j = 0; j < IPT; ++j)
    if (i0 + j < NP) kmin = min(kmin, key[j]), kmax = max(kmax, key[j]);
  for (int d = 32; d >= 1; d >>= 1) {
    kmin = min(kmin, (uint32_t)__shfl_xor((int)kmin, d));
    kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, d));
  }
  __shared__ uint32_t s_min[THREADS / 64], s_max[THREADS / 64];
  if ((tid & 63) == 0) s_min[tid >> 6] = kmin, s_max[tid >> 6] = kmax;
  __syncthreads();
#pragma unroll
  for (int w = 0; w < THREADS / 64; ++w) kmin = min(kmin, s_min[w]), kmax = max(kmax, s_max[w]);
  const uint32_t diff = kmin ^ kmax;
  const int top = diff ? 31 - __clz(diff) : 0;  // highest differing bit
  int shift = max(top - 7, 0);
  uint32_t decided = shift + 8 < 32 ? ~((1u << (shift + 8)) - 1u) : 0u;  // key bits fixed so far
  uint32_t prefix = kmax & decided;
  int remaining = k;  // rank of the k-th largest key among the keys sharing the prefix
  // The last window may overlap bits that are already fixed; keys are filtered on all
  // fixed bits, so the digit found repeats them.
  for (;; shift = max(shift - 8, 0)) {
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
#pragma unroll
    for (int j = 0; j < IPT; ++j) {
      const bool in = (key[j] & decided) == prefix;
      if (in && i0 + j < NP) atomicAdd(&hist[(key[j] >> shift) & 255u], 1);
    }
    __syncthreads();
    const int cnt = tid < 256 ? hist[255 - tid] : 0;  // digits in descending order
    int tot;
    const int above = block_exscan(cnt, waves, &tot);  // keys with a larger digit
    if (tid < 256 && above < remaining && remaining <= above + cnt) {
      s_prefix = (prefix & ~(255u << shift)) | ((uint32_t)(255 - tid) << shift);
      s_remaining = remaining - above;
      s_cand = cnt;  // keys that share the new prefix
      s_ncand = 0;
    }
    __syncthreads();
    prefix = s_prefix;
    remaining = s_remaining;
    decided = ~((1u << shift) - 1u);
    if (shift == 0) break;
    if (s_cand <= 64) {
      // Few keys are left: list them, and let one wavefront rank them directly.
#pragma unroll
      for (int j = 0; j < IPT; ++j)
        if (i0 + j < NP && (key[j] & decided) == prefix) cand[atomicAdd(&s_ncand, 1)] = key[j];
      __syncthreads();
      const int c = s_cand;
      if (tid < c) {
        const uint32_t mine = cand[tid];
        int gt = 0, ge = 0;
        for (int i = 0; i < c; ++i) {
          const uint32_t o = cand[i];
          gt += o > mine;
          ge += o >= mine;
        }
        if (gt < remaining && remaining <= ge) {  // equal keys all write the same pair
          s_prefix = mine;
          s_remaining = remaining - gt;
        }
      }
      __syncthreads();
      prefix = s_prefix;
      remaining = s_remaining;
      break;
    }
  }
  // prefix = key of the k-th largest score; `remaining` of the pages equal to it are
  // taken, lowest page index first.
  int eq = 0;
#pragma unroll
  for (int j = 0; j < IPT; ++j) eq += (i0 + j < NP) && key[j] == prefix;
  int tot;
  const int eq_before = block_exscan(eq, waves, &tot);
  int sel = 0;
  uint32_t take = 0;  // bit j: page i0 + j is selected
  {
    int e = eq_before;
#pragma unroll
    for (int j = 0; j < IPT; ++j) {
      if (i0 + j < NP) {
        bool t = key[j] > prefix;
        if (key[j] == prefix) t = e++ < remaining;
        if (t) {
          take |= 1u << j;
          ++sel;
        }
      }
    }
  }
  int pos = block_exscan(sel, waves, &tot);
#pragma unroll
  for (int j = 0; j < IPT; ++j)
    if (((take >> j) & 1u) && pos < k) emit(pos++, i0 + j);
}

}  // namespace stc
