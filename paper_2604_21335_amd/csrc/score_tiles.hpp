// Quest page scores of a range of bounds tiles by one workgroup (the arithmetic and the tile
// layout are described at the top of score.hip).  The query operands of the matrix-core
// products live in shared memory, one 64-bit operand per (head group, channel, lane), so that
// the registers of a wavefront hold only tile data and partial sums: the form with at most 128
// registers, i.e. four wavefronts per SIMD, also for more than four heads per KV head.
#pragma once
#include "stc_common.hpp"

namespace stc {

typedef __attribute__((ext_vector_type(4))) short score_bf16x4;
typedef __attribute__((ext_vector_type(4))) float score_f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t score_u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t score_u32x2;

// Bytes of shared memory for the query operands of one KV head's R query heads.
template <int D, int R>
__host__ __device__ constexpr int score_q_lds_bytes() {
  return ((R + 3) / 4) * (D / 8) * 64 * 8;
}

// Fills the operand table for the R heads at `qs` ([R][D] bf16).  Entry (g, c, lane) is the A
// operand of lane `lane` for channel c of its chunk and head 4g + lane%4: the query value in
// the k-slot of the channel's minimum when it is negative, of its maximum otherwise, zeros in
// the three other slots (the channel pair of a B operand occupies two slots each).  All
// threads of the workgroup call it; the caller synchronises before the table is read.
template <int D, int R, int THREADS>
__device__ __forceinline__ void score_fill_q(const uint16_t* __restrict__ qs, unsigned char* qlds) {
  constexpr int CH = D / 8, NG = (R + 3) / 4, PIECES = CH / 8;  // 16-byte pieces per chunk
  // one work item = 8 adjacent channels of one (head group, lane): a single 16-byte load
  for (int it = threadIdx.x; it < NG * PIECES * 64; it += THREADS) {
    const int l = it & 63, piece = (it >> 6) % PIECES, g = it / (64 * PIECES);
    const int head = 4 * g + (l & 3), e = (l >> 2) & 7;
    score_u32x4 v = {0u, 0u, 0u, 0u};
    if (head < R) v = *(const score_u32x4*)(qs + head * D + e * CH + piece * 8);
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t lo = w[i] & 0xffffu, hi = w[i] >> 16;  // channels 2i and 2i+1 of the piece
      const uint32_t qa0 = (lo & 0x8000u) ? lo : lo << 16;
      const uint32_t qa1 = (hi & 0x8000u) ? hi : hi << 16;
      const int c = piece * 8 + 2 * i;
      *(score_u32x2*)(qlds + (size_t)((g * CH + c) * 64 + l) * 8) = score_u32x2{qa0, 0u};
      *(score_u32x2*)(qlds + (size_t)((g * CH + c + 1) * 64 + l) * 8) = score_u32x2{0u, qa1};
    }
  }
}

// Scores tiles t0 + wave, t0 + wave + WAVES, ... < t1 of one stream.  `base` = the stream's
// tiles + lane; out = the stream's score row(s).  DEPTH tiles of the wavefront are requested
// ahead (DEPTH - 1 in flight behind the one being computed).  `prologue` is run by every thread
// once the first tiles have been requested: it fills the operand table (score_fill_q) and
// synchronises the workgroup, so that the latency of the query loads hides behind the tiles'.
template <int D, int R, bool PER_HEAD, int WAVES, int DEPTH = 2, class Prologue>
__device__ __forceinline__ void score_tile_range(const score_u32x4* __restrict__ base,
                                                 float* __restrict__ out, int NP, int t0, int t1,
                                                 const unsigned char* qlds, int wave, int lane,
                                                 Prologue prologue) {
  constexpr int CH = D / 8, NJ = CH / 4, NG = (R + 3) / 4, T16 = NJ * 64;
  const int tlast = t1 - 1;
  uint32_t qoff = lane * 8;
  auto load_tile = [&](score_u32x4 (&dst)[NJ], int tt) {
    const score_u32x4* pt = base + (size_t)min(tt, tlast) * T16;  // past the range: last tile again
#pragma unroll
    for (int j = 0; j < NJ; ++j) dst[j] = pt[j * 64];
  };
  auto score_tile = [&](const score_u32x4 (&cur)[NJ], int tt) {
    float best = 0.f;
    // the operand table is read anew for every tile: an address the compiler cannot see through
    // keeps its loads inside the tile loop instead of pinning every operand in a register
    asm volatile("" : "+v"(qoff));
    const unsigned char* ql = qlds + qoff;
    const int page = tt * kBoundsTilePages + 4 * (lane >> 5) + (lane & 3);
    const bool writer = (lane & 0x1c) == kChunkSumLanes && page < NP;
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      const score_f32x4 zero = {0.f, 0.f, 0.f, 0.f};
      score_f32x4 u[NJ];  // per 16-byte unit: sum of its four channels, per head row
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        const score_bf16x4 b01 = __builtin_bit_cast(score_bf16x4, score_u32x2{cur[j].x, cur[j].y});
        const score_bf16x4 b23 = __builtin_bit_cast(score_bf16x4, score_u32x2{cur[j].z, cur[j].w});
        score_f32x4 t[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const score_bf16x4 a =
              *(const score_bf16x4*)(ql + (size_t)((g * CH + 4 * j + k) * 64) * 8);
          t[k] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(a, k < 2 ? b01 : b23, zero, 0, 0, 0);
        }
        u[j] = (t[0] + t[1]) + (t[2] + t[3]);
      }
#pragma unroll
      for (int w = 1; w < NJ; w *= 2)
#pragma unroll
        for (int j = 0; j < NJ; j += 2 * w) u[j] += u[j + w];
      const int rows = (R - 4 * g) < 4 ? (R - 4 * g) : 4;
#pragma unroll
      for (int i = 0; i < rows; ++i) {
        const float s = chunk_tree_sum(u[0][i]);
        if (PER_HEAD) {
          if (writer) out[(size_t)(4 * g + i) * NP + page] = s == 0.f ? 0.f : s;
        } else {
          best = (g == 0 && i == 0) ? s : fmaxf(best, s);
        }
      }
    }
    if (!PER_HEAD && writer) out[page] = best == 0.f ? 0.f : best;
  };

  int t = t0 + wave;
  const bool any = t < t1;  // wave-uniform
  score_u32x4 d[DEPTH][NJ];
  if (any) static_for<0, DEPTH>([&](auto k) { load_tile(d[k], t + k * WAVES); });
  __builtin_amdgcn_sched_barrier(0);  // the tile requests go out first
  prologue();
  if (!any) return;
  for (; t < t1; t += DEPTH * WAVES) {
    static_for<0, DEPTH>([&](auto k) {
      if (k == 0 || t + k * WAVES < t1) {
        score_tile(d[k], t + k * WAVES);
        load_tile(d[k], t + (k + DEPTH) * WAVES);
      }
    });
  }
}

}  // namespace stc
