// Quest page scores (query-aware token-level stage, Sec. 3.2):
//   U_h[p] = sum_c max(q_h[c]*mn[p,c], q_h[c]*mx[p,c]),  score[p] = max_h U_h[p]
// in float, the D terms summed as a balanced tree over adjacent channels.
//
// Because mn <= mx, the larger product is q*mx for q >= 0 and q*mn for q < 0, so with
// q- = min(q, 0) and q+ = max(q, 0) a term is q-*mn + q+*mx, where one of the two products
// is an exact zero.  That is a 2-slot dot product, and the matrix cores compute it:
// v_mfma_f32_4x4x4_16b_bf16 multiplies, per block, a 4x4 A (rows = query heads, 4 k-slots)
// with a 4x4 B (k-slots, columns = pages).  A k-slot pair holds (mn, mx) of one channel
// and the A row holds (q-, q+) in that pair and zeros in the other pair.  A product of two
// bf16 values is exact in float and the other three addends are zeros, so the result is
// the exact term whatever rounding the unit applies to longer sums (it does not round
// sums of two non-zero products to nearest, which is why the pair sums stay on the VALU).
// All additions of the tree are then ordinary float additions, in the fixed order.
//
// The bounds are stored in tiles of 8 pages laid out for this kernel (see
// bounds_tile_unit): a wavefront fetches a tile with D/32 fully contiguous 1 KiB
// requests and every 64-bit register pair it receives is a B operand as it stands.
// Lane l of a wavefront holds, for page 4*(l/32) + l%4 of the tile, the D/8 channels
// of chunk (l/4)%8; the 16 blocks of the MFMA are the 16 (page group, chunk) pairs.
#include "score_tiles.hpp"
#include "stc_common.hpp"
#include "stc_kernels.hpp"
#include "topk_block.hpp"

namespace stc {

typedef __attribute__((ext_vector_type(4))) short bf16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

__device__ __forceinline__ bf16x4 as_bf16x4(uint32_t w0, uint32_t w1) {
  return __builtin_bit_cast(bf16x4, (u32x2){w0, w1});
}

// Two head groups of 128 channels need 168 registers: exactly three wavefronts per SIMD.
// (Left to itself the compiler aims higher and spills.)
#define STC_SCORE_WAVES_PER_SIMD \
  amdgpu_waves_per_eu((D == 128 && R > 4) ? 3 : 4, (D == 128 && R > 4) ? 3 : 8)

// PER_HEAD: every query head's own score is written ([B, Hq, NP]) instead of the maximum
// over the heads of the KV head ([B, Hkv, NP]).
// SELECT: one workgroup of 8 wavefronts scores a whole stream (NP <= 2048) into LDS and then
// selects the stream's k pages itself (`score` is then an optional copy of the scores): the
// form for many streams of few pages each, where a stream per workgroup still fills the chip
// and the selection needs no launch of its own.
constexpr int kScoreSelectPages = 2048;
template <int D, int R, bool PER_HEAD, bool SELECT>
__global__ __launch_bounds__(SELECT ? 512 : 256) __attribute__((STC_SCORE_WAVES_PER_SIMD))
void score_mfma_kernel(const u32x4* __restrict__ tiles, const uint16_t* __restrict__ q,
                       float* __restrict__ score, int NP, int Hq, int Hkv, int tiles_per_block,
                       int tiles_cap, int32_t* __restrict__ page_idx, int k_pages) {
  static_assert(!(SELECT && PER_HEAD), "one list per KV head");
  constexpr int CH = D / 8;        // channels per lane
  constexpr int NJ = CH / 4;       // 16-byte units per lane and tile
  constexpr int NG = (R + 3) / 4;  // groups of 4 query heads (MFMA rows)
  constexpr int T16 = NJ * 64;     // 16-byte units per tile
  constexpr int WAVES = SELECT ? 8 : 4;
  __shared__ __align__(16) float s_score[SELECT ? kScoreSelectPages : 4];
  const int stream = SELECT ? blockIdx.x : blockIdx.y;
  const int b = stream / Hkv, kvh = stream % Hkv;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int row = lane & 3, e = (lane >> 2) & 7;
  const int ntiles = (NP + kBoundsTilePages - 1) / kBoundsTilePages;

  // A operands, one word per (head group, channel): the query value in the low half when
  // it is negative (it meets the channel's minimum there), else in the high half (maximum).
  uint32_t qa[NG][CH];
#pragma unroll
  for (int g = 0; g < NG; ++g) {
    const int head = 4 * g + row;
    const uint16_t* qp = q + ((size_t)b * Hq + kvh * R + min(head, R - 1)) * D + e * CH;
#pragma unroll
    for (int c = 0; c < CH; c += 2) {
      const uint32_t w = *(const uint32_t*)(qp + c);
      const uint32_t lo = w & 0xffffu, hi = w >> 16;
      qa[g][c] = head < R ? ((lo & 0x8000u) ? lo : lo << 16) : 0u;
      qa[g][c + 1] = head < R ? ((hi & 0x8000u) ? hi : hi << 16) : 0u;
    }
  }

  const int t0 = SELECT ? 0 : blockIdx.x * tiles_per_block;
  const int t1 = SELECT ? ntiles : min(t0 + tiles_per_block, ntiles);
  const u32x4* base = tiles + (size_t)stream * tiles_cap * T16 + lane;  // capacity stride
  float* out = SELECT ? s_score : score + (size_t)stream * (PER_HEAD ? R : 1) * NP;
  const int tlast = t1 - 1;

  // tile index past the block's range: its last tile is fetched again (never stored)
#define STC_LOAD_TILE(dst, tt)                                    \
  {                                                               \
    const u32x4* pt_ = base + (size_t)min((tt), tlast) * T16;     \
    _Pragma("unroll") for (int j = 0; j < NJ; ++j) dst[j] = pt_[j * 64]; \
  }
#define STC_SCORE_TILE(cur, tt)                                                                  \
  {                                                                                              \
    float best = 0.f;                                                                            \
    _Pragma("unroll") for (int g = 0; g < NG; ++g) {                                             \
      f32x4 term[CH]; /* [channel][head row] */                                                  \
      const f32x4 zero = {0.f, 0.f, 0.f, 0.f};                                                   \
      _Pragma("unroll") for (int j = 0; j < NJ; ++j) {                                           \
        const bf16x4 b01 = as_bf16x4(cur[j].x, cur[j].y), b23 = as_bf16x4(cur[j].z, cur[j].w);   \
        term[4 * j + 0] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(                                \
            as_bf16x4(qa[g][4 * j + 0], 0u), b01, zero, 0, 0, 0);                                \
        term[4 * j + 1] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(                                \
            as_bf16x4(0u, qa[g][4 * j + 1]), b01, zero, 0, 0, 0);                                \
        term[4 * j + 2] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(                                \
            as_bf16x4(qa[g][4 * j + 2], 0u), b23, zero, 0, 0, 0);                                \
        term[4 * j + 3] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(                                \
            as_bf16x4(0u, qa[g][4 * j + 3]), b23, zero, 0, 0, 0);                                \
      }                                                                                          \
      const int rows = (R - 4 * g) < 4 ? (R - 4 * g) : 4;                                        \
      _Pragma("unroll") for (int i = 0; i < rows; ++i) {                                         \
        float v[CH];                                                                             \
        _Pragma("unroll") for (int c = 0; c < CH; ++c) v[c] = term[c][i];                        \
        _Pragma("unroll") for (int w = 1; w < CH; w *= 2)                                        \
          _Pragma("unroll") for (int c = 0; c < CH; c += 2 * w) v[c] += v[c + w];                \
        const float u = chunk_tree_sum(v[0]);                                                    \
        if (PER_HEAD) {                                                                          \
          const int page = (tt) * kBoundsTilePages + 4 * (lane >> 5) + (lane & 3);               \
          if ((lane & 0x1c) == kChunkSumLanes && page < NP)                                      \
            out[(size_t)(4 * g + i) * NP + page] = u == 0.f ? 0.f : u;                           \
        } else {                                                                                 \
          best = (g == 0 && i == 0) ? u : fmaxf(best, u);                                        \
        }                                                                                        \
      }                                                                                          \
    }                                                                                            \
    if (!PER_HEAD) {                                                                             \
      const int page = (tt) * kBoundsTilePages + 4 * (lane >> 5) + (lane & 3);                   \
      if ((lane & 0x1c) == kChunkSumLanes && page < NP) out[page] = best == 0.f ? 0.f : best;    \
    }                                                                                            \
  }

  // two tiles of this wavefront are always in flight behind the one being computed
  int t = t0 + wave;
  u32x4 d0[NJ], d1[NJ];
  STC_LOAD_TILE(d0, t);
  STC_LOAD_TILE(d1, t + WAVES);
  for (; t < t1; t += 2 * WAVES) {
    STC_SCORE_TILE(d0, t);
    STC_LOAD_TILE(d0, t + 2 * WAVES);
    if (t + WAVES < t1) {
      STC_SCORE_TILE(d1, t + WAVES);
      STC_LOAD_TILE(d1, t + 3 * WAVES);
    }
  }
#undef STC_LOAD_TILE
#undef STC_SCORE_TILE
  if constexpr (SELECT) {
    __syncthreads();
    if (score)
      for (int i = threadIdx.x; i < NP; i += 64 * WAVES) score[(size_t)stream * NP + i] = s_score[i];
    int32_t* list = page_idx + (size_t)stream * k_pages;
    topk_block<kScoreSelectPages / (64 * WAVES), 64 * WAVES>(
        s_score, NP, k_pages, [list](int pos, int page) { list[pos] = page; });
  }
}

// The same scores with the query operands in shared memory (score_tiles.hpp): at most 128
// registers, so four wavefronts per SIMD also for five to eight heads per KV head.
template <int D, int R, bool PER_HEAD, int WAVES>
__global__ __launch_bounds__(64 * WAVES) __attribute__((amdgpu_waves_per_eu(4, 8)))
void score_lds_kernel(const u32x4* __restrict__ tiles, const uint16_t* __restrict__ q,
                      float* __restrict__ score, int NP, int Hq, int Hkv, int tiles_per_block,
                      int tiles_cap) {
  constexpr int T16 = (D / 32) * 64;
  __shared__ __align__(16) unsigned char s_q[score_q_lds_bytes<D, R>()];
  const int stream = blockIdx.y;
  const int b = stream / Hkv, kvh = stream % Hkv;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int ntiles = (NP + kBoundsTilePages - 1) / kBoundsTilePages;
  const int t0 = blockIdx.x * tiles_per_block;
  const int t1 = min(t0 + tiles_per_block, ntiles);
  const uint16_t* qs = q + ((size_t)b * Hq + kvh * R) * D;
  score_tile_range<D, R, PER_HEAD, WAVES, 1>(
      (const score_u32x4*)tiles + (size_t)stream * tiles_cap * T16 + lane,
      score + (size_t)stream * (PER_HEAD ? R : 1) * NP, NP, t0, t1, s_q, wave, lane, [&] {
        score_fill_q<D, R, 64 * WAVES>(qs, s_q);
        __syncthreads();
      });
}

// A bf16 value widened to float, with subnormal inputs read as zero (what the matrix cores do
// with the operands of the kernel above).
__device__ __forceinline__ float daz(float x) {
  return (__float_as_uint(x) & 0x7f800000u) ? x : 0.f;
}

// Any number of query heads per KV head (up to 16), one head at a time on the VALU: the
// same tiles, the same lane assignment and the same order of additions.
template <int D>
__global__ __launch_bounds__(256) void score_any_kernel(const u32x4* __restrict__ tiles,
                                                        const uint16_t* __restrict__ q,
                                                        float* __restrict__ score, int NP, int Hq,
                                                        int Hkv, int R, int tiles_per_block,
                                                        int per_head, int tiles_cap) {
  constexpr int CH = D / 8, NJ = CH / 4, T16 = NJ * 64;
  const int stream = blockIdx.y;
  const int b = stream / Hkv, kvh = stream % Hkv;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int e = (lane >> 2) & 7;
  const int ntiles = (NP + kBoundsTilePages - 1) / kBoundsTilePages;
  const int t0 = blockIdx.x * tiles_per_block, t1 = min(t0 + tiles_per_block, ntiles);
  const u32x4* base = tiles + (size_t)stream * tiles_cap * T16 + lane;  // capacity stride
  float* out = score + (size_t)stream * (per_head ? R : 1) * NP;
  for (int t = t0 + wave; t < t1; t += 4) {
    uint32_t w[CH];
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const u32x4 v = base[(size_t)t * T16 + j * 64];
      w[4 * j] = v.x, w[4 * j + 1] = v.y, w[4 * j + 2] = v.z, w[4 * j + 3] = v.w;
    }
    float best = 0.f;
    const int page = t * kBoundsTilePages + 4 * (lane >> 5) + (lane & 3);
    const bool writer = (lane & 0x1c) == kChunkSumLanes && page < NP;
    for (int h = 0; h < R; ++h) {
      const uint16_t* qp = q + ((size_t)b * Hq + kvh * R + h) * D + e * CH;
      float v[CH];
#pragma unroll
      for (int c = 0; c < CH; ++c) {
        const float qc = daz(__uint_as_float((uint32_t)qp[c] << 16));
        v[c] = fmaxf(qc * daz(bf16_lo(w[c])), qc * daz(bf16_hi(w[c])));
      }
#pragma unroll
      for (int s = 1; s < CH; s *= 2)
#pragma unroll
        for (int c = 0; c < CH; c += 2 * s) v[c] += v[c + s];
      const float u = chunk_tree_sum(v[0]);
      if (per_head && writer) out[(size_t)h * NP + page] = u == 0.f ? 0.f : u;
      best = h == 0 ? u : fmaxf(best, u);
    }
    if (!per_head && writer) out[page] = best == 0.f ? 0.f : best;
  }
}

template <int D>
static void launch_score_d(const stc_shape_t& s, const void* q, const void* bounds, float* score,
                           int NP, bool per_head, hipStream_t st) {
  const int streams = s.B * s.Hkv;
  const int R = s.Hq / s.Hkv;
  const int ntiles = (NP + kBoundsTilePages - 1) / kBoundsTilePages;
  const int tcap = bounds_tiles(token_cap(s));  // tiles per stream in memory
  // about three workgroups per CU (what the register budget keeps resident), so the whole
  // grid runs as one generation and the per-wavefront set-up is paid once per several tiles
  const int want_blocks = max(1, 768 / streams);
  int tpb = (ntiles + want_blocks - 1) / want_blocks;
  tpb = (tpb + 3) / 4 * 4;  // one tile per wavefront and round
  dim3 grid((ntiles + tpb - 1) / tpb, streams);
  const u32x4* t4 = (const u32x4*)bounds;
  const uint16_t* q16 = (const uint16_t*)q;
  if (D == 128 && R > 4 && R <= 8) {
    // query operands in shared memory.  Many small workgroups (about 2048: two tiles per
    // wavefront on the headline shape) whose wavefronts request one tile at a time: measured,
    // the memory system delivers more with fewer requests outstanding per wavefront (13.3 us
    // against 14.6 with two tiles requested ahead and a third as many workgroups)
    constexpr int WV = 4;
    const int want = max(1, 2048 / streams);
    int tp = (ntiles + want - 1) / want;
    tp = (tp + WV - 1) / WV * WV;
    dim3 g2((ntiles + tp - 1) / tp, streams);
#define STC_SCORE_LDS_CASE(RR)                                                                 \
  case RR:                                                                                     \
    if (per_head)                                                                              \
      score_lds_kernel<D, RR, true, WV><<<g2, 64 * WV, 0, st>>>(t4, q16, score, NP, s.Hq,      \
                                                                s.Hkv, tp, tcap);              \
    else                                                                                       \
      score_lds_kernel<D, RR, false, WV><<<g2, 64 * WV, 0, st>>>(t4, q16, score, NP, s.Hq,     \
                                                                 s.Hkv, tp, tcap);             \
    break;
    switch (R) {
      STC_SCORE_LDS_CASE(5)
      STC_SCORE_LDS_CASE(6)
      STC_SCORE_LDS_CASE(7)
      STC_SCORE_LDS_CASE(8)
    }
#undef STC_SCORE_LDS_CASE
    return;
  }
#define STC_SCORE_CASE(RR)                                                                    \
  case RR:                                                                                    \
    if (per_head)                                                                             \
      score_mfma_kernel<D, RR, true, false><<<grid, 256, 0, st>>>(t4, q16, score, NP, s.Hq,   \
                                                                  s.Hkv, tpb, tcap, nullptr, 0); \
    else                                                                                      \
      score_mfma_kernel<D, RR, false, false><<<grid, 256, 0, st>>>(t4, q16, score, NP, s.Hq,  \
                                                                   s.Hkv, tpb, tcap, nullptr, 0); \
    break;
  switch (R) {
    STC_SCORE_CASE(1)
    STC_SCORE_CASE(2)
    STC_SCORE_CASE(3)
    STC_SCORE_CASE(4)
    STC_SCORE_CASE(5)
    STC_SCORE_CASE(6)
    STC_SCORE_CASE(7)
    STC_SCORE_CASE(8)
    default:
      score_any_kernel<D><<<grid, 256, 0, st>>>(t4, q16, score, NP, s.Hq, s.Hkv, R, tpb,
                                                per_head ? 1 : 0, tcap);
  }
#undef STC_SCORE_CASE
}

// Scoring and selection of a whole stream by one workgroup (see SELECT above).
template <int D>
static int launch_score_select_d(const stc_shape_t& s, const void* q, const void* bounds,
                                 float* score, int32_t* page_idx, int k_pages, int NP,
                                 hipStream_t st) {
  const int streams = s.B * s.Hkv;
  const int tcap = bounds_tiles(token_cap(s));
  const u32x4* t4 = (const u32x4*)bounds;
  const uint16_t* q16 = (const uint16_t*)q;
#define STC_SCORE_SELECT_CASE(RR)                                                            \
  case RR:                                                                                   \
    score_mfma_kernel<D, RR, false, true><<<streams, 512, 0, st>>>(t4, q16, score, NP, s.Hq, \
                                                                   s.Hkv, 0, tcap, page_idx, \
                                                                   k_pages);                 \
    break;
  switch (s.Hq / s.Hkv) {
    STC_SCORE_SELECT_CASE(1)
    STC_SCORE_SELECT_CASE(2)
    STC_SCORE_SELECT_CASE(3)
    STC_SCORE_SELECT_CASE(4)
    STC_SCORE_SELECT_CASE(5)
    STC_SCORE_SELECT_CASE(6)
    STC_SCORE_SELECT_CASE(7)
    STC_SCORE_SELECT_CASE(8)
    default:
      return -1;
  }
#undef STC_SCORE_SELECT_CASE
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

// Where the single workgroup per stream wins (measured on 64..512 streams of 256..2048 pages
// against scoring and selection as two launches): always on short streams, where both forms
// are bound by their launches; with few heads per KV head (registers for two workgroups per
// CU) from 128 streams on; with many heads once every CU has a stream.
bool score_can_select(const stc_shape_t& s, int k_pages) {
  const int NP = (s.N + kPage - 1) / kPage;
  const int R = s.Hq / s.Hkv, streams = s.B * s.Hkv;
  if (k_pages >= NP || NP > kScoreSelectPages || R > 8) return false;
  return NP <= 256 || (R <= 4 && streams >= 128) || streams >= 256;
}

int launch_score_select(const stc_shape_t& s, const void* q, const void* bounds, float* score,
                        int32_t* page_idx, int k_pages, hipStream_t st) {
  const int NP = (s.N + kPage - 1) / kPage;
  return s.D == 128 ? launch_score_select_d<128>(s, q, bounds, score, page_idx, k_pages, NP, st)
                    : launch_score_select_d<64>(s, q, bounds, score, page_idx, k_pages, NP, st);
}

int launch_score(const stc_shape_t& s, const void* q, const void* bounds, float* score,
                 bool per_head, hipStream_t st) {
  const int NP = (s.N + kPage - 1) / kPage;
  if (s.D == 128)
    launch_score_d<128>(s, q, bounds, score, NP, per_head, st);
  else
    launch_score_d<64>(s, q, bounds, score, NP, per_head, st);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

}  // namespace stc
