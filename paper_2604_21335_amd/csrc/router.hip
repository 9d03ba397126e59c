// Value-group router (App. B.1): one linear projection from the layer-input hidden state of a
// token to its G group logits, logits[t, g] = sum_c h[t, c] * W[g, c] (+ bias[g]).
//
// The masks are integer decisions taken on these logits, so the float summation order is
// fixed: d_model is cut into chunks of 128 adjacent channels, a chunk is summed as a balanced
// tree over adjacent channels, and the chunk sums are accumulated left to right; the bias is
// added last.
//
// The products come from the matrix cores, exactly: v_mfma_f32_4x4x4_16b_bf16 multiplies, per
// block, a 4x4 A (rows = 4 groups, 4 k-slots) with a 4x4 B (k-slots, columns = 4 tokens).  A
// B register pair holds 4 adjacent channels of the lane's token as loaded; the A row holds the
// weight of ONE of those channels in its slot and zeros in the other three, so every output is
// a single product of two bf16 values (exact in float) plus exact zeros, whatever rounding the
// unit applies to longer sums.  All additions are ordinary float additions in the fixed order.
//
// Lane l of a wavefront: token 4*(l/32) + l%4 of a group of 8 tokens, channels
// 16*((l/4)%8) .. +16 of the current chunk (two 16-byte loads of h).  The 16 blocks of the MFMA
// are the 16 (token quad, 16-channel piece) pairs; the lane supplies the A row of group l%4
// (+4 per further MFMA group) for its block's channels.  Per (token, group) the 16 products of
// a lane are summed as a pair tree in the lane, the 8 pieces by the rotations and the row
// exchange of chunk_tree_sum; the lanes with (l & 0x1c) == 4 hold the chunk sums and carry the
// accumulators.  A wavefront works on TG groups of 8 tokens per chunk, so the weights of a
// chunk are fetched and masked once for 8*TG tokens.
//
// Inputs are zero or normal bf16 numbers (the matrix cores read subnormal bf16 inputs as
// zero), with products in the normal float range.
#include "stc_common.hpp"
#include "stc_kernels.hpp"

namespace stc {

typedef __attribute__((ext_vector_type(4))) short bf16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

__device__ __forceinline__ bf16x4 router_bf16x4(uint32_t w0, uint32_t w1) {
  return __builtin_bit_cast(bf16x4, (u32x2){w0, w1});
}

template <int G>
struct RouterCfg {
  static constexpr int NH = (G + 3) / 4;        // MFMA row groups of 4 router outputs
  static constexpr int TG = G == 16 ? 1 : 2;    // groups of 8 tokens per wavefront
  static constexpr int WAVE_TOKENS = 8 * TG;
  static constexpr int BLOCK_TOKENS = 4 * WAVE_TOKENS;
};

template <int G>
__global__ __launch_bounds__(256) void router_logits_kernel(const uint4* __restrict__ h,
                                                            const uint4* __restrict__ W,
                                                            const float* __restrict__ bias,
                                                            float* __restrict__ logits, int N,
                                                            int d_model, int Hkv,
                                                            int bias_stride) {
  using C = RouterCfg<G>;
  constexpr int NH = C::NH, TG = C::TG;
  const int b = blockIdx.y;
  if (bias) bias += (size_t)b * bias_stride;  // 0: one bias for the batch; G: one per element
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int j = lane & 3, dp = (lane >> 2) & 7, tq = lane >> 5;
  const int t_first = blockIdx.x * C::BLOCK_TOKENS + wave * C::WAVE_TOKENS + 4 * tq + j;
  const int nc = d_model / 128;
  const int row16 = d_model / 8;  // 16-byte pieces per row

  // rows past the end repeat the last token (never stored)
  const uint4* hp[TG];
#pragma unroll
  for (int g8 = 0; g8 < TG; ++g8)
    hp[g8] = h + ((size_t)b * N + min(t_first + 8 * g8, N - 1)) * row16 + dp * 2;
  // the A rows this lane supplies: router output 4*hh + j (none beyond G: zeros)
  const uint4* wp[NH];
#pragma unroll
  for (int hh = 0; hh < NH; ++hh) wp[hh] = W + (size_t)min(4 * hh + j, G - 1) * row16 + dp * 2;

  float acc[TG][NH][4];
#pragma unroll
  for (int g8 = 0; g8 < TG; ++g8)
#pragma unroll
    for (int hh = 0; hh < NH; ++hh)
#pragma unroll
      for (int i = 0; i < 4; ++i) acc[g8][hh][i] = 0.f;

  uint4 hx[TG][2], wx[NH][2];
#pragma unroll
  for (int g8 = 0; g8 < TG; ++g8) hx[g8][0] = hp[g8][0], hx[g8][1] = hp[g8][1];
#pragma unroll
  for (int hh = 0; hh < NH; ++hh) wx[hh][0] = wp[hh][0], wx[hh][1] = wp[hh][1];

  for (int c = 0; c < nc; ++c) {
    // A operands of this chunk: the weight of channel ch alone in its half of its dword
    uint32_t aw[NH][16];
#pragma unroll
    for (int hh = 0; hh < NH; ++hh) {
      const uint32_t wd[8] = {wx[hh][0].x, wx[hh][0].y, wx[hh][0].z, wx[hh][0].w,
                              wx[hh][1].x, wx[hh][1].y, wx[hh][1].z, wx[hh][1].w};
      const bool live = 4 * hh + j < G;
#pragma unroll
      for (int d = 0; d < 8; ++d) {
        aw[hh][2 * d] = live ? (wd[d] & 0xffffu) : 0u;
        aw[hh][2 * d + 1] = live ? (wd[d] & 0xffff0000u) : 0u;
      }
    }
    uint4 cur[TG][2];
#pragma unroll
    for (int g8 = 0; g8 < TG; ++g8) cur[g8][0] = hx[g8][0], cur[g8][1] = hx[g8][1];
    if (c + 1 < nc) {  // next chunk's requests go out before this chunk's arithmetic
#pragma unroll
      for (int g8 = 0; g8 < TG; ++g8)
        hx[g8][0] = hp[g8][(c + 1) * 16], hx[g8][1] = hp[g8][(c + 1) * 16 + 1];
#pragma unroll
      for (int hh = 0; hh < NH; ++hh)
        wx[hh][0] = wp[hh][(c + 1) * 16], wx[hh][1] = wp[hh][(c + 1) * 16 + 1];
    }
#pragma unroll
    for (int g8 = 0; g8 < TG; ++g8) {
      const uint32_t hd[8] = {cur[g8][0].x, cur[g8][0].y, cur[g8][0].z, cur[g8][0].w,
                              cur[g8][1].x, cur[g8][1].y, cur[g8][1].z, cur[g8][1].w};
#pragma unroll
      for (int hh = 0; hh < NH; ++hh) {
        // four channels (one B pair) at a time: their products, then the two tree levels
        // inside the pair; node[p][i] = sum over channels 4p..4p+3 for router output 4*hh + i
        f32x4 node[4];
        const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int p = 0; p < 4; ++p) {
          const bf16x4 bb = router_bf16x4(hd[2 * p], hd[2 * p + 1]);
          const f32x4 t0 = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(
              router_bf16x4(aw[hh][4 * p + 0], 0u), bb, zero, 0, 0, 0);
          const f32x4 t1 = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(
              router_bf16x4(aw[hh][4 * p + 1], 0u), bb, zero, 0, 0, 0);
          const f32x4 t2 = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(
              router_bf16x4(0u, aw[hh][4 * p + 2]), bb, zero, 0, 0, 0);
          const f32x4 t3 = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(
              router_bf16x4(0u, aw[hh][4 * p + 3]), bb, zero, 0, 0, 0);
#pragma unroll
          for (int i = 0; i < 4; ++i) node[p][i] = (t0[i] + t1[i]) + (t2[i] + t3[i]);
        }
        const int rows = (G - 4 * hh) < 4 ? (G - 4 * hh) : 4;
#pragma unroll
        for (int i = 0; i < rows; ++i) {
          const float v = (node[0][i] + node[1][i]) + (node[2][i] + node[3][i]);
          acc[g8][hh][i] += chunk_tree_sum(v);
        }
      }
    }
  }

  if ((lane & 0x1c) != kChunkSumLanes) return;
#pragma unroll
  for (int g8 = 0; g8 < TG; ++g8) {
    const int t = t_first + 8 * g8;
    if (t >= N) continue;
    float o[4 * NH];
#pragma unroll
    for (int hh = 0; hh < NH; ++hh)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int g = 4 * hh + i;
        o[g] = g < G ? acc[g8][hh][i] + (bias ? bias[g] : 0.f) : 0.f;
      }
    for (int kvh = 0; kvh < Hkv; ++kvh) {
      float* dst = logits + (((size_t)b * Hkv + kvh) * N + t) * G;
      if constexpr (G >= 4) {
#pragma unroll
        for (int hh = 0; hh < NH; ++hh)
          *(f32x4*)(dst + 4 * hh) = f32x4{o[4 * hh], o[4 * hh + 1], o[4 * hh + 2], o[4 * hh + 3]};
      } else {
#pragma unroll
        for (int g = 0; g < G; ++g) dst[g] = o[g];
      }
    }
  }
}

int launch_router_logits(const void* h, const void* W, const float* bias, int bias_stride,
                         float* logits, int B, int Hkv, int N, int d_model, int G,
                         hipStream_t st) {
#define STC_ROUTER_CASE(GG)                                                                      \
  case GG: {                                                                                     \
    dim3 grid((N + RouterCfg<GG>::BLOCK_TOKENS - 1) / RouterCfg<GG>::BLOCK_TOKENS, B);           \
    router_logits_kernel<GG><<<grid, 256, 0, st>>>((const uint4*)h, (const uint4*)W, bias,       \
                                                   logits, N, d_model, Hkv, bias_stride);        \
    break;                                                                                       \
  }
  switch (G) {
    STC_ROUTER_CASE(1)
    STC_ROUTER_CASE(2)
    STC_ROUTER_CASE(4)
    STC_ROUTER_CASE(8)
    STC_ROUTER_CASE(16)
    default:
      return -1;
  }
#undef STC_ROUTER_CASE
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

}  // namespace stc
