// Value-group router (App. B.1): one linear projection from the layer-input hidden state of a
// token to its G group logits, logits[t, g] = sum_c h[t, c] * W[g, c] (+ bias[g]).
//
// The masks are integer decisions taken on these logits, so the float summation order is
// fixed: d_model is cut into chunks of 128 adjacent channels, a chunk is summed as a balanced
// tree over adjacent channels, and the chunk sums are accumulated left to right; the bias is
// added last.  Products of two bf16 values are exact in float, so fusing a product into the
// following addition changes no bit.
//
// A row of 16 lanes owns one token: a lane holds 8 adjacent channels of the current chunk
// (one 16-byte load of h, one of each W row), sums them as a pair tree and the 16 lanes finish
// the tree with an xor butterfly.  A wavefront works on 4 tokens, a workgroup on 16.
#include "stc_common.hpp"
#include "stc_kernels.hpp"

namespace stc {

template <int G>
__global__ __launch_bounds__(256) void router_logits_kernel(const uint4* __restrict__ h,
                                                            const uint4* __restrict__ W,
                                                            const float* __restrict__ bias,
                                                            float* __restrict__ logits, int N,
                                                            int d_model, int Hkv) {
  const int b = blockIdx.y;
  const int sub = threadIdx.x & 15;
  const int t = blockIdx.x * 16 + (threadIdx.x >> 4);
  const int tc = min(t, N - 1);  // rows past the end repeat the last token (never stored)
  const int nc = d_model / 128;
  const int row16 = d_model / 8;  // 16-byte pieces per row
  const uint4* hp = h + ((size_t)b * N + tc) * row16 + sub;
  const uint4* wp = W + sub;
  float acc[G];
#pragma unroll
  for (int g = 0; g < G; ++g) acc[g] = 0.f;
  uint4 hv = hp[0];
  for (int c = 0; c < nc; ++c) {
    const uint4 cur = hv;
    if (c + 1 < nc) hv = hp[(c + 1) * 16];
    const uint32_t hw[4] = {cur.x, cur.y, cur.z, cur.w};
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const uint4 wv = wp[(size_t)g * row16 + c * 16];
      const uint32_t ww[4] = {wv.x, wv.y, wv.z, wv.w};
      float s2[4];
#pragma unroll
      for (int i = 0; i < 4; ++i)
        s2[i] = fmaf(bf16_hi(hw[i]), bf16_hi(ww[i]), bf16_lo(hw[i]) * bf16_lo(ww[i]));
      float u = (s2[0] + s2[1]) + (s2[2] + s2[3]);
      u = row_tree_sum<16>(u);
      acc[g] += u;
    }
  }
  if (t < N && sub < G) {
    // lane `sub` of the row stores group `sub` (every lane of the row holds all G sums)
    float v = 0.f;
#pragma unroll
    for (int g = 0; g < G; ++g)
      if (g == sub) v = acc[g];
    if (bias) v += bias[sub];
    for (int kvh = 0; kvh < Hkv; ++kvh)
      logits[(((size_t)b * Hkv + kvh) * N + t) * G + sub] = v;
  }
}

int launch_router_logits(const void* h, const void* W, const float* bias, float* logits, int B,
                         int Hkv, int N, int d_model, int G, hipStream_t st) {
  dim3 grid((N + 15) / 16, B);
#define STC_ROUTER_CASE(GG)                                                                     \
  case GG:                                                                                      \
    router_logits_kernel<GG><<<grid, 256, 0, st>>>((const uint4*)h, (const uint4*)W, bias,      \
                                                   logits, N, d_model, Hkv);                    \
    break;
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
