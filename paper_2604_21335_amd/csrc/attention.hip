// Routed decode attention over the selected pages (paper Sec. 3.3: softmax over
// full-width keys, values read from the group-packed store, dropped groups
// contribute nothing, no renormalisation).  Split over pages with per-split
// online-softmax partials and a fixed-order combine.
#include "stc_common.hpp"
#include "stc_kernels.hpp"

namespace stc {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kNegBig = -1.0e30f;  // "no token seen yet" running maximum

// Partial result of one (query head, split): [0] running max (base-2 logits),
// [1] sum of weights, [2 .. 2+D) weighted value sum.
__host__ __device__ constexpr int partial_stride(int D) { return D + 2; }

// ---------------------------------------------------------------------------
// General kernel: one wavefront per (query head, split); the R wavefronts of a
// block share the stream's pages.
//   QK: a page of K is 16*D*2 contiguous bytes; load instruction j takes bytes
//       [j*1024, (j+1)*1024) of it, 16 bytes per lane, so lane l holds 8
//       channels (l % (D/8))*8.. of token j*TPI + l/(D/8).  The D/8 lanes of a
//       token are reduced with DPP; every lane of the token ends with its logit.
//   PV: lane l owns channels 2l, 2l+1 (D = 128) of the output; for every token
//       of the page it fetches its dword of the token's packed group if the
//       group was kept.
// ---------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(1024) void attn_split_kernel(
    const uint4* __restrict__ q, const uint4* __restrict__ K, const uint32_t* __restrict__ vpacked,
    const uint16_t* __restrict__ mask, const uint32_t* __restrict__ tok_off,
    const int32_t* __restrict__ page_idx, float* __restrict__ partial, float* __restrict__ out,
    int Hq, int Hkv, int N, int NP, int G, long long cap, int k_pages, int splits,
    int pages_per_split) {
  constexpr int LPT = D / 8;         // lanes per token row
  constexpr int TPI = 64 / LPT;      // tokens per load instruction
  constexpr int NJ = kPage / TPI;    // load instructions per page
  constexpr int CL = D / 2;          // lanes that own output channels (2 each)
  const int stream = blockIdx.y;
  const int split = blockIdx.x;
  const int b = stream / Hkv, kvh = stream % Hkv;
  const int R = Hq / Hkv;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int head = b * Hq + kvh * R + wave;  // flat (b, query head)
  const int sub = lane % LPT, row = lane / LPT;
  const int gd = D / G;
  const float scale = kLog2e / sqrtf((float)D);

  float qf[8];
  {
    const uint4 v = q[(size_t)head * LPT + sub];
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      qf[2 * i] = bf16_lo(w[i]) * scale;
      qf[2 * i + 1] = bf16_hi(w[i]) * scale;
    }
  }
  // value side: which group this lane's two channels belong to
  const bool vlane = lane < CL;
  const int g = vlane ? (2 * lane) / gd : 0;
  const int within = vlane ? (2 * lane) % gd : 0;  // channel offset inside the group
  const uint32_t below = (1u << g) - 1u;
  const uint32_t* vbase = vpacked + (size_t)stream * (size_t)cap * (gd / 2);

  float m_run = kNegBig, l_part = 0.f, acc0 = 0.f, acc1 = 0.f;

  const int pi0 = split * pages_per_split;
  const int pi1 = min(pi0 + pages_per_split, k_pages);
  for (int pi = pi0; pi < pi1; ++pi) {
    const int p = page_idx[(size_t)stream * k_pages + pi];
    if (p < 0 || p >= NP) continue;  // wave-uniform
    const int t0 = p * kPage;
    // per-token mask and offset of the page, one token per lane (lanes 0..15)
    uint32_t mk = 0, off = 0;
    if (lane < kPage && t0 + lane < N) {
      mk = mask[(size_t)stream * N + t0 + lane];
      off = tok_off[(size_t)stream * (N + 1) + t0 + lane];
    }
    // ---- logits
    const uint4* kp = K + ((size_t)stream * N + t0) * LPT;
    float s[NJ];
    float m_page = kNegBig;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const int tok = j * TPI + row;
      const bool valid = t0 + tok < N;
      float d = 0.f;
      if (valid) {
        const uint4 v = kp[j * 64 + lane];
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          d = fmaf(qf[2 * i], bf16_lo(w[i]), d);
          d = fmaf(qf[2 * i + 1], bf16_hi(w[i]), d);
        }
      }
      d = row_tree_sum<LPT>(d);
      s[j] = valid ? d : kNegBig;
      m_page = fmaxf(m_page, s[j]);
    }
    // maximum over the page: across the token rows of the wavefront
    for (int dlt = LPT; dlt < 64; dlt <<= 1) m_page = fmaxf(m_page, __shfl_xor(m_page, dlt));
    const float m_new = fmaxf(m_run, m_page);
    const float rescale = exp2f(m_run - m_new);
    m_run = m_new;
    float pw[NJ];
    float psum = 0.f;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      pw[j] = s[j] > 0.5f * kNegBig ? exp2f(s[j] - m_new) : 0.f;
      psum += pw[j];
    }
    l_part = l_part * rescale + psum;  // this lane's token row only
    acc0 *= rescale;
    acc1 *= rescale;
    // ---- values: issue the page's loads, then accumulate
    uint32_t vv[kPage];
#pragma unroll
    for (int tt = 0; tt < kPage; ++tt) {
      const uint32_t mt = __builtin_amdgcn_readlane(mk, tt);
      const uint32_t ot = __builtin_amdgcn_readlane(off, tt);
      const long long slot = (long long)ot + __popc(mt & below);
      vv[tt] = 0;
      if (vlane && ((mt >> g) & 1u) && slot < cap) vv[tt] = vbase[slot * (gd / 2) + within / 2];
    }
#pragma unroll
    for (int tt = 0; tt < kPage; ++tt) {
      const float pt = readlane_f32(pw[tt / TPI], (tt % TPI) * LPT);
      acc0 = fmaf(pt, bf16_lo(vv[tt]), acc0);
      acc1 = fmaf(pt, bf16_hi(vv[tt]), acc1);
    }
  }
  // sum of weights: one lane per token row holds that row's share
  float l = (sub == 0) ? l_part : 0.f;
  for (int dlt = 32; dlt >= 1; dlt >>= 1) l += __shfl_xor(l, dlt);

  if (splits == 1) {
    if (vlane) {
      const float inv = l > 0.f ? 1.f / l : 0.f;
      float2* o = (float2*)(out + (size_t)head * D) + lane;
      *o = make_float2(acc0 * inv, acc1 * inv);
    }
  } else {
    float* pr = partial + ((size_t)head * splits + split) * partial_stride(D);
    if (lane == 0) {
      pr[0] = m_run;
      pr[1] = l;
    }
    if (vlane) {
      pr[2 + 2 * lane] = acc0;
      pr[2 + 2 * lane + 1] = acc1;
    }
  }
}

// Merge the split partials of one query head in ascending split order.
template <int D>
__global__ __launch_bounds__(D) void attn_combine_kernel(const float* __restrict__ partial,
                                                         float* __restrict__ out, int splits) {
  const int head = blockIdx.x;
  const int c = threadIdx.x;
  const float* pr = partial + (size_t)head * splits * partial_stride(D);
  float m = kNegBig;
  for (int s = 0; s < splits; ++s) m = fmaxf(m, pr[s * partial_stride(D)]);
  float l = 0.f, a = 0.f;
  for (int s = 0; s < splits; ++s) {
    const float* ps = pr + s * partial_stride(D);
    const float w = exp2f(ps[0] - m);
    l = fmaf(w, ps[1], l);
    a = fmaf(w, ps[2 + c], a);
  }
  out[(size_t)head * D + c] = l > 0.f ? a / l : 0.f;
}

int attention_splits(const stc_shape_t& s, int k_pages) {
  const int streams = s.B * s.Hkv;
  // enough workgroups to fill 256 CUs several times over, at least 2 pages each
  int want = (2048 + streams - 1) / streams;
  int max_splits = (k_pages + 1) / 2;
  int splits = want < 1 ? 1 : want;
  if (splits > max_splits) splits = max_splits;
  if (splits < 1) splits = 1;
  const int pps = (k_pages + splits - 1) / splits;
  return (k_pages + pps - 1) / pps;  // no empty splits
}

size_t attention_ws_bytes(const stc_shape_t& s, int k_pages) {
  const int splits = attention_splits(s, k_pages);
  if (splits <= 1) return 0;
  return (size_t)s.B * s.Hq * splits * partial_stride(s.D) * sizeof(float);
}

int launch_attention(const stc_shape_t& s, const void* q, const void* K, const void* vpacked,
                     const uint16_t* mask, const uint32_t* tok_off, const int32_t* page_idx,
                     int k_pages, float* out, void* ws, hipStream_t st) {
  const int NP = (s.N + kPage - 1) / kPage;
  const int streams = s.B * s.Hkv;
  const int R = s.Hq / s.Hkv;
  const int splits = attention_splits(s, k_pages);
  const int pps = (k_pages + splits - 1) / splits;
  dim3 grid(splits, streams);
  float* partial = (float*)ws;
  if (s.D == 128)
    attn_split_kernel<128><<<grid, 64 * R, 0, st>>>(
        (const uint4*)q, (const uint4*)K, (const uint32_t*)vpacked, mask, tok_off, page_idx,
        partial, out, s.Hq, s.Hkv, s.N, NP, s.G, (long long)s.v_cap_groups, k_pages, splits, pps);
  else
    attn_split_kernel<64><<<grid, 64 * R, 0, st>>>(
        (const uint4*)q, (const uint4*)K, (const uint32_t*)vpacked, mask, tok_off, page_idx,
        partial, out, s.Hq, s.Hkv, s.N, NP, s.G, (long long)s.v_cap_groups, k_pages, splits, pps);
  if (hipGetLastError() != hipSuccess) return -1;
  if (splits > 1) {
    if (s.D == 128)
      attn_combine_kernel<128><<<s.B * s.Hq, 128, 0, st>>>(partial, out, splits);
    else
      attn_combine_kernel<64><<<s.B * s.Hq, 64, 0, st>>>(partial, out, splits);
    if (hipGetLastError() != hipSuccess) return -1;
  }
  return 0;
}

}  // namespace stc
