// Routed decode attention over the selected pages (paper Sec. 3.3: softmax over
// full-width keys, values read from the group-packed store, dropped groups
// contribute nothing, no renormalisation).  Split over pages with online-softmax
// partials, merged inside the workgroup and then by a fixed-order combine.
//
// The R <= 16 query heads of a KV head share every K page and every packed V
// run, so both contractions are 16-wide dense tiles and run on the matrix cores
// (v_mfma_f32_16x16x32_bf16, float accumulation):
//   S^T[token][head] = K_page[token][:] . q[head][:]        (contract channels)
//   O^T[chan][head] += V~^T[chan][token] . P^T[token][head] (contract tokens)
// S^T leaves the first MFMA with tokens along the registers of a lane, which is
// the operand layout the second MFMA wants for P^T, so the weights never leave
// registers.  Each weight is split into two bf16 parts (p = hi + lo) so the
// product with V carries ~2^-17 relative error instead of bf16's 2^-9.
// V~^T (zero-filled, token-contiguous per channel) is gathered from an LDS copy
// of the page's packed run through a per-page table of group addresses.
#include "stc_common.hpp"
#include "stc_kernels.hpp"

namespace stc {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kNegBig = -1.0e30f;  // "no token seen yet" running maximum
constexpr int kAttnWaves = 4;        // wavefronts per workgroup

// Partial result of one (query head, split): [0] running max (base-2 logits),
// [1] sum of weights, [2 .. 2+D) weighted value sum.
__host__ __device__ constexpr int partial_stride(int D) { return D + 2; }

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  f32x2 v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));  // round to nearest even
}

__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int D>
struct AttnCfg {
  static constexpr int KC = D / 32;                  // QK MFMAs per page (32 channels each)
  static constexpr int CB = D / 16;                  // output channel blocks of 16
  static constexpr int UNITS = D / 8;                // 16-byte value units per token
  static constexpr int VBYTES = kPage * D * 2;       // largest packed run of a page
  static constexpr int TBYTES = kPage * UNITS * 4;   // address table of a page
  static constexpr int ZBYTES = 32;                  // zeros read for dropped groups
  static constexpr int WAVE_LDS = 2 * VBYTES + 2 * TBYTES + ZBYTES;
};

// One wavefront walks `ppw` pages of one stream, two at a time; the 4 wavefronts
// of a workgroup then merge their partial results in LDS.
template <int D>
__global__ __launch_bounds__(64 * kAttnWaves) void attn_mfma_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ K,
    const unsigned char* __restrict__ vpacked, const uint16_t* __restrict__ mask,
    const uint32_t* __restrict__ tok_off, const int32_t* __restrict__ page_idx,
    float* __restrict__ partial, float* __restrict__ out, int Hq, int Hkv, int N, int NP, int G,
    long long cap, int k_pages, int splits, int ppw) {
  using C = AttnCfg<D>;
  __shared__ __align__(16) unsigned char lds[kAttnWaves * C::WAVE_LDS];
  const int stream = blockIdx.y, split = blockIdx.x;
  const int b = stream / Hkv, kvh = stream % Hkv;
  const int R = Hq / Hkv;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r16 = lane & 15, kg = lane >> 4;  // MFMA row/column and k-group of this lane
  const int gd = D / G;
  const int gbytes = gd * 2;
  const float scale = kLog2e / sqrtf((float)D);

  unsigned char* wl = lds + wave * C::WAVE_LDS;
  const uint32_t zero_addr = 2 * C::VBYTES + 2 * C::TBYTES;  // offsets relative to wl
  if (lane < C::ZBYTES / 4) ((uint32_t*)(wl + zero_addr))[lane] = 0;

  // B operand of the QK product: this lane's 8 channels of head r16 for every 32-channel step
  uint4 qreg[C::KC];
#pragma unroll
  for (int j = 0; j < C::KC; ++j) {
    qreg[j] = make_uint4(0, 0, 0, 0);
    if (r16 < R)
      qreg[j] = *(const uint4*)(q + ((size_t)b * Hq + kvh * R + r16) * D + 32 * j + 8 * kg);
  }

  f32x4 acc[C::CB];
#pragma unroll
  for (int cb = 0; cb < C::CB; ++cb) acc[cb] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m_run = kNegBig, l_part = 0.f;

  const uint16_t* Ks = K + (size_t)stream * N * D;
  const uint16_t* mask_s = mask + (size_t)stream * N;
  const uint32_t* off_s = tok_off + (size_t)stream * (N + 1);
  const unsigned char* vs = vpacked + (size_t)stream * (size_t)cap * gbytes;
  const int32_t* pidx = page_idx + (size_t)stream * k_pages;

  const int pi0 = (split * kAttnWaves + wave) * ppw;
  const int pi1 = min(pi0 + ppw, k_pages);
  const int ttok = lane >> 2, tq = lane & 3;  // table-building role: token and quarter of its units
  const uint32_t j2 = (uint32_t)(r16 & 7) * 2;  // byte offset of this lane's channel inside a unit
  const int half = r16 >> 3;

  for (int pi = pi0; pi < pi1; pi += 2) {
    int pg[2];
    pg[0] = pidx[pi];
    pg[1] = (pi + 1 < pi1) ? pidx[pi + 1] : -1;
    uint4 kreg[2][C::KC];
    bool tokvalid[2];
#pragma unroll
    for (int x = 0; x < 2; ++x) {
      const bool pvalid = pg[x] >= 0 && pg[x] < NP;  // wave-uniform
      const int t0 = pvalid ? pg[x] * kPage : 0;
      // ---- K rows: lane (token r16, k-group kg) takes 16 bytes per 32-channel step
      tokvalid[x] = pvalid && (t0 + r16 < N);
#pragma unroll
      for (int j = 0; j < C::KC; ++j) {
        kreg[x][j] = make_uint4(0, 0, 0, 0);
        if (tokvalid[x])
          kreg[x][j] = *(const uint4*)(Ks + (size_t)(t0 + r16) * D + 32 * j + 8 * kg);
      }
      // ---- packed V run of the page -> LDS, plus the table of unit addresses
      unsigned char* vbuf = wl + x * C::VBYTES;
      uint32_t* tab = (uint32_t*)(wl + 2 * C::VBYTES + x * C::TBYTES);
      uint32_t mk = 0, off = 0;
      long long run0 = 0, run1 = 0;
      if (pvalid) {
        if (t0 + ttok < N) {
          mk = mask_s[t0 + ttok];
          off = off_s[t0 + ttok];
        }
        run0 = off_s[t0];
        run1 = off_s[min(t0 + kPage, N)];
      }
      run1 = min(run1, cap);
      long long rg = run1 - run0;               // groups of this page present in the store
      rg = max(0ll, min(rg, (long long)kPage * G));
      const int run_bytes = (int)rg * gbytes;
      const unsigned char* vsrc = vs + run0 * gbytes;
#pragma unroll
      for (int i = 0; i < C::VBYTES / 1024; ++i) {
        const int bo = (i * 64 + lane) * 16;
        if (bo < run_bytes) *(uint4*)(vbuf + bo) = *(const uint4*)(vsrc + bo);
      }
#pragma unroll
      for (int uu = 0; uu < C::UNITS / 4; ++uu) {
        const int u = tq * (C::UNITS / 4) + uu;      // 8-channel unit of token ttok
        const int g = (u * 8) / gd;
        const int within = u * 16 - g * gbytes;      // bytes into the group
        const long long slot = (long long)off - run0 + __popc(mk & ((1u << g) - 1u));
        const bool kept = ((mk >> g) & 1u) && slot >= 0 && slot < rg;
        const uint32_t ent = kept ? (uint32_t)(x * C::VBYTES + (int)slot * gbytes + within)
                                  : zero_addr;
        tab[((u & 1) * C::CB + (u >> 1)) * kPage + ttok] = ent;
      }
    }
    wave_lds_sync();

    // ---- logits S^T[token][head] for both pages
    float s[2][4];
    float mx = kNegBig;
#pragma unroll
    for (int x = 0; x < 2; ++x) {
      f32x4 sv = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int j = 0; j < C::KC; ++j)
        sv = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(kreg[x][j]), as_bf16x8(qreg[j]), sv,
                                                     0, 0, 0);
      // this lane holds tokens 4*kg + i of page x for head r16
      const bool pvalid = pg[x] >= 0 && pg[x] < NP;
      const int t0 = pvalid ? pg[x] * kPage : 0;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const bool tv = pvalid && (t0 + 4 * kg + i < N);
        s[x][i] = tv ? sv[i] * scale : kNegBig;
        mx = fmaxf(mx, s[x][i]);
      }
    }
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(m_run, mx);
    const float rescale = exp2f(m_run - m_new);
    m_run = m_new;
    float p[8];
    float psum = 0.f;
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        p[x * 4 + i] = s[x][i] > 0.5f * kNegBig ? exp2f(s[x][i] - m_new) : 0.f;
        psum += p[x * 4 + i];
      }
    l_part = l_part * rescale + psum;
#pragma unroll
    for (int cb = 0; cb < C::CB; ++cb) acc[cb] *= rescale;
    // weights as two bf16 parts; contraction index: (kg, e) e<4 page 0, e>=4 page 1
    uint4 phi, plo;
    {
      uint32_t h[4], l[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        h[r] = pack_bf16(p[2 * r], p[2 * r + 1]);
        l[r] = pack_bf16(p[2 * r] - bf16_lo(h[r]), p[2 * r + 1] - bf16_hi(h[r]));
      }
      phi = make_uint4(h[0], h[1], h[2], h[3]);
      plo = make_uint4(l[0], l[1], l[2], l[3]);
    }
    // ---- O^T += V~^T . P^T per 16-channel block
#pragma unroll
    for (int cb = 0; cb < C::CB; ++cb) {
      uint32_t a[4];
#pragma unroll
      for (int x = 0; x < 2; ++x) {
        const uint32_t* tab = (const uint32_t*)(wl + 2 * C::VBYTES + x * C::TBYTES);
        const uint4 e = *(const uint4*)(tab + (half * C::CB + cb) * kPage + 4 * kg);
        const uint32_t v0 = *(const uint16_t*)(wl + e.x + j2);
        const uint32_t v1 = *(const uint16_t*)(wl + e.y + j2);
        const uint32_t v2 = *(const uint16_t*)(wl + e.z + j2);
        const uint32_t v3 = *(const uint16_t*)(wl + e.w + j2);
        a[2 * x] = v0 | (v1 << 16);
        a[2 * x + 1] = v2 | (v3 << 16);
      }
      const bf16x8 av = as_bf16x8(make_uint4(a[0], a[1], a[2], a[3]));
      acc[cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, as_bf16x8(phi), acc[cb], 0, 0, 0);
      acc[cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, as_bf16x8(plo), acc[cb], 0, 0, 0);
    }
    wave_lds_sync();  // the next pair overwrites the staging buffers
  }

  // sum of weights of head r16 over this wavefront's tokens
  float l = l_part + __shfl_xor(l_part, 16);
  l += __shfl_xor(l, 32);

  // ---- merge the 4 wavefronts: each leaves (m, l, acc[R][D]) in its own LDS region
  float* macc = (float*)wl;                    // [16][D]
  float* mml = (float*)(wl + 16 * D * 4);      // [16][2]
  static_assert(16 * D * 4 + 16 * 2 * 4 <= C::WAVE_LDS, "merge buffer fits the staging area");
#pragma unroll
  for (int cb = 0; cb < C::CB; ++cb)
    *(f32x4*)(macc + r16 * D + cb * 16 + 4 * kg) = acc[cb];  // channels cb*16 + 4*kg + i
  if (kg == 0) {
    mml[r16 * 2] = m_run;
    mml[r16 * 2 + 1] = l;
  }
  __syncthreads();
  for (int i = threadIdx.x; i < R * D; i += 64 * kAttnWaves) {
    const int head = i / D, c = i % D;
    float mw[kAttnWaves], m = kNegBig;
#pragma unroll
    for (int w = 0; w < kAttnWaves; ++w) {
      mw[w] = ((const float*)(lds + w * C::WAVE_LDS + 16 * D * 4))[head * 2];
      m = fmaxf(m, mw[w]);
    }
    float lsum = 0.f, a = 0.f;
#pragma unroll
    for (int w = 0; w < kAttnWaves; ++w) {
      const float wgt = exp2f(mw[w] - m);
      lsum = fmaf(wgt, ((const float*)(lds + w * C::WAVE_LDS + 16 * D * 4))[head * 2 + 1], lsum);
      a = fmaf(wgt, ((const float*)(lds + w * C::WAVE_LDS))[head * D + c], a);
    }
    const size_t hf = (size_t)b * Hq + kvh * R + head;
    if (splits == 1) {
      out[hf * D + c] = lsum > 0.f ? a / lsum : 0.f;
    } else {
      float* pr = partial + (hf * splits + split) * partial_stride(D);
      pr[2 + c] = a;
      if (c == 0) {
        pr[0] = m;
        pr[1] = lsum;
      }
    }
  }
}

// Merge the split partials of one query head in ascending split order.  Each
// thread owns one channel; partials are fetched 8 splits at a time so the loads
// of a batch are in flight together.
template <int D>
__global__ __launch_bounds__(D) void attn_combine_kernel(const float* __restrict__ partial,
                                                         float* __restrict__ out, int splits) {
  constexpr int ST = partial_stride(D);
  const int head = blockIdx.x;
  const int c = threadIdx.x;
  const float* pr = partial + (size_t)head * splits * ST;
  float m = kNegBig;
  for (int s0 = 0; s0 < splits; s0 += 8) {
    float v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = s0 + i < splits ? pr[(s0 + i) * ST] : kNegBig;
#pragma unroll
    for (int i = 0; i < 8; ++i) m = fmaxf(m, v[i]);
  }
  float l = 0.f, a = 0.f;
  for (int s0 = 0; s0 < splits; s0 += 8) {
    float ms[8], ls[8], as[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const bool ok = s0 + i < splits;
      const float* ps = pr + (s0 + i) * ST;
      ms[i] = ok ? ps[0] : kNegBig;
      ls[i] = ok ? ps[1] : 0.f;
      as[i] = ok ? ps[2 + c] : 0.f;
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float w = exp2f(ms[i] - m);
      l = fmaf(w, ls[i], l);
      a = fmaf(w, as[i], a);
    }
  }
  out[(size_t)head * D + c] = l > 0.f ? a / l : 0.f;
}

// Pages per wavefront: as many as keep at least ~1024 workgroups in the grid
// (4 per CU), and never more than the pages there are.
static int attention_ppw(const stc_shape_t& s, int k_pages) {
  const int streams = s.B * s.Hkv;
  int ppw = 8;
  while (ppw > 2 &&
         (long long)streams * ((k_pages + kAttnWaves * ppw - 1) / (kAttnWaves * ppw)) < 1024)
    ppw >>= 1;
  while (ppw > 2 && kAttnWaves * (ppw / 2) >= k_pages) ppw >>= 1;  // no idle wavefronts
  return ppw;
}

int attention_splits(const stc_shape_t& s, int k_pages) {
  const int per_block = kAttnWaves * attention_ppw(s, k_pages);
  return (k_pages + per_block - 1) / per_block;
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
  const int ppw = attention_ppw(s, k_pages);
  const int splits = attention_splits(s, k_pages);
  dim3 grid(splits, streams);
  float* partial = (float*)ws;
  if (s.D == 128)
    attn_mfma_kernel<128><<<grid, 64 * kAttnWaves, 0, st>>>(
        (const uint16_t*)q, (const uint16_t*)K, (const unsigned char*)vpacked, mask, tok_off,
        page_idx, partial, out, s.Hq, s.Hkv, s.N, NP, s.G, (long long)s.v_cap_groups, k_pages,
        splits, ppw);
  else
    attn_mfma_kernel<64><<<grid, 64 * kAttnWaves, 0, st>>>(
        (const uint16_t*)q, (const uint16_t*)K, (const unsigned char*)vpacked, mask, tok_off,
        page_idx, partial, out, s.Hq, s.Hkv, s.N, NP, s.G, (long long)s.v_cap_groups, k_pages,
        splits, ppw);
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
