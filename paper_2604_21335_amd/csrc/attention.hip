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
// Both K and the routed (zero-filled) V of a page pass through a dense LDS tile.
#include "stc_common.hpp"
#include "stc_kernels.hpp"
#include "topk_block.hpp"

namespace stc {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
// 16-byte register values are native vectors: copies of the HIP uint4 struct go through
// memcpy, which can leave a register array in scratch memory
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kNegBig = -1.0e30f;  // "no token seen yet" running maximum
constexpr int kTailPage = 1 << 30;   // flag of a page slot that lies in the uncompressed tail

// Partial result of one (query head, split): [0] running max (base-2 logits),
// [1] sum of weights, [2 .. 2+D) weighted value sum.
__host__ __device__ constexpr int partial_stride(int D) { return D + 2; }

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

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
  static constexpr int KC = D / 32;         // QK MFMAs per page (32 channels each)
  static constexpr int CB = D / 16;         // output channels per lane and token (see PV below)
  static constexpr int LPR = D / 8;         // 16-byte pieces (lanes of a flat load) per token row
  static constexpr int NLD = kPage * D * 2 / 1024;  // flat 1 KiB loads per page of K (or of a full V run)
  static constexpr int ROW = D * 2 + 16;    // LDS bytes per token row of the K tile (padded)
  static constexpr int TILE = kPage * ROW;  // K tile of a page; reused for the page's packed V run
  static constexpr int META = 2 * TILE;     // per pair: 2 x 16 words (mask | relative offset << 16)
  static constexpr int ZERO = META + 128;   // 16 zero bytes: what dropped units read
  static constexpr int WAVE_LDS = ZERO + 16;
  // merge buffer of a wavefront: 16 head rows of D floats, each row padded by 4 floats so that
  // the 16 heads' 16-byte writes of one channel group fall into different banks
  static constexpr int MROW = D + 4;
  static constexpr int MML = 16 * MROW * 4;  // byte offset of the 16 (m, l) pairs behind it
  static_assert(MML + 16 * 2 * 4 <= 2 * TILE, "merge buffer fits the tiles");
};

// 16 zero bytes in device memory: where lanes beyond the end of a packed run read
__device__ u32x4 stc_zero16 = {0u, 0u, 0u, 0u};  // never written


// One wavefront takes one pair of page slots of one stream; the WAVES wavefronts of a workgroup
// then merge their partial results in LDS.
// Page slots are the selected pages of the compressed cache followed, with TAIL, by the pages
// of the uncompressed tail; kv_div query-head streams may share one KV head's cache.
//
// Per pair of pages:
//   1. K pages and packed V runs are read flat (every request is 1 KiB of adjacent
//      addresses, 16 bytes per lane) and staged in LDS.  Loading straight into the
//      MFMA operand layout, or unit by unit for V, turns each request into scattered
//      32..64-byte pieces and costs about 30 % of the achievable bandwidth.
//   2. QK: lane (token r16, k-group kg) reads 16 bytes per 32-channel step from the
//      K tile; S^T = K.q^T; online softmax per head; weights split into hi+lo bf16.
//   3. PV: lane (r16, kg) owns the CB adjacent channels r16*CB.. (one 16-byte value
//      unit for D = 128).  For each of its 8 tokens it computes where that unit sits
//      in the staged run (slot = offset of the token + rank of the group among the
//      kept ones) or takes zeros if the group was dropped, reads it, transposes the
//      8x8 block in registers with byte permutes and feeds MFMA row m of block cb
//      <-> channel m*CB + cb.  The accumulators of a lane cover channels 32*kg...
// Request order: page indices; masks/offsets and the K rows of the pair; then, as soon as
// the offsets are there, the pair's V runs.  All loads are unconditional (addresses of absent pages or
// tokens collapse to one valid location and the result is discarded) so that they
// stay in flight across the arithmetic.
// SELECT_IPT > 0: no page list is given; every workgroup first selects the stream's k pages
// from the page scores itself (the same selection as the stand-alone kernel, SELECT_IPT keys
// per thread), keeps the ones of its own split and writes them to the list.  Tail pages keep
// their slots behind the k selected ones.
// Arguments of the attention kernels (one struct, passed by value).
struct AttnParams {
  const uint16_t *q, *K;
  const unsigned char* vpacked;
  const uint16_t* mask;
  const uint32_t* tok_off;
  const int32_t* page_idx;
  float *partial, *out;
  int Hq, Hkv, N, NP, G;
  uint32_t cap;
  int k_pages, splits;
  const uint16_t *K_tail, *V_tail;
  int n_tail, tail_cap, kv_div;
  const uint16_t* page_heads;
  int Ncap;
  const float* sel_score;
  int32_t* sel_list;
  int nx;  // > 0: one-dimensional grid, stream s on the workgroups i with i % nx == s % nx
};

// The work of one workgroup: split `split` of stream `stream`.  `lds` = WAVES * WAVE_LDS bytes
// of shared memory.
template <int D, int WAVES, bool TAIL, int SELECT_IPT>
__device__ __forceinline__ void attn_block(const AttnParams& P, const int stream, const int split,
                                           unsigned char* lds) {
  using C = AttnCfg<D>;
  constexpr int ppw = 2;  // pages per wavefront
  const uint16_t* __restrict__ q = P.q;
  const uint16_t* __restrict__ K = P.K;
  const unsigned char* __restrict__ vpacked = P.vpacked;
  const uint16_t* __restrict__ mask = P.mask;
  const uint32_t* __restrict__ tok_off = P.tok_off;
  const int32_t* __restrict__ page_idx = P.page_idx;
  float* __restrict__ partial = P.partial;
  float* __restrict__ out = P.out;
  const int Hq = P.Hq, Hkv = P.Hkv, N = P.N, NP = P.NP, G = P.G;
  const uint32_t cap = P.cap;
  const int k_pages = P.k_pages, splits = P.splits;
  const uint16_t* __restrict__ K_tail = P.K_tail;
  const uint16_t* __restrict__ V_tail = P.V_tail;
  const int n_tail = P.n_tail, tail_cap = P.tail_cap, kv_div = P.kv_div;
  const uint16_t* __restrict__ page_heads = P.page_heads;
  const int Ncap = P.Ncap;
  const float* __restrict__ sel_score = P.sel_score;
  int32_t* __restrict__ sel_list = P.sel_list;
  const int b = stream / Hkv, kvh = stream % Hkv;
  const int R = Hq / Hkv;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r16 = lane & 15, kg = lane >> 4;  // MFMA row/column and k-group of this lane
  const int gd = D / G;
  const uint32_t gbytes = gd * 2;
  const int lg_upg = 31 - __clz(gd / 8);  // log2(16-byte units per group)
  const float scale = kLog2e / sqrtf((float)D);

  unsigned char* wl = lds + wave * C::WAVE_LDS;
  if (lane < 4) *(uint32_t*)(wl + C::ZERO + lane * 4) = 0;

  // per-stream bases (wave-uniform); everything below is addressed with 32-bit byte offsets.
  // kv_div > 1: the launch has one "stream" (page list, query, output) per query head and
  // kv_div of them share the cache of one KV head.
  const int kvs = stream / kv_div;
  const unsigned char* Ks = (const unsigned char*)K + (size_t)kvs * Ncap * D * 2;
  const unsigned char* mask_s = (const unsigned char*)mask + (size_t)kvs * Ncap * 2;
  const unsigned char* off_s = (const unsigned char*)tok_off + (size_t)kvs * (Ncap + 1) * 4;
  const unsigned char* vs = vpacked + (size_t)kvs * (size_t)cap * gbytes;
  // the uncompressed tail: dense K and V rows, i.e. a packed store in which every token kept
  // every group; its pages follow the selected ones in the list of page slots
  const unsigned char* Kts = (const unsigned char*)K_tail + (size_t)kvs * tail_cap * D * 2;
  const unsigned char* vts = (const unsigned char*)V_tail + (size_t)kvs * tail_cap * D * 2;
  const int tail_pages = TAIL ? (n_tail + kPage - 1) / kPage : 0;
  const uint32_t full_mask = (1u << G) - 1u;

  // this wavefront's pages: lane i holds page slot pi0 + i (-1: none; kTailPage | p: tail page)
  const int pi0 = (split * WAVES + wave) * ppw;
  const int npages = max(0, min(ppw, k_pages + tail_pages - pi0));
  int my_pg = -1;
  int my_heads = 0xffff;  // heads of the group that attend the page (all, unless a list is given)
  if (lane < npages) {
    const int slot = pi0 + lane;
    if (slot < k_pages) {
      my_pg = page_idx ? page_idx[(size_t)stream * k_pages + slot] : slot;  // no list: pages 0..
      // every page attended and the caller wants the list: each wavefront writes its own part
      if (SELECT_IPT == 0 && !page_idx && sel_list)
        sel_list[(size_t)stream * k_pages + slot] = slot;
      if (page_heads) my_heads = page_heads[(size_t)stream * k_pages + slot];
      if (my_pg < 0 || my_pg >= NP) my_pg = -1;
    } else {
      my_pg = kTailPage | (slot - k_pages);
    }
  }
  // (a workgroup whose page slots all lie in the uncompressed tail needs no list)
  if constexpr (SELECT_IPT > 0) if (split * WAVES * ppw < k_pages) {
    __shared__ int32_t s_pages[WAVES * ppw];
    if (threadIdx.x < WAVES * ppw) s_pages[threadIdx.x] = -1;
    __syncthreads();
    const int lo = split * WAVES * ppw;  // first list position of this workgroup
    int32_t* list = sel_list + (size_t)stream * k_pages;
    topk_block<SELECT_IPT, 64 * WAVES>(sel_score + (size_t)stream * NP, NP, k_pages,
                                       [&](int pos, int page) {
                                         const unsigned r = (unsigned)(pos - lo);
                                         if (r < (unsigned)(WAVES * ppw)) {
                                           s_pages[r] = page;
                                           list[pos] = page;
                                         }
                                       });
    __syncthreads();
    if (lane < npages && pi0 + lane < k_pages) my_pg = s_pages[wave * ppw + lane];
  }
  const int npairs = (npages + 1) / 2;

  // PV role: the value unit this lane reads for each of its tokens
  const uint32_t unit = (D == 128) ? r16 : (r16 >> 1);
  const uint32_t u_g = unit >> lg_upg;                    // its group
  const uint32_t u_below = (1u << u_g) - 1u;              // groups stored before it
  const uint32_t u_within = (unit - (u_g << lg_upg)) * 16 + ((D == 128) ? 0 : (r16 & 1) * 8);

  // lanes 0..15 carry the tokens of the pair's first page, 16..31 of its second page
  uint32_t mk, off, run0[2], run1[2];
  bool mvalid;
  u32x4 kreg[2][C::NLD];
  int pgs[2];

  // Lanes 0..15 fetch mask and offset of the tokens of the pair's first page, lanes
  // 16..31 of its second page; lanes 32 and 33 fetch the offset just past each page
  // (the end of its packed run).  Vector loads on purpose: scalar loads of these
  // scattered words queue up in the scalar cache for several microseconds.
  // Page slot -> page number, token limit of its store, and whether it is a tail page.
  auto is_tail = [&](int pg) { return TAIL && pg >= kTailPage; };  // never, if no tail is given
  auto page_no = [&](int pg) { return pg & (kTailPage - 1); };
  auto tok_lim = [&](int pg) { return (uint32_t)(is_tail(pg) ? n_tail : N); };
  uint32_t moi;   // token index behind off[] (tail pages derive their offsets from it)
  bool mtail;     // this lane's meta words belong to a tail page
  auto issue_meta = [&]() {
#pragma unroll
    for (int x = 0; x < 2; ++x) pgs[x] = __builtin_amdgcn_readlane(my_pg, x);
    const int pg = (lane & 1) ? pgs[1] : pgs[0];          // lanes 32, 33
    const int pgt = (lane & 16) ? pgs[1] : pgs[0];        // token lanes
    const uint32_t t = (pgt < 0 ? 0 : page_no(pgt) * kPage) + r16;
    const bool tv = lane < 32 && pgt >= 0 && t < tok_lim(pgt);
    const uint32_t tend =
        pg < 0 ? 0u : min((uint32_t)page_no(pg) * kPage + kPage, tok_lim(pg));
    const uint32_t oi = tv ? t : ((lane == 32 || lane == 33) ? tend : 0u);
    const bool tl = lane < 32 ? (pgt >= 0 && is_tail(pgt)) : (pg >= 0 && is_tail(pg));
    mvalid = tv;
    moi = oi;
    mtail = tl;
    // tail lanes read word 0 of the stream's arrays and replace the result later
    mk = *(const uint16_t*)(mask_s + ((tv && !tl) ? t : 0u) * 2);  // discarded if !tv
    off = *(const uint32_t*)(off_s + (tl ? 0u : oi) * 4);
  };
  // start and end of the packed runs of a pair (wave-uniform), once the offsets are there.
  // A tail token keeps every group and its G groups sit at token index * G.
  auto finish_meta = [&]() {
    if (mtail) {
      mk = full_mask;
      off = moi * G;
    }
#pragma unroll
    for (int x = 0; x < 2; ++x) {
      run0[x] = __builtin_amdgcn_readlane(off, 16 * x);  // token 0 of a page is valid
      run1[x] = __builtin_amdgcn_readlane(off, 32 + x);
    }
  };
  auto issue_k = [&]() {
#pragma unroll
    for (int x = 0; x < 2; ++x) {
      const int pg = pgs[x];
      const uint32_t t0 = pg < 0 ? 0 : page_no(pg) * kPage;
      const uint32_t lim = tok_lim(pg);
      const unsigned char* kb = (pg >= 0 && is_tail(pg)) ? Kts : Ks;  // wave-uniform
#pragma unroll
      for (int j = 0; j < C::NLD; ++j) {
        const uint32_t tok = (j * 64 + lane) / C::LPR;
        const bool tv = pg >= 0 && (t0 + tok < lim);
        // rows of absent tokens read the store's first bytes: their logits are discarded
        const uint32_t ko = tv ? t0 * (D * 2) + (j * 64 + lane) * 16 : 0;
        kreg[x][j] = *(const u32x4*)(kb + ko);
      }
    }
  };
  // Groups of a page present in the store (wave-uniform).
  auto run_groups = [&](int x) -> uint32_t {
    const uint32_t r0 = run0[x];
    const uint32_t store = is_tail(pgs[x]) ? (uint32_t)tail_cap * G : cap;
    const uint32_t r1 = pgs[x] < 0 ? 0u : min(run1[x], store);
    const uint32_t rg = r1 > r0 ? r1 - r0 : 0u;
    return min(rg, (uint32_t)(kPage * G));
  };
  // Packed V runs of a pair, flat; lanes past the end of a run read the zero line.
#define STC_ISSUE_V(vreg)                                                                      \
  static_for<0, 2>([&](auto x) {                                                               \
    const uint32_t rbytes = run_groups(x) * gbytes + vgate;                                \
    const unsigned char* vrun =                                                                \
        ((pgs[x] >= 0 && is_tail(pgs[x])) ? vts : vs) + (size_t)run0[x] * gbytes;  \
    static_for<0, C::NLD>([&](auto j) {                                                        \
      const uint32_t bo = (j * 64 + lane) * 16;                                                \
      /* one address computed with integer selects, so that it stays a single request */      \
      const uintptr_t a = bo < rbytes ? (uintptr_t)vrun + bo : (uintptr_t)&stc_zero16;         \
      vreg[x][j] = *(const __attribute__((address_space(1))) u32x4*)a; /* global, not flat */  \
    });                                                                                        \
  })

  f32x4 acc[C::CB];
#pragma unroll
  for (int cb = 0; cb < C::CB; ++cb) acc[cb] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m_run = kNegBig, l_part = 0.f;

  // The scheduling fences keep the request order stated above.
  issue_meta();
  __builtin_amdgcn_sched_barrier(0);
  issue_k();
  __builtin_amdgcn_sched_barrier(0);

  // B operand of the QK product: this lane's 8 channels of head r16 for every 32-channel step
  u32x4 qreg[C::KC];
  {
    const unsigned char* qs = (const unsigned char*)q + ((size_t)b * Hq + kvh * R) * D * 2;
    const uint32_t qo = ((r16 < R ? r16 : 0) * D + 8 * kg) * 2;
#pragma unroll
    for (int j = 0; j < C::KC; ++j)
      qreg[j] = *(const u32x4*)(qs + (qo + 64 * j));  // columns >= R repeat head 0, never used
  }
  __builtin_amdgcn_sched_barrier(0);

  // logits of a pair, online softmax; leaves the weights of the pair in phi/plo
  u32x4 phi, plo;
  auto qk_softmax = [&]() {
    // K rows of the pair -> LDS tiles (row stride ROW), then back in MFMA operand layout
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
      for (int j = 0; j < C::NLD; ++j)
        *(u32x4*)(wl + (x * C::TILE + ((j * 64 + lane) / C::LPR) * C::ROW +
                        (lane % C::LPR) * 16)) = kreg[x][j];
    wave_lds_sync();
    float s[2][4];
    float mx = kNegBig;
#pragma unroll
    for (int x = 0; x < 2; ++x) {
      f32x4 sv = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int j = 0; j < C::KC; ++j) {
        // A operand: token r16, channels 32*j + 8*kg .. +8 from the K tile
        const u32x4 a = *(const u32x4*)(wl + (x * C::TILE + r16 * C::ROW + (4 * j + kg) * 16));
        sv = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(a), as_bf16x8(qreg[j]), sv, 0, 0, 0);
      }
      // this lane holds tokens 4*kg + i of page x for head r16
      const int pg = pgs[x];
      const uint32_t t0 = pg < 0 ? 0 : page_no(pg) * kPage;
      const uint32_t lim = tok_lim(pg);
      // a head that did not select this page gives its tokens no weight
      const bool mine = (__builtin_amdgcn_readlane(my_heads, x) >> r16) & 1;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const bool tv = pg >= 0 && mine && (t0 + 4 * kg + i < lim);
        s[x][i] = tv ? sv[i] * scale : -INFINITY;  // weight of an absent token is exactly 0
        mx = fmaxf(mx, s[x][i]);
      }
    }
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(m_run, mx);
    const float rescale = __builtin_amdgcn_exp2f(m_run - m_new);
    m_run = m_new;
    float p[8];
    float psum = 0.f;
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        p[x * 4 + i] = __builtin_amdgcn_exp2f(s[x][i] - m_new);  // m_new is finite
        psum += p[x * 4 + i];
      }
    l_part = l_part * rescale + psum;
    // weights as two bf16 parts; contraction index: (kg, e) e<4 page 0, e>=4 page 1
    uint32_t h[4], l[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      h[r] = pack_bf16(p[2 * r], p[2 * r + 1]);
      l[r] = pack_bf16(p[2 * r] - bf16_lo(h[r]), p[2 * r + 1] - bf16_hi(h[r]));
    }
    phi = u32x4{h[0], h[1], h[2], h[3]};
    plo = u32x4{l[0], l[1], l[2], l[3]};
  };

  // packed runs of a pair -> LDS, then O^T += V~^T . P^T
#define STC_PV(vreg)                                                                           \
  {                                                                                            \
    wave_lds_sync(); /* the K tiles have been read */                                          \
    static_for<0, 2>([&](auto x) {                                                             \
      static_for<0, C::NLD>([&](auto j) {                                                      \
        *(u32x4*)(wl + (x * C::TILE + (j * 64 + lane) * 16)) = vreg[x][j];                     \
      });                                                                                      \
    });                                                                                        \
    if (lane < 32) { /* token lane: kept-group mask and offset relative to the run */         \
      const uint32_t r0 = (lane & 16) ? run0[1] : run0[0];                             \
      const uint32_t rel = min(off - r0, 0xffffu);                                         \
      *(uint32_t*)(wl + C::META + lane * 4) = (mvalid ? mk : 0u) | (rel << 16);        \
    }                                                                                          \
    wave_lds_sync();                                                                           \
    /* t[e]: channels r16*CB .. +CB of token e of this lane's k-group (e < 4: page 0) */       \
    uint32_t t[8][C::CB / 2];                                                                  \
    _Pragma("unroll") for (int x = 0; x < 2; ++x) {                                            \
      const uint32_t rg = run_groups(x);                                                   \
      const u32x4 mt = *(const u32x4*)(wl + C::META + x * 64 + kg * 16);                       \
      _Pragma("unroll") for (int i = 0; i < 4; ++i) {                                          \
        const uint32_t m = mt[i] & 0xffffu;                                                    \
        const uint32_t slot = (mt[i] >> 16) + __popc(m & u_below);                             \
        const bool kept = ((m >> u_g) & 1u) && slot < rg;                                      \
        const uint32_t a = kept ? x * C::TILE + slot * gbytes + u_within : (uint32_t)C::ZERO;  \
        if constexpr (D == 128) {                                                              \
          const u32x4 v = *(const u32x4*)(wl + a);                                             \
          t[x * 4 + i][0] = v.x, t[x * 4 + i][1] = v.y, t[x * 4 + i][2] = v.z,                 \
                       t[x * 4 + i][3] = v.w;                                                  \
        } else {                                                                               \
          const u32x2 v = *(const u32x2*)(wl + a);                                             \
          t[x * 4 + i][0] = v.x, t[x * 4 + i][1] = v.y;                                        \
        }                                                                                      \
      }                                                                                        \
    }                                                                                          \
    _Pragma("unroll") for (int cb = 0; cb < C::CB; ++cb) {                                     \
      const uint32_t sel = (cb & 1) ? 0x07060302u : 0x05040100u;                               \
      uint32_t a[4];                                                                           \
      _Pragma("unroll") for (int r = 0; r < 4; ++r) a[r] =                                     \
          __builtin_amdgcn_perm(t[2 * r + 1][cb >> 1], t[2 * r][cb >> 1], sel);                \
      const bf16x8 av = as_bf16x8(u32x4{a[0], a[1], a[2], a[3]});                              \
      acc[cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, as_bf16x8(phi), acc[cb], 0, 0, 0); \
      acc[cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, as_bf16x8(plo), acc[cb], 0, 0, 0); \
    }                                                                                          \
    wave_lds_sync(); /* the next pair overwrites the tiles */                                  \
  }

  if (npairs > 0) {
    // The value requests of a pair are held back until its masks/offsets have arrived:
    // a wavefront then has one pair of K pages or one pair of V runs plus the next K
    // pages outstanding, which keeps the chip-wide volume of outstanding requests near
    // what the memory system sustains.  (Requesting everything at once is slower.)
    finish_meta();
    uint32_t vgate;
    asm volatile("v_and_b32 %0, 0, %1" : "=v"(vgate) : "v"(off ^ mk));  // 0, after they arrive
    u32x4 vregA[2][C::NLD];
    STC_ISSUE_V(vregA);
    __builtin_amdgcn_sched_barrier(0);
    qk_softmax();
    __builtin_amdgcn_sched_barrier(0);
    STC_PV(vregA);
  }

  // sum of weights of head r16 over this wavefront's tokens
  float l = l_part + __shfl_xor(l_part, 16);
  l += __shfl_xor(l, 32);

  // ---- merge the workgroup's wavefronts: each leaves (m, l, acc[16][D]) in its own LDS region.
  // acc[cb][i] of lane (head r16, kg) is channel (4*kg + i)*CB + cb.
  float* macc = (float*)wl;             // [16][MROW]
  float* mml = (float*)(wl + C::MML);    // [16][2]
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    float* dst = macc + r16 * C::MROW + (4 * kg + i) * C::CB;
#pragma unroll
    for (int c4 = 0; c4 < C::CB / 4; ++c4)
      *(f32x4*)(dst + 4 * c4) = f32x4{acc[4 * c4][i], acc[4 * c4 + 1][i], acc[4 * c4 + 2][i],
                                      acc[4 * c4 + 3][i]};
  }
  if (kg == 0) {
    mml[r16 * 2] = m_run;
    mml[r16 * 2 + 1] = l;
  }
  __syncthreads();
  for (int i = threadIdx.x; i < R * D; i += 64 * WAVES) {
    const int head = i / D, c = i % D;
    float mw[WAVES], m = kNegBig;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) {
      mw[w] = ((const float*)(lds + w * C::WAVE_LDS + C::MML))[head * 2];
      m = fmaxf(m, mw[w]);
    }
    float lsum = 0.f, a = 0.f;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) {
      const float wgt = __builtin_amdgcn_exp2f(mw[w] - m);
      lsum = fmaf(wgt, ((const float*)(lds + w * C::WAVE_LDS + C::MML))[head * 2 + 1], lsum);
      a = fmaf(wgt, ((const float*)(lds + w * C::WAVE_LDS))[head * C::MROW + c], a);
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

#undef STC_ISSUE_V
#undef STC_PV

template <int D, int WAVES, bool TAIL, int SELECT_IPT>
__global__ __launch_bounds__(64 * WAVES) void attn_mfma_kernel(const AttnParams P) {
  extern __shared__ __align__(16) unsigned char lds[];  // WAVES * AttnCfg<D>::WAVE_LDS bytes
  int stream = blockIdx.y, split = blockIdx.x;
  if (P.nx > 0) {
    // Workgroup i of a launch runs on XCD i % 8: all workgroups of a stream get the same i % nx,
    // so that what they share (the stream's page scores, its query) passes through one L2
    const int x = blockIdx.x % P.nx, slot = blockIdx.x / P.nx;
    stream = (slot / P.splits) * P.nx + x;
    split = slot % P.splits;
  }
  attn_block<D, WAVES, TAIL, SELECT_IPT>(P, stream, split, lds);
}

// Merge the split partials of one query head in ascending split order.  Each
// thread owns one channel; partials are fetched 8 splits at a time (one round of
// loads for up to 8 splits) and folded in with a running maximum.
template <int D>
__global__ __launch_bounds__(D) void attn_combine_kernel(const float* __restrict__ partial,
                                                         float* __restrict__ out, int splits) {
  constexpr int ST = partial_stride(D);
  const int head = blockIdx.x;
  const int c = threadIdx.x;
  const float* pr = partial + (size_t)head * splits * ST;
  float m = kNegBig, l = 0.f, a = 0.f;
  for (int s0 = 0; s0 < splits; s0 += 8) {
    float ms[8], ls[8], as[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float* ps = pr + min(s0 + i, splits - 1) * ST;
      ms[i] = ps[0], ls[i] = ps[1], as[i] = ps[2 + c];
    }
    float mb = m;
#pragma unroll
    for (int i = 0; i < 8; ++i) mb = fmaxf(mb, s0 + i < splits ? ms[i] : kNegBig);
    const float r = __builtin_amdgcn_exp2f(m - mb);
    l *= r, a *= r, m = mb;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float w = s0 + i < splits ? __builtin_amdgcn_exp2f(ms[i] - mb) : 0.f;
      l = fmaf(w, ls[i], l);
      a = fmaf(w, as[i], a);
    }
  }
  out[(size_t)head * D + c] = l > 0.f ? a / l : 0.f;
}

// Shape of the launch: wavefronts per workgroup, pages per wavefront, workgroups per stream.
// Measured on the paper-shaped workloads, one pair of pages per wavefront and 8 wavefronts
// per workgroup is the fastest shape whenever it still gives every CU a workgroup; with few
// streams, workgroups of 4 wavefronts (twice as many of them) fill the chip better.  The
// two-pairs-per-wavefront form of the kernel is kept for tuning builds only.
struct AttnPlan {
  int waves, ppw, splits;
};

// Few streams of 2049..8192 pages (a long context at batch 1) can select inside the attention
// kernel, 16 keys per thread: that wants workgroups of 512 threads, so the plan (which depends
// on the shape alone: the two-call step gives the same bits) uses them there.
static bool long_select_shape(const stc_shape_t& s, int k_pages) {
  const int NP = (s.N + kPage - 1) / kPage;
  return NP > 2048 && NP <= 8192 && k_pages > 8 &&
         (long long)s.B * s.Hkv * ((k_pages + 15) / 16) <= 128;
}

static AttnPlan attention_plan(const stc_shape_t& s, int k_pages) {
  const int streams = s.B * s.Hkv;
  AttnPlan p{8, 2, 0};
  if (k_pages <= 8 || (long long)streams * ((k_pages + 15) / 16) < 256) p.waves = 4;
  if (long_select_shape(s, k_pages)) p.waves = 8;
  p.splits = (k_pages + p.waves * p.ppw - 1) / (p.waves * p.ppw);
  return p;
}

int attention_splits(const stc_shape_t& s, int k_pages) { return attention_plan(s, k_pages).splits; }

// The per-query-head form is the ordinary launch on a shape with one KV head per query head
// (the kernel then maps kv_div of those onto one cache).
static stc_shape_t launch_shape(const stc_shape_t& s, bool per_head) {
  stc_shape_t t = s;
  if (per_head) t.Hkv = s.Hq;
  return t;
}

// Room for the split partials of any launch over at most k_pages page slots: the plan with
// the most workgroups per stream (4 wavefronts of 2 pages each), so that the size never
// shrinks when k_pages grows and a buffer sized for the largest count serves every smaller one.
size_t attention_ws_bytes(const stc_shape_t& s0, int k_pages, bool per_head) {
  const stc_shape_t s = launch_shape(s0, per_head);
  const int splits = (k_pages + 7) / 8;
  if (splits <= 1) return 0;
  return (size_t)s.B * s.Hq * splits * partial_stride(s.D) * sizeof(float);
}

namespace {

struct AttnLaunch {
  AttnParams p;
  dim3 grid;
  hipStream_t st;
};

template <int D, int WAVES, bool TAIL, int SELECT_IPT>
int attn_go(const AttnLaunch& a) {
  // workgroups of 8 wavefronts at D = 128 need more than the default 64 KiB of LDS
  constexpr int lds_bytes = WAVES * AttnCfg<D>::WAVE_LDS;
  static std::atomic<uint64_t> allowed{0};
  if (!allow_dynamic_lds((const void*)attn_mfma_kernel<D, WAVES, TAIL, SELECT_IPT>, lds_bytes,
                         allowed))
    return -1;
  attn_mfma_kernel<D, WAVES, TAIL, SELECT_IPT><<<a.grid, 64 * WAVES, lds_bytes, a.st>>>(a.p);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

template <int D>
int attn_dispatch(const AttnLaunch& a, const AttnPlan& plan, bool tail, bool select) {
  if (select) {  // selection inside the kernel: 2048 (8192) keys over the workgroup's threads
    if (a.p.NP > 2048) return tail ? attn_go<D, 8, true, 16>(a) : attn_go<D, 8, false, 16>(a);
    if (plan.waves == 8)
      return tail ? attn_go<D, 8, true, 4>(a) : attn_go<D, 8, false, 4>(a);
    return tail ? attn_go<D, 4, true, 8>(a) : attn_go<D, 4, false, 8>(a);
  }
  if (plan.waves == 8) return tail ? attn_go<D, 8, true, 0>(a) : attn_go<D, 8, false, 0>(a);
  return tail ? attn_go<D, 4, true, 0>(a) : attn_go<D, 4, false, 0>(a);
}

}  // namespace

// Selection inside the attention kernel repeats a stream's top-k in each of its workgroups.
// Measured against the separate selection launch it is faster while all workgroups are
// resident at once (two per compute unit) and a stream's keys fit four per thread, and
// slower beyond (the repeated prologue then delays a second round of workgroups).
bool attention_can_select(const stc_shape_t& s, int k_pages, int tail_pages) {
  const int NP = (s.N + kPage - 1) / kPage;
  if (k_pages >= NP) return false;
  // long streams: only where the launch is latency-bound anyway (few workgroups)
  if (NP > 2048) return long_select_shape(s, k_pages + tail_pages);
  // the workgroups that select must all be resident at once; those that hold only pages of
  // the tail skip the selection and may come in a second round
  const AttnPlan p = attention_plan(s, k_pages + tail_pages);
  const long long streams = (long long)s.B * s.Hkv;
  const int per_wg = p.waves * p.ppw;
  return streams * ((k_pages + per_wg - 1) / per_wg) <= 512 && streams * p.splits <= 768;
}

int launch_attention(const stc_shape_t& s0, const void* q, const void* K, const void* vpacked,
                     const uint16_t* mask, const uint32_t* tok_off, const int32_t* page_idx,
                     int k_pages, const void* K_tail, const void* V_tail, int n_tail, int tail_cap,
                     bool per_head, const uint16_t* page_heads, const float* sel_score,
                     int32_t* sel_list, float* out, void* ws, hipStream_t st) {
  const stc_shape_t s = launch_shape(s0, per_head);
  const int NP = (s.N + kPage - 1) / kPage;
  const int streams = s.B * s.Hkv;
  const int tail_pages = (n_tail + kPage - 1) / kPage;
  if (tail_pages == 0) K_tail = V_tail = K;  // any valid address: never read
  const AttnPlan plan = attention_plan(s, k_pages + tail_pages);
  AttnLaunch a{{(const uint16_t*)q, (const uint16_t*)K, (const unsigned char*)vpacked, mask, tok_off,
                page_idx, (float*)ws, out, s.Hq, s.Hkv, s.N, NP, s.G, (uint32_t)s.v_cap_groups,
                k_pages, plan.splits, (const uint16_t*)K_tail, (const uint16_t*)V_tail, n_tail,
                tail_cap, per_head ? s0.Hq / s0.Hkv : 1, page_heads, token_cap(s), sel_score,
                sel_list, 0},
               dim3(plan.splits, streams), st};
  if (sel_score && (NP > 8192 || per_head || page_heads)) return -1;
  // with the selection inside, the workgroups of a stream all read the stream's scores: keep
  // them on one XCD (measured on the headline shape: 34.2 against 34.6 us per step)
  constexpr int kXcds = 8;
  if (sel_score && plan.splits > 1 && streams % kXcds == 0) {
    a.p.nx = kXcds;
    a.grid = dim3(plan.splits * streams, 1);
  }
  const int rc = s.D == 128 ? attn_dispatch<128>(a, plan, tail_pages > 0, sel_score != nullptr)
                            : attn_dispatch<64>(a, plan, tail_pages > 0, sel_score != nullptr);
  if (rc) return -1;
  if (plan.splits > 1) {
    if (s.D == 128)
      attn_combine_kernel<128><<<s.B * s.Hq, 128, 0, st>>>(a.p.partial, out, plan.splits);
    else
      attn_combine_kernel<64><<<s.B * s.Hq, 64, 0, st>>>(a.p.partial, out, plan.splits);
    if (hipGetLastError() != hipSuccess) return -1;
  }
  return 0;
}

// New token of every stream -> row n_tail of the stream's uncompressed tail (K and V).
template <int D>
__global__ __launch_bounds__(256) void append_tail_kernel(const uint4* __restrict__ k_new,
                                                          const uint4* __restrict__ v_new,
                                                          uint4* __restrict__ K_tail,
                                                          uint4* __restrict__ V_tail, int streams,
                                                          int n_tail, int tail_cap) {
  constexpr int LPR = D / 8;  // 16-byte pieces per row
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= streams * LPR) return;
  const int stream = i / LPR, piece = i % LPR;
  const size_t dst = ((size_t)stream * tail_cap + n_tail) * LPR + piece;
  K_tail[dst] = k_new[i];
  V_tail[dst] = v_new[i];
}

int launch_append_tail(const stc_shape_t& s, const void* k_new, const void* v_new, void* K_tail,
                       void* V_tail, int n_tail, int tail_cap, hipStream_t st) {
  const int streams = s.B * s.Hkv;
  const int n = streams * (s.D / 8);
  if (s.D == 128)
    append_tail_kernel<128><<<(n + 255) / 256, 256, 0, st>>>(
        (const uint4*)k_new, (const uint4*)v_new, (uint4*)K_tail, (uint4*)V_tail, streams, n_tail,
        tail_cap);
  else
    append_tail_kernel<64><<<(n + 255) / 256, 256, 0, st>>>(
        (const uint4*)k_new, (const uint4*)v_new, (uint4*)K_tail, (uint4*)V_tail, streams, n_tail,
        tail_cap);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

}  // namespace stc
