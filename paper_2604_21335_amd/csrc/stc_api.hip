// C ABI of libstc: argument validation and dispatch to the kernel launchers.
#include "../../include/stc.h"
#include "stc_kernels.hpp"

namespace {

constexpr int kMaxGridY = 65535;

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

bool shape_ok(const stc_shape_t* s) {
  if (s->B < 1 || s->Hq < 1 || s->Hkv < 1 || s->N < 1) return false;
  if (s->Hq % s->Hkv != 0 || s->Hq / s->Hkv > 16) return false;
  if (s->D != 64 && s->D != 128) return false;
  if (s->P != 16) return false;
  if (s->G < 1 || s->G > 16 || (s->G & (s->G - 1)) != 0) return false;
  if (s->D % s->G != 0 || s->D / s->G < 8) return false;
  if (s->v_cap_groups < 0) return false;
  if (s->N_cap != 0 && (s->N_cap < s->N || (long long)s->N_cap > (1ll << 30))) return false;
  if ((long long)s->B * s->Hkv > kMaxGridY) return false;
  if ((long long)s->N > (1ll << 30)) return false;
  // the packed store is addressed with 32-bit group offsets
  if ((long long)stc::token_cap(*s) * s->G >= (1ll << 32)) return false;
  return true;
}

int num_pages(const stc_shape_t* s) { return (s->N + s->P - 1) / s->P; }

size_t select_ws_bytes(const stc_shape_t* s, bool per_head = false) {
  return (size_t)s->B * (per_head ? s->Hq : s->Hkv) * num_pages(s) * sizeof(float);
}

// Page scores at the front of the workspace of stc_decode_step, padded so that the attention
// partials behind them start on a 256-byte boundary.
size_t step_score_bytes(const stc_shape_t* s, int k_pages) {
  if (k_pages >= num_pages(s)) return 0;
  return (select_ws_bytes(s) + 255) & ~(size_t)255;
}

// Scratch memory of stc_decode_step_static: one copy per GPU, held until the process ends.
// In host code the array's name is only a handle; its address on the current device comes
// from hipGetSymbolAddress (static_scratch below) and is what the kernels are given.
static __device__ __align__(256) unsigned char scratch[STC_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

// Device address of `scratch` on the current device, looked up once per device.
void* static_scratch() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (p) return p;
  if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return nullptr;
  g_scratch_ptr[dev].store(p, std::memory_order_release);
  return p;
}

}  // namespace

extern "C" {

int stc_version(void) { return 2; }

const char* stc_status_string(int status) {
  switch (status) {
    case STC_OK: return "ok";
    case STC_ERR_NULL: return "a required pointer is NULL";
    case STC_ERR_SHAPE: return "shape or argument out of range";
    case STC_ERR_ALIGN: return "pointer is not 16-byte aligned";
    case STC_ERR_WORKSPACE: return "workspace missing or too small";
    case STC_ERR_LAUNCH: return "kernel launch failed";
    default: return "unknown status";
  }
}

size_t stc_workspace_bytes(const stc_shape_t* shape, int which_call, int k_pages) {
  if (!shape || !shape_ok(shape)) return 0;
  switch (which_call) {
    case STC_WS_ROUTE: return stc::route_ws_bytes(*shape);
    case STC_WS_SELECT: return k_pages >= num_pages(shape) ? 0 : select_ws_bytes(shape);
    case STC_WS_ATTENTION:
      if (k_pages < 1 || k_pages > num_pages(shape)) return 0;
      return stc::attention_ws_bytes(*shape, k_pages);
    case STC_WS_ATTENTION_TAIL:  // k_pages counts the tail's pages too
      if (k_pages < 1) return 0;
      return stc::attention_ws_bytes(*shape, k_pages);
    case STC_WS_SELECT_PER_HEAD:
      return k_pages >= num_pages(shape) ? 0 : select_ws_bytes(shape, true);
    case STC_WS_ATTENTION_PER_HEAD:
      if (k_pages < 1 || k_pages > num_pages(shape)) return 0;
      return stc::attention_ws_bytes(*shape, k_pages, true);
    case STC_WS_STEP:
      if (k_pages < 1 || k_pages > num_pages(shape)) return 0;
      return step_score_bytes(shape, k_pages) + stc::attention_ws_bytes(*shape, k_pages);
    case STC_WS_STEP_TAIL:  // k_pages counts the tail's pages too; scores always have room
      if (k_pages < 1) return 0;
      return step_score_bytes(shape, 0) + stc::attention_ws_bytes(*shape, k_pages);
    default: return 0;
  }
}

size_t stc_bounds_bytes(const stc_shape_t* shape) {
  if (!shape || !shape_ok(shape)) return 0;
  const size_t tiles = stc::bounds_tiles(stc::token_cap(*shape));
  return (size_t)shape->B * shape->Hkv * tiles * stc::kBoundsTilePages * shape->D * 4;
}

int stc_build_page_bounds(const stc_shape_t* shape, const void* K, void* bounds, void* stream) {
  if (!shape || !K || !bounds) return STC_ERR_NULL;
  if (!shape_ok(shape)) return STC_ERR_SHAPE;
  if (!aligned16(K) || !aligned16(bounds)) return STC_ERR_ALIGN;
  return stc::launch_bounds(*shape, K, bounds, (hipStream_t)stream) ? STC_ERR_LAUNCH : STC_OK;
}

int stc_route_and_pack_values(const stc_shape_t* shape, int mode, const void* V,
                              const float* logits, const uint8_t* kcount, int fixed_k,
                              const uint16_t* mask_in, uint16_t* mask, uint32_t* tok_off,
                              void* vpacked, int32_t* dev_status, void* ws, size_t ws_bytes,
                              void* stream) {
  if (!shape || !V || !mask || !tok_off || !vpacked) return STC_ERR_NULL;
  if (!shape_ok(shape)) return STC_ERR_SHAPE;
  const int base_mode = mode & ~STC_ROUTE_SHARED;
  if (base_mode == STC_ROUTE_TOPK) {
    if (!logits) return STC_ERR_NULL;
    if (!kcount && (fixed_k < 0 || fixed_k > shape->G)) return STC_ERR_SHAPE;
  } else if (base_mode == STC_ROUTE_GLOBAL) {
    if (!logits) return STC_ERR_NULL;
    if (fixed_k < 0 || fixed_k > shape->G) return STC_ERR_SHAPE;
  } else if (base_mode == STC_ROUTE_MASK) {
    if (!mask_in) return STC_ERR_NULL;
    if ((mode & STC_ROUTE_SHARED) && (const void*)mask_in == (const void*)mask) return STC_ERR_SHAPE;
  } else {
    return STC_ERR_SHAPE;
  }
  if (!aligned16(V) || !aligned16(vpacked) || !aligned16(mask) || !aligned16(tok_off) ||
      (logits && !aligned16(logits)) || (mask_in && !aligned16(mask_in)))
    return STC_ERR_ALIGN;
  if (!ws || ws_bytes < stc::route_ws_bytes(*shape) || !aligned16(ws)) return STC_ERR_WORKSPACE;
  return stc::launch_route_pack(*shape, mode, V, logits, kcount, fixed_k, mask_in, mask, tok_off,
                                vpacked, dev_status, ws, (hipStream_t)stream)
             ? STC_ERR_LAUNCH
             : STC_OK;
}

namespace {

int select_pages_impl(const stc_shape_t* shape, const void* q, const void* bounds, int k_pages,
                      int32_t* page_idx, float* page_score, void* ws, size_t ws_bytes,
                      bool per_head, void* stream) {
  if (!shape || !page_idx) return STC_ERR_NULL;
  if (!shape_ok(shape) || k_pages < 1) return STC_ERR_SHAPE;
  if (!aligned16(page_idx)) return STC_ERR_ALIGN;
  float* score = page_score;
  if (k_pages < num_pages(shape)) {
    if (!q || !bounds) return STC_ERR_NULL;
    if (!aligned16(q) || !aligned16(bounds) || (page_score && !aligned16(page_score)))
      return STC_ERR_ALIGN;
    if (!score) {
      if (!ws || ws_bytes < select_ws_bytes(shape, per_head) || !aligned16(ws))
        return STC_ERR_WORKSPACE;
      score = (float*)ws;
    }
  }
  return stc::launch_select(*shape, q, bounds, k_pages, page_idx, score, per_head,
                            (hipStream_t)stream)
             ? STC_ERR_LAUNCH
             : STC_OK;
}

}  // namespace

int stc_select_pages(const stc_shape_t* shape, const void* q, const void* bounds, int k_pages,
                     int32_t* page_idx, float* page_score, void* ws, size_t ws_bytes,
                     void* stream) {
  return select_pages_impl(shape, q, bounds, k_pages, page_idx, page_score, ws, ws_bytes, false,
                           stream);
}

int stc_select_pages_per_head(const stc_shape_t* shape, const void* q, const void* bounds,
                              int k_pages, int32_t* page_idx, float* page_score, void* ws,
                              size_t ws_bytes, void* stream) {
  return select_pages_impl(shape, q, bounds, k_pages, page_idx, page_score, ws, ws_bytes, true,
                           stream);
}

int stc_score_pages(const stc_shape_t* shape, const void* q, const void* bounds,
                    float* page_score, void* stream) {
  if (!shape || !q || !bounds || !page_score) return STC_ERR_NULL;
  if (!shape_ok(shape)) return STC_ERR_SHAPE;
  if (!aligned16(q) || !aligned16(bounds) || !aligned16(page_score)) return STC_ERR_ALIGN;
  return stc::launch_score(*shape, q, bounds, page_score, false, (hipStream_t)stream) ? STC_ERR_LAUNCH
                                                                               : STC_OK;
}

namespace {

// Argument checks of the attention calls; launches nothing.
int decode_attention_check(const stc_shape_t* shape, const void* q, const void* K,
                           const void* vpacked, const uint16_t* mask, const uint32_t* tok_off,
                           const int32_t* page_idx, int k_pages, const void* K_tail,
                           const void* V_tail, int n_tail, int tail_cap, bool per_head,
                           const float* out, const void* ws, size_t ws_bytes) {
  if (!shape || !q || !K || !vpacked || !mask || !tok_off || !out) return STC_ERR_NULL;
  if (!shape_ok(shape) || k_pages < 1 || k_pages > num_pages(shape) || shape->v_cap_groups < 1)
    return STC_ERR_SHAPE;
  // the kernels address one stream's keys and packed values with 32-bit byte offsets
  if ((long long)stc::token_cap(*shape) * shape->D * 2 >= (1ll << 32) ||
      shape->v_cap_groups * (shape->D / shape->G) * 2 >= (1ll << 32))
    return STC_ERR_SHAPE;
  if (n_tail < 0 || tail_cap < 0 || n_tail > tail_cap ||
      (long long)tail_cap * shape->D * 2 >= (1ll << 32))
    return STC_ERR_SHAPE;
  if (n_tail > 0 && (!K_tail || !V_tail)) return STC_ERR_NULL;
  if (!aligned16(q) || !aligned16(K) || !aligned16(vpacked) || !aligned16(mask) ||
      !aligned16(tok_off) || (page_idx && !aligned16(page_idx)) || !aligned16(out) ||
      (n_tail > 0 && (!aligned16(K_tail) || !aligned16(V_tail))))
    return STC_ERR_ALIGN;
  const int slots = k_pages + (n_tail + shape->P - 1) / shape->P;
  if (per_head && (long long)shape->B * shape->Hq > kMaxGridY) return STC_ERR_SHAPE;
  const size_t need = stc::attention_ws_bytes(*shape, slots, per_head);
  if (need && (!ws || ws_bytes < need || !aligned16(ws))) return STC_ERR_WORKSPACE;
  return STC_OK;
}

int decode_attention_impl(const stc_shape_t* shape, const void* q, const void* K,
                          const void* vpacked, const uint16_t* mask, const uint32_t* tok_off,
                          const int32_t* page_idx, int k_pages, const void* K_tail,
                          const void* V_tail, int n_tail, int tail_cap, bool per_head,
                          const uint16_t* page_heads, float* out, void* ws, size_t ws_bytes,
                          void* stream) {
  const int rc = decode_attention_check(shape, q, K, vpacked, mask, tok_off, page_idx, k_pages,
                                        K_tail, V_tail, n_tail, tail_cap, per_head, out, ws,
                                        ws_bytes);
  if (rc) return rc;
  return stc::launch_attention(*shape, q, K, vpacked, mask, tok_off, page_idx, k_pages, K_tail,
                               V_tail, n_tail, tail_cap, per_head, page_heads, nullptr, nullptr,
                               out, ws, (hipStream_t)stream)
             ? STC_ERR_LAUNCH
             : STC_OK;
}

}  // namespace

int stc_decode_attention(const stc_shape_t* shape, const void* q, const void* K,
                         const void* vpacked, const uint16_t* mask, const uint32_t* tok_off,
                         const int32_t* page_idx, int k_pages, float* out, void* ws,
                         size_t ws_bytes, void* stream) {
  return decode_attention_impl(shape, q, K, vpacked, mask, tok_off, page_idx, k_pages, nullptr,
                               nullptr, 0, 0, false, nullptr, out, ws, ws_bytes, stream);
}

int stc_decode_attention_per_head(const stc_shape_t* shape, const void* q, const void* K,
                                  const void* vpacked, const uint16_t* mask,
                                  const uint32_t* tok_off, const int32_t* page_idx, int k_pages,
                                  float* out, void* ws, size_t ws_bytes, void* stream) {
  return decode_attention_impl(shape, q, K, vpacked, mask, tok_off, page_idx, k_pages, nullptr,
                               nullptr, 0, 0, true, nullptr, out, ws, ws_bytes, stream);
}

int stc_decode_attention_tail(const stc_shape_t* shape, const void* q, const void* K,
                              const void* vpacked, const uint16_t* mask, const uint32_t* tok_off,
                              const int32_t* page_idx, int k_pages, const void* K_tail,
                              const void* V_tail, int n_tail, int tail_cap, float* out, void* ws,
                              size_t ws_bytes, void* stream) {
  return decode_attention_impl(shape, q, K, vpacked, mask, tok_off, page_idx, k_pages, K_tail,
                               V_tail, n_tail, tail_cap, false, nullptr, out, ws, ws_bytes, stream);
}

namespace {

// Selection followed by attention (with or without a tail) on one stream.  score_bytes =
// size of the score region at the front of the workspace.
int decode_step_impl(const stc_shape_t* shape, const void* q, const void* bounds, const void* K,
                     const void* vpacked, const uint16_t* mask, const uint32_t* tok_off,
                     int k_pages, const void* K_tail, const void* V_tail, int n_tail,
                     int tail_cap, int32_t* page_idx, float* out, void* ws, size_t ws_bytes,
                     size_t score_bytes, void* stream) {
  if (!shape || !q || !bounds || !page_idx) return STC_ERR_NULL;
  if (!shape_ok(shape) || k_pages < 1 || k_pages > num_pages(shape)) return STC_ERR_SHAPE;
  if (!aligned16(bounds) || !aligned16(page_idx)) return STC_ERR_ALIGN;
  const bool selecting = k_pages < num_pages(shape);
  if (selecting && (!ws || ws_bytes < score_bytes || !aligned16(ws))) return STC_ERR_WORKSPACE;
  char* attn_ws = ws ? (char*)ws + score_bytes : nullptr;
  const size_t attn_bytes = ws_bytes >= score_bytes ? ws_bytes - score_bytes : 0;
  const int rc = decode_attention_check(shape, q, K, vpacked, mask, tok_off, nullptr, k_pages,
                                        K_tail, V_tail, n_tail, tail_cap, false, out, attn_ws,
                                        attn_bytes);
  if (rc) return rc;
  const hipStream_t st = (hipStream_t)stream;
  const int tail_pages = (n_tail + shape->P - 1) / shape->P;
  if (!selecting) {  // every page: the attention kernel writes the list 0 .. NP-1 itself
    return stc::launch_attention(*shape, q, K, vpacked, mask, tok_off, nullptr, k_pages, K_tail,
                                 V_tail, n_tail, tail_cap, false, nullptr, nullptr, page_idx, out,
                                 attn_ws, st)
               ? STC_ERR_LAUNCH
               : STC_OK;
  }
  if (!stc::attention_can_select(*shape, k_pages, tail_pages)) {
    if (stc::launch_select(*shape, q, bounds, k_pages, page_idx, (float*)ws, false, st) ||
        stc::launch_attention(*shape, q, K, vpacked, mask, tok_off,
                              selecting ? page_idx : nullptr, k_pages, K_tail, V_tail, n_tail,
                              tail_cap, false, nullptr, nullptr, nullptr, out, attn_ws, st))
      return STC_ERR_LAUNCH;
    return STC_OK;
  }
  if (stc::launch_score(*shape, q, bounds, (float*)ws, false, st) ||
      stc::launch_attention(*shape, q, K, vpacked, mask, tok_off, nullptr, k_pages, K_tail,
                            V_tail, n_tail, tail_cap, false, nullptr, (const float*)ws, page_idx,
                            out, attn_ws, st))
    return STC_ERR_LAUNCH;
  return STC_OK;
}

}  // namespace

int stc_decode_step(const stc_shape_t* shape, const void* q, const void* bounds, const void* K,
                    const void* vpacked, const uint16_t* mask, const uint32_t* tok_off,
                    int k_pages, int32_t* page_idx, float* out, void* ws, size_t ws_bytes,
                    void* stream) {
  if (!shape) return STC_ERR_NULL;
  if (!shape_ok(shape)) return STC_ERR_SHAPE;
  return decode_step_impl(shape, q, bounds, K, vpacked, mask, tok_off, k_pages, nullptr, nullptr,
                          0, 0, page_idx, out, ws, ws_bytes, step_score_bytes(shape, k_pages),
                          stream);
}

int stc_decode_step_tail(const stc_shape_t* shape, const void* q, const void* bounds,
                         const void* K, const void* vpacked, const uint16_t* mask,
                         const uint32_t* tok_off, int k_pages, const void* K_tail,
                         const void* V_tail, int n_tail, int tail_cap, int32_t* page_idx,
                         float* out, void* ws, size_t ws_bytes, void* stream) {
  if (!shape) return STC_ERR_NULL;
  if (!shape_ok(shape)) return STC_ERR_SHAPE;
  return decode_step_impl(shape, q, bounds, K, vpacked, mask, tok_off, k_pages, K_tail, V_tail,
                          n_tail, tail_cap, page_idx, out, ws, ws_bytes,
                          step_score_bytes(shape, 0), stream);
}

int stc_decode_step_static(const stc_shape_t* shape, const void* q, const void* bounds,
                           const void* K, const void* vpacked, const uint16_t* mask,
                           const uint32_t* tok_off, int k_pages, int32_t* page_idx, float* out,
                           void* stream) {
  if (!shape) return STC_ERR_NULL;
  if (!shape_ok(shape) || k_pages < 1 || k_pages > num_pages(shape)) return STC_ERR_SHAPE;
  const size_t score_bytes = step_score_bytes(shape, k_pages);
  const size_t need = score_bytes + stc::attention_ws_bytes(*shape, k_pages);
  if (need > (size_t)STC_STATIC_SCRATCH_BYTES) return STC_ERR_WORKSPACE;
  void* ws = static_scratch();
  if (!ws) return STC_ERR_LAUNCH;
  // every byte of the scratch region that a kernel of the step reads (page scores, split
  // partials) has been written earlier in the same step, so nothing needs clearing
  return decode_step_impl(shape, q, bounds, K, vpacked, mask, tok_off, k_pages, nullptr, nullptr,
                          0, 0, page_idx, out, ws, STC_STATIC_SCRATCH_BYTES, score_bytes, stream);
}

int stc_flush_tail(const stc_shape_t* shape, void* K_tail, void* V_tail, int n_flush, int n_tail,
                   int tail_cap, int mode, const float* logits, const uint8_t* kcount, int fixed_k,
                   const uint16_t* mask_in, void* K, void* bounds, uint16_t* mask,
                   uint32_t* tok_off, void* vpacked, int32_t* dev_status, void* stream) {
  if (!shape || !K_tail || !V_tail || !K || !bounds || !mask || !tok_off || !vpacked)
    return STC_ERR_NULL;
  if (!shape_ok(shape) || n_flush < 1 || n_flush > n_tail || n_tail > tail_cap ||
      (long long)shape->N + n_flush > stc::token_cap(*shape))
    return STC_ERR_SHAPE;
  if (mode == STC_ROUTE_TOPK) {
    if (!logits) return STC_ERR_NULL;
    if (!kcount && (fixed_k < 0 || fixed_k > shape->G)) return STC_ERR_SHAPE;
  } else if (mode == STC_ROUTE_MASK) {
    if (!mask_in) return STC_ERR_NULL;
  } else {
    return STC_ERR_SHAPE;  // a global budget is not incremental
  }
  if (!aligned16(K_tail) || !aligned16(V_tail) || !aligned16(K) || !aligned16(bounds) ||
      !aligned16(mask) || !aligned16(tok_off) || !aligned16(vpacked) ||
      (logits && !aligned16(logits)) || (mask_in && !aligned16(mask_in)))
    return STC_ERR_ALIGN;
  return stc::launch_flush_tail(*shape, K_tail, V_tail, n_flush, n_tail, tail_cap, mode, logits, kcount,
                                fixed_k, mask_in, K, bounds, mask, tok_off, vpacked, dev_status,
                                (hipStream_t)stream)
             ? STC_ERR_LAUNCH
             : STC_OK;
}

int stc_union_pages(const stc_shape_t* shape, const int32_t* page_idx_per_head, int k_pages,
                    int32_t* union_idx, uint16_t* union_heads, int union_cap, void* stream) {
  if (!shape || !page_idx_per_head || !union_idx || !union_heads) return STC_ERR_NULL;
  if (!shape_ok(shape) || k_pages < 1 || k_pages > num_pages(shape)) return STC_ERR_SHAPE;
  const long long R = shape->Hq / shape->Hkv;
  // every selected page must fit; the lists are staged in 64 KiB of LDS
  const long long need = R * k_pages < num_pages(shape) ? R * k_pages : num_pages(shape);
  if (union_cap < need || R * k_pages * 4 > 65536) return STC_ERR_SHAPE;
  if (!aligned16(page_idx_per_head) || !aligned16(union_idx) || !aligned16(union_heads))
    return STC_ERR_ALIGN;
  return stc::launch_union_pages(*shape, page_idx_per_head, k_pages, union_idx, union_heads,
                                 union_cap, (hipStream_t)stream)
             ? STC_ERR_LAUNCH
             : STC_OK;
}

int stc_decode_attention_union(const stc_shape_t* shape, const void* q, const void* K,
                               const void* vpacked, const uint16_t* mask, const uint32_t* tok_off,
                               const int32_t* union_idx, const uint16_t* union_heads,
                               int union_cap, float* out, void* ws, size_t ws_bytes,
                               void* stream) {
  if (!union_idx || !union_heads) return STC_ERR_NULL;
  if (!aligned16(union_heads)) return STC_ERR_ALIGN;
  return decode_attention_impl(shape, q, K, vpacked, mask, tok_off, union_idx, union_cap, nullptr,
                               nullptr, 0, 0, false, union_heads, out, ws, ws_bytes, stream);
}

int stc_append_tail(const stc_shape_t* shape, const void* k_new, const void* v_new, void* K_tail,
                    void* V_tail, int n_tail, int tail_cap, void* stream) {
  if (!shape || !k_new || !v_new || !K_tail || !V_tail) return STC_ERR_NULL;
  if (!shape_ok(shape) || n_tail < 0 || n_tail >= tail_cap) return STC_ERR_SHAPE;
  if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(K_tail) || !aligned16(V_tail))
    return STC_ERR_ALIGN;
  return stc::launch_append_tail(*shape, k_new, v_new, K_tail, V_tail, n_tail, tail_cap,
                                 (hipStream_t)stream)
             ? STC_ERR_LAUNCH
             : STC_OK;
}

int stc_router_logits(int32_t B, int32_t Hkv, int32_t N, int32_t d_model, int32_t G,
                      const void* h, const void* W, const float* bias, int32_t bias_per_batch,
                      float* logits, void* stream) {
  if (!h || !W || !logits) return STC_ERR_NULL;
  if (bias_per_batch != 0 && bias_per_batch != 1) return STC_ERR_SHAPE;
  if (B < 1 || Hkv < 1 || N < 1 || d_model < 128 || d_model % 128 != 0 || B > kMaxGridY ||
      !(G == 1 || G == 2 || G == 4 || G == 8 || G == 16))
    return STC_ERR_SHAPE;
  if (!aligned16(h) || !aligned16(W) || !aligned16(logits) || (bias && ((uintptr_t)bias & 3)))
    return STC_ERR_ALIGN;
  return stc::launch_router_logits(h, W, bias, bias_per_batch ? G : 0, logits, B, Hkv, N, d_model,
                                   G, (hipStream_t)stream)
             ? STC_ERR_LAUNCH
             : STC_OK;
}

int stc_compact_tokens(const void* src, const int32_t* token_idx, void* dst, int32_t B,
                       int32_t Hkv, int32_t N_src, int32_t n_keep, int32_t D,
                       int32_t* dev_status, void* stream) {
  if (!src || !token_idx || !dst) return STC_ERR_NULL;
  if (B < 1 || Hkv < 1 || N_src < 1 || n_keep < 1 || (D != 64 && D != 128)) return STC_ERR_SHAPE;
  if ((long long)B * Hkv > kMaxGridY) return STC_ERR_SHAPE;
  if (!aligned16(src) || !aligned16(dst) || !aligned16(token_idx)) return STC_ERR_ALIGN;
  return stc::launch_compact(src, token_idx, dst, B, Hkv, N_src, n_keep, D, dev_status,
                             (hipStream_t)stream)
             ? STC_ERR_LAUNCH
             : STC_OK;
}

}  // extern "C"
