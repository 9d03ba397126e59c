// Internal launch interface between the C ABI (stc_api.hip) and the kernels.
// Every launcher enqueues on `st`, never synchronises, and returns 0 or -1
// (the HIP runtime refused a launch).  Shapes have been validated by the caller.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>

#include "../../include/stc.h"

namespace stc {

constexpr int kBoundsTilePages = 8;  // pages per tile of the bounds layout

// Token capacity of a stream's K, mask, tok_off and bounds arrays (their per-stream strides).
inline int token_cap(const stc_shape_t& s) { return s.N_cap ? s.N_cap : s.N; }
__host__ __device__ inline int bounds_tiles(int tokens) {
  return ((tokens + 15) / 16 + kBoundsTilePages - 1) / kBoundsTilePages;
}

// Raises a kernel's limit of dynamic LDS, once per device of the process (`done` holds one bit
// per device: the attribute belongs to the device's copy of the kernel).  False if the runtime
// refuses.  The only thing the library remembers between calls.
inline bool allow_dynamic_lds(const void* kernel, int bytes, std::atomic<uint64_t>& done) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return false;
  if ((done.load(std::memory_order_acquire) >> dev) & 1u) return true;
  if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess)
    return false;
  done.fetch_or(1ull << dev, std::memory_order_release);
  return true;
}

int launch_bounds(const stc_shape_t& s, const void* K, void* bounds, hipStream_t st);

size_t route_ws_bytes(const stc_shape_t& s);
int launch_route_pack(const stc_shape_t& s, int mode, const void* V, const float* logits,
                      const uint8_t* kcount, int fixed_k, const uint16_t* mask_in, uint16_t* mask,
                      uint32_t* tok_off, void* vpacked, int32_t* dev_status, void* ws,
                      hipStream_t st);

// per_head: one score row per query head ([B, Hq, NP]) instead of one per KV head
int launch_score(const stc_shape_t& s, const void* q, const void* bounds, float* score,
                 bool per_head, hipStream_t st);
// One workgroup per stream scores the stream and selects its pages (many streams of at most
// 2048 pages); `score` may be nullptr.  Only if score_can_select().
bool score_can_select(const stc_shape_t& s, int k_pages);
int launch_score_select(const stc_shape_t& s, const void* q, const void* bounds, float* score,
                        int32_t* page_idx, int k_pages, hipStream_t st);
int launch_select(const stc_shape_t& s, const void* q, const void* bounds, int k_pages,
                  int32_t* page_idx, float* score, bool per_head, hipStream_t st);

int attention_splits(const stc_shape_t& s, int k_pages);
size_t attention_ws_bytes(const stc_shape_t& s, int k_pages, bool per_head = false);
int launch_attention(const stc_shape_t& s, const void* q, const void* K, const void* vpacked,
                     const uint16_t* mask, const uint32_t* tok_off, const int32_t* page_idx,
                     int k_pages, const void* K_tail, const void* V_tail, int n_tail, int tail_cap,
                     bool per_head, const uint16_t* page_heads, const float* sel_score,
                     int32_t* sel_list, float* out, void* ws, hipStream_t st);
// sel_score != nullptr: no page list is read; the attention workgroups select the k pages of
// their stream from these scores themselves and write the list to sel_list.  Only if
// attention_can_select().
bool attention_can_select(const stc_shape_t& s, int k_pages, int tail_pages);
// Union of the page lists of the query heads of every KV head (ascending, padded with -1) and
// the heads that selected each page.
int launch_union_pages(const stc_shape_t& s, const int32_t* page_idx_per_head, int k_pages,
                       int32_t* union_idx, uint16_t* union_heads, int U, hipStream_t st);
int launch_flush_tail(const stc_shape_t& s, void* K_tail, void* V_tail, int n, int n_tail,
                      int tail_cap, int mode, const float* logits, const uint8_t* kcount,
                      int fixed_k, const uint16_t* mask_in, void* K, void* bounds, uint16_t* mask,
                      uint32_t* tok_off, void* vpacked, int32_t* dev_status, hipStream_t st);
int launch_append_tail(const stc_shape_t& s, const void* k_new, const void* v_new, void* K_tail,
                       void* V_tail, int n_tail, int tail_cap, hipStream_t st);

int launch_router_logits(const void* h, const void* W, const float* bias, int bias_stride,
                         float* logits, int B, int Hkv, int N, int d_model, int G, hipStream_t st);

int launch_compact(const void* src, const int32_t* token_idx, void* dst, int B, int Hkv, int N_src,
                   int n_keep, int D, int32_t* dev_status, hipStream_t st);

}  // namespace stc
