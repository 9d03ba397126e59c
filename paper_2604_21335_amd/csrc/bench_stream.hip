// Benchmark-only helper (its own small library, not part of the C ABI of libstc): a plain
// streaming read of device memory, the ceiling that HBM-bound kernels are measured against on
// the same box.  Every lane issues independent 16-byte loads of adjacent addresses (a
// wavefront request is 1 KiB), several of them in flight per lane.
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
constexpr int kThreads = 256;

// CONTIG: every workgroup reads one contiguous piece of the buffer (as the kernels of the
// library do with their tiles and pages); else the whole grid strides through it together.
template <int UNROLL, bool CONTIG>
__global__ __launch_bounds__(kThreads) void stream_read_kernel(const u32x4* __restrict__ src,
                                                                size_t n16, uint32_t* sink) {
  size_t i, end, stride;
  if (CONTIG) {
    const size_t per = (n16 + gridDim.x - 1) / gridDim.x;
    i = (size_t)blockIdx.x * per + threadIdx.x;
    end = min(n16, (size_t)(blockIdx.x + 1) * per);
    stride = kThreads;
  } else {
    i = (size_t)blockIdx.x * kThreads + threadIdx.x;
    end = n16;
    stride = (size_t)gridDim.x * kThreads;
  }
  u32x4 acc = {0u, 0u, 0u, 0u};
  for (; i + (UNROLL - 1) * stride < end; i += UNROLL * stride) {
    u32x4 v[UNROLL];
#pragma unroll
    for (int j = 0; j < UNROLL; ++j) v[j] = src[i + j * stride];
#pragma unroll
    for (int j = 0; j < UNROLL; ++j) acc ^= v[j];
  }
  for (; i < end; i += stride) acc ^= src[i];
  // keeps the loads alive; the store itself almost never happens
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u) *sink = acc.x;
}

}  // namespace

extern "C" {

// Reads `bytes` (a multiple of 16) of device memory at `src` once.  `sink` is a device
// uint32.  blocks <= 0 picks 8 workgroups of 256 threads per compute unit.  unroll: loads in
// flight per lane (4, 8 or 16; else 8).  contiguous != 0: one contiguous piece per workgroup.
// Returns 0, or -1 on a bad argument or a launch error.
int stcb_stream_read(const void* src, size_t bytes, void* sink, int blocks, int unroll,
                     int contiguous, void* stream) {
  if (!src || !sink || (bytes & 15u)) return -1;
  if (blocks <= 0) {
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess)
      (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    blocks = 8 * cus;
  }
  const u32x4* s = (const u32x4*)src;
  const size_t n16 = bytes / 16;
  uint32_t* k = (uint32_t*)sink;
  hipStream_t st = (hipStream_t)stream;
#define STCB_GO(U)                                                                    \
  if (contiguous)                                                                     \
    stream_read_kernel<U, true><<<blocks, kThreads, 0, st>>>(s, n16, k);              \
  else                                                                                \
    stream_read_kernel<U, false><<<blocks, kThreads, 0, st>>>(s, n16, k)
  if (unroll == 4) {
    STCB_GO(4);
  } else if (unroll == 16) {
    STCB_GO(16);
  } else {
    STCB_GO(8);
  }
#undef STCB_GO
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

}  // extern "C"
