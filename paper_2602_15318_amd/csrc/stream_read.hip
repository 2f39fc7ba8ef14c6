// Measurement aid: a kernel that only reads a byte range (16-byte non-temporal loads, grid-stride,
// 8 loads in flight per lane) -- what moving the bytes costs on this device without any
// arithmetic, timed by bench.py beside the attention kernel that reads the same bytes.
#include "common.hpp"

namespace sparrow {

namespace {

constexpr int kUnroll = 8;

__global__ void __launch_bounds__(256)
stream_read_kernel(const u32x4 *__restrict__ p, size_t n16, unsigned int *sink) {
  const size_t tid = (size_t)blockIdx.x * 256 + threadIdx.x, stride = (size_t)gridDim.x * 256;
  unsigned int acc = 0u;
  size_t i = tid;
  for (; i + (kUnroll - 1) * stride < n16; i += kUnroll * stride) {
    u32x4 v[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) v[u] = __builtin_nontemporal_load(p + i + u * stride);
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  for (; i < n16; i += stride) {
    const u32x4 v = __builtin_nontemporal_load(p + i);
    acc ^= v.x ^ v.y ^ v.z ^ v.w;
  }
  // the word is written by (at most) the lanes whose running XOR is all ones: enough to keep the
  // loads alive, rare enough not to count as traffic
  if (acc == 0xffffffffu) sink[0] = acc;
}

}  // namespace

hipError_t launch_stream_read(const void *p, size_t bytes, unsigned int *sink, hipStream_t st) {
  hipLaunchKernelGGL(stream_read_kernel, dim3(1024), dim3(256), 0, st, (const u32x4 *)p, bytes / 16, sink);
  return hipGetLastError();
}

}  // namespace sparrow
