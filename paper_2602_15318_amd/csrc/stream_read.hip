// Measurement aid: a kernel that only reads a byte range (16-byte non-temporal loads, a chosen
// number of them in flight per lane) -- what moving the bytes costs on this device without any
// arithmetic, timed by bench.py beside the attention kernel that reads the same bytes.  The
// launch shape is a parameter so that bench.py can look for the fastest read of a layer's K/V
// (the measured ceiling the attention kernel is graded against, beside the published HBM peak).
#include "common.hpp"

namespace sparrow {

namespace {

// kUnroll loads in flight per lane.  regions = 0: the grid sweeps the range front to back
// (consecutive workgroups read consecutive 4 KB pieces, grid-stride); regions = 1: every
// workgroup reads one contiguous region of its own, as the workgroups of the attention kernel do.
template <int kUnroll>
__global__ void __launch_bounds__(256)
stream_read_kernel(const u32x4 *__restrict__ p, size_t n16, unsigned int *sink, int regions) {
  size_t i, end, stride;
  if (regions) {
    const size_t per = (n16 + gridDim.x - 1) / gridDim.x;
    i = (size_t)blockIdx.x * per + threadIdx.x;
    end = min(n16, ((size_t)blockIdx.x + 1) * per);
    stride = 256;
  } else {
    i = (size_t)blockIdx.x * 256 + threadIdx.x;
    end = n16;
    stride = (size_t)gridDim.x * 256;
  }
  unsigned int acc = 0u;
  for (; i + (kUnroll - 1) * stride < end; i += kUnroll * stride) {
    u32x4 v[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) v[u] = __builtin_nontemporal_load(p + i + u * stride);
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  for (; i < end; i += stride) {
    const u32x4 v = __builtin_nontemporal_load(p + i);
    acc ^= v.x ^ v.y ^ v.z ^ v.w;
  }
  // the word is written by (at most) the lanes whose running XOR is all ones: enough to keep the
  // loads alive, rare enough not to count as traffic
  if (acc == 0xffffffffu) sink[0] = acc;
}

}  // namespace

hipError_t launch_stream_read(const void *p, size_t bytes, unsigned int *sink, int workgroups,
                              int in_flight, int regions, hipStream_t st) {
  const dim3 grid(workgroups), block(256);
  const u32x4 *q = (const u32x4 *)p;
  const size_t n16 = bytes / 16;
  switch (in_flight) {
    case 2: hipLaunchKernelGGL(stream_read_kernel<2>, grid, block, 0, st, q, n16, sink, regions); break;
    case 4: hipLaunchKernelGGL(stream_read_kernel<4>, grid, block, 0, st, q, n16, sink, regions); break;
    case 8: hipLaunchKernelGGL(stream_read_kernel<8>, grid, block, 0, st, q, n16, sink, regions); break;
    case 16: hipLaunchKernelGGL(stream_read_kernel<16>, grid, block, 0, st, q, n16, sink, regions); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace sparrow
