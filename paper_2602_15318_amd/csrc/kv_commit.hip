// Post-accept commit: the K/V rows of the accepted draft nodes move up behind the context, in
// path order, in every layer; the hidden row of the last accepted node is gathered for the draft's
// next input.  Pure data movement (a few hundred KB), one launch for all layers.
//
// Grid (2 * n_layers + 1, B, Hkv): block x < 2 * n_layers owns one (layer, K or V, sequence, KV
// head); sources and destinations overlap only inside such a block (destination j <= source
// path[j]), so it reads all accepted rows into registers, synchronises, then writes.  The extra
// x index gathers the hidden rows (z = 0 only).
#include "common.hpp"
#include "kv_commit.hpp"

namespace sparrow {

namespace {

constexpr int kCommitThreads = 256;
constexpr int kCommitMaxPasses = 8;    // 64 rows of 512 bytes at 256 threads x 16 bytes

__global__ void __launch_bounds__(kCommitThreads)
kv_commit_kernel(CommitArgs a) {
  const int b = blockIdx.y;
  const int len = min(max(a.accept_len[b], 0), a.n_q);
  const int32_t *path = a.accept_path + (int64_t)b * a.n_q;
  if ((int)blockIdx.x == 2 * a.n_layers) {
    if (blockIdx.z != 0 || a.hidden == nullptr) return;
    int node = len > 0 ? path[len - 1] : -1;
    node = min(max(node, -1), a.n_q - 1);
    const int64_t row = (int64_t)b * (a.n_q + 1) + 1 + node;
    const int chunks = a.H * a.esize / 16;
    const u32x4 *src = (const u32x4 *)((const unsigned char *)a.hidden + row * a.H * a.esize);
    u32x4 *dst = (u32x4 *)((unsigned char *)a.next_hidden + (int64_t)b * a.H * a.esize);
    for (int i = threadIdx.x; i < chunks; i += kCommitThreads) dst[i] = src[i];
    return;
  }
  if (len == 0) return;
  const int layer = blockIdx.x >> 1;
  unsigned char *base = (unsigned char *)((blockIdx.x & 1) ? a.v[layer] : a.k[layer]);
  const int c = blockIdx.z;
  const int64_t first = (int64_t)a.cu_len[b + 1] - a.n_q;        // first draft row
  const int chunks = a.d * a.esize / 16;                          // 16-byte chunks per head row
  const int rows_per_pass = kCommitThreads / chunks;
  const int r0 = threadIdx.x / chunks, ch = threadIdx.x % chunks;
  auto addr = [&](int64_t row) {
    return (u32x4 *)(base + (row * a.stride_tok + (int64_t)c * a.stride_head) * a.esize) + ch;
  };
  u32x4 regs[kCommitMaxPasses];
#pragma unroll
  for (int p = 0; p < kCommitMaxPasses; ++p) {
    const int j = r0 + p * rows_per_pass;
    if (j < len) {
      const int node = min(max(path[j], 0), a.n_q - 1);           // never outside the draft rows
      regs[p] = *addr(first + node);
    }
  }
  __syncthreads();
#pragma unroll
  for (int p = 0; p < kCommitMaxPasses; ++p) {
    const int j = r0 + p * rows_per_pass;
    if (j < len) *addr(first + j) = regs[p];
  }
}

}  // namespace

hipError_t launch_kv_commit(const CommitArgs &a, hipStream_t st) {
  dim3 grid(2 * a.n_layers + 1, a.B, a.Hkv);
  hipLaunchKernelGGL(kv_commit_kernel, grid, dim3(kCommitThreads), 0, st, a);
  return hipGetLastError();
}

}  // namespace sparrow
