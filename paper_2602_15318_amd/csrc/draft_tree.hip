// Dynamic draft tree: top-k log-probabilities over the vocabulary, best-first level expansion,
// final selection.  Everything after the lm_head GEMM is small (a few KB to a few MB), so the
// kernels are written for few launches and short dependent chains, not for bandwidth:
//   topk_chunk_kernel   grid (64 chunks, M rows): the chunk's softmax statistics and its k largest
//                       logits (a thread owns ~10 logits in registers; k rounds of a per-wavefront
//                       argmax, then a merge of the four wavefronts' lists);
//   topk_merge_kernel   one wavefront per row: k rounds of a 64-lane argmax over the heads of the
//                       chunk lists; the k best are written in order with their log-softmax from
//                       the row's statistics;
//   tree_expand_kernel  one workgroup: appends the candidates of a level to the pool with their
//                       cumulative scores and ranks them for the next frontier;
//   tree_select_kernel  one workgroup: ranks the whole pool, keeps the `total` best, renumbers
//                       them in pool order (block scan over the keep flags).
// "Better" is always: higher value, then lower index -- the order of the oracle.
#include "common.hpp"
#include "draft_tree.hpp"

namespace sparrow {

namespace {

constexpr int kTopkThreads = 256;
constexpr int kTopkPerThread = 16;      // logits a thread may own: chunks of up to 4096 tokens

__device__ __forceinline__ bool better(float va, int ia, float vb, int ib) {
  return va > vb || (va == vb && ia < ib);
}

// One workgroup of 4 wavefronts per (chunk of the vocabulary, row); a thread owns up to 16 logits
// in registers.  The chunk's softmax statistics (max and sum of exp2 in the log2 domain) come from
// the same registers.  Top k: every wavefront takes the k best of its own logits by k rounds of a
// 64-lane argmax on the vector ALU (value by maximum, then the lowest index among the lanes that
// hold it; no barrier, no LDS crossbar), then wavefront 0 merges the four sorted lists.
__global__ void __launch_bounds__(kTopkThreads)
topk_chunk_kernel(TopkArgs a) {
  constexpr int kWaves = kTopkThreads / 64;
  __shared__ float red[kWaves];
  __shared__ float lv[kWaves][kTreeMaxWidth];
  __shared__ int li[kWaves][kTreeMaxWidth];
  const int c = blockIdx.x, r = blockIdx.y;
  const int per = (a.V + kStatChunks - 1) / kStatChunks;
  const int v0 = min(a.V, c * per), v1 = min(a.V, v0 + per);
  const float *lg = a.logits + (int64_t)r * a.V;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  float val[kTopkPerThread];
#pragma unroll
  for (int j = 0; j < kTopkPerThread; ++j) {
    const int v = v0 + threadIdx.x + j * kTopkThreads;
    val[j] = v < v1 ? lg[v] : -INFINITY;
  }
  // ---- statistics of the chunk (temperature 1): m = max of l log2 e, s = sum of exp2(l log2 e - m)
  {
    constexpr float kLog2e = 1.4426950408889634f;
    float m = -INFINITY;
#pragma unroll
    for (int j = 0; j < kTopkPerThread; ++j) m = fmaxf(m, val[j]);
    m = wave_max_valu(m);
    if (lane == 0) red[w] = m;
    __syncthreads();
    m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    __syncthreads();
    const float ms = v1 > v0 ? m * kLog2e : kNegBig;       // an empty chunk: (kNegBig, 0)
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < kTopkPerThread; ++j) s += fast_exp2(fmaf(val[j], kLog2e, -ms));   // exp2(-inf) = 0
    s = wave_sum_valu(s);
    if (lane == 0) red[w] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
      float *o = a.stats + ((int64_t)r * kStatChunks + c) * 2;
      o[0] = ms;
      o[1] = v1 > v0 ? red[0] + red[1] + red[2] + red[3] : 0.f;
    }
  }
  // ---- the wavefront's k best, in decreasing order (ties: lower index first)
  for (int round = 0; round < a.k; ++round) {
    float bv = -INFINITY;
    int bj = 0;
#pragma unroll
    for (int j = 0; j < kTopkPerThread; ++j)
      if (val[j] > bv) { bv = val[j]; bj = j; }             // ascending index: the lowest wins a tie
    const float wv = wave_max_valu(bv);
    const int bi = v0 + (int)threadIdx.x + bj * kTopkThreads;
    const int wi = wave_min_valu((bv == wv && bv > -INFINITY) ? bi : 0x7fffffff);
    // the winner leaves its owner's registers (an exhausted wavefront yields -inf / 0x7fffffff)
#pragma unroll
    for (int j = 0; j < kTopkPerThread; ++j)
      if (j == bj && bi == wi) val[j] = -INFINITY;
    if (lane == 0) { lv[w][round] = wi == 0x7fffffff ? -INFINITY : wv; li[w][round] = wi; }
  }
  __syncthreads();
  // ---- merge of the four lists: lane l < 4 walks list l, every round the best head wins
  if (w == 0) {
    int pos = 0;
    float hv = lane < kWaves ? lv[lane][0] : -INFINITY;
    int hi = lane < kWaves ? li[lane][0] : 0x7fffffff;
    for (int round = 0; round < a.k; ++round) {
      const float wv = wave_max_valu(hv);
      const int wi = wave_min_valu((hv == wv && hi != 0x7fffffff) ? hi : 0x7fffffff);
      if (lane == 0) {
        const int64_t o = ((int64_t)r * kStatChunks + c) * a.k + round;
        a.cand_val[o] = wi == 0x7fffffff ? -INFINITY : wv;
        a.cand_idx[o] = wi;
      }
      if (hi == wi && wi != 0x7fffffff) {                   // the owner of the winner moves on
        ++pos;
        hv = pos < a.k ? lv[lane][pos] : -INFINITY;
        hi = pos < a.k ? li[lane][pos] : 0x7fffffff;
      }
    }
  }
}

__global__ void __launch_bounds__(64)
topk_merge_kernel(TopkArgs a) {
  // one wavefront per row: lane c walks chunk c's list (already in decreasing order); every round
  // the best list head of the 64 lanes is the row's next token
  const int r = blockIdx.x, lane = threadIdx.x;
  const float pm = a.stats[((int64_t)r * kStatChunks + lane) * 2];
  const float ps = a.stats[((int64_t)r * kStatChunks + lane) * 2 + 1];
  // the lane's whole list goes to LDS first (all loads in flight at once: one round trip); the
  // walk then costs an LDS read per round instead of a dependent global load
  __shared__ float sv[kTreeMaxWidth][64];
  __shared__ int si[kTreeMaxWidth][64];
  const float *cv = a.cand_val + ((int64_t)r * kStatChunks + lane) * a.k;
  const int32_t *ci = a.cand_idx + ((int64_t)r * kStatChunks + lane) * a.k;
#pragma unroll
  for (int j = 0; j < kTreeMaxWidth; ++j) {
    sv[j][lane] = j < a.k ? cv[j] : -INFINITY;
    si[j][lane] = j < a.k ? ci[j] : 0x7fffffff;
  }
  const float m = wave_max_valu(pm);
  const float Z = wave_sum_valu(ps * fast_exp2(pm - m));
  const float lse = (m + fast_log2(Z)) * kLn2;       // m is in the log2 domain (l log2 e)
  int pos = 0;
  float hv = sv[0][lane];                            // (a lane reads only what it wrote itself)
  int hi = si[0][lane];
  for (int round = 0; round < a.k; ++round) {
    const float wv = wave_max_valu(hv);
    const int wi = wave_min_valu((hv == wv && hi != 0x7fffffff) ? hi : 0x7fffffff);
    if (wi == 0x7fffffff) break;                     // every list exhausted (uniform)
    if (lane == 0) {
      a.ids[(int64_t)r * a.k + round] = wi;
      a.logp[(int64_t)r * a.k + round] = wv - lse;
    }
    if (hi == wi) {                                  // the owner of the winner moves on
      ++pos;
      hv = pos < a.k ? sv[pos][lane] : -INFINITY;
      hi = pos < a.k ? si[pos][lane] : 0x7fffffff;
    }
  }
}

__global__ void __launch_bounds__(256)
tree_expand_kernel(ExpandArgs a) {
  __shared__ float sc[kTreeMaxWidth * kTreeMaxWidth];
  const int tid = threadIdx.x;
  const int n_new = a.n_front * a.width;
  if (tid < n_new) {
    const int f = tid / a.width;
    const int p = a.front_in ? a.front_in[f] : -1;
    const float s = (p >= 0 ? a.pool_score[p] : 0.f) + a.cand_logp[tid];
    a.pool_tok[a.n_pool + tid] = a.cand_ids[tid];
    a.pool_par[a.n_pool + tid] = p;
    a.pool_score[a.n_pool + tid] = s;
    sc[tid] = s;
  }
  __syncthreads();
  if (tid < n_new) {
    const float s = sc[tid];
    int rank = 0;
    for (int j = 0; j < n_new; ++j) rank += better(sc[j], j, s, tid) ? 1 : 0;
    if (rank < a.width) a.front_out[rank] = a.n_pool + tid;
  }
}

__global__ void __launch_bounds__(1024)
tree_select_kernel(SelectArgs a) {
  __shared__ __attribute__((aligned(16))) float sc[kTreeMaxPool];
  __shared__ int new_id[kTreeMaxPool];
  __shared__ int wave_cnt[16];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int n = a.n_pool;
  const int keep = min(a.total, n);
  for (int i = tid; i < ((n + 3) & ~3); i += 1024) sc[i] = i < n ? a.pool_score[i] : -INFINITY;
  __syncthreads();
  // thread t owns pool entries t*E .. t*E+E-1, E = 1 or 2 (pool order = renumbering order)
  const int E = n > 1024 ? 2 : 1;
  int flag[2] = {0, 0};
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int i = E * tid + u;
    if (u < E && i < n) {
      const float s = sc[i];
      int rank = 0;
      // four scores per LDS read (the tail of the array is padded with -inf)
#pragma unroll 4
      for (int j = 0; j < n; j += 4) {
        const f32x4 q = *reinterpret_cast<const f32x4 *>(&sc[j]);
        rank += (int)better(q[0], j, s, i) + (int)better(q[1], j + 1, s, i) +
                (int)better(q[2], j + 2, s, i) + (int)better(q[3], j + 3, s, i);
      }
      flag[u] = rank < keep ? 1 : 0;
    }
  }
  int incl = flag[0] + flag[1];
  const int mine = incl;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int up = __shfl_up(incl, o, 64);
    if (lane >= o) incl += up;
  }
  if (lane == 63) wave_cnt[w] = incl;
  __syncthreads();
  int base = 0;
  for (int k = 0; k < w; ++k) base += wave_cnt[k];
  int pos = base + incl - mine;
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int i = E * tid + u;
    if (u < E && i < n) new_id[i] = flag[u] ? pos : -1;
    pos += flag[u];
  }
  __syncthreads();
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int i = E * tid + u;
    if (u < E && i < n && new_id[i] >= 0) {
      const int p = a.pool_par[i];
      a.parent[new_id[i]] = (p >= 0 && p < n) ? new_id[p] : -1;
      a.ids[new_id[i]] = a.pool_tok[i];
      a.pool_index[new_id[i]] = i;
    }
  }
}

}  // namespace

hipError_t launch_topk(const TopkArgs &a, hipStream_t st) {
  hipLaunchKernelGGL(topk_chunk_kernel, dim3(kStatChunks, a.M), dim3(kTopkThreads), 0, st, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(topk_merge_kernel, dim3(a.M), dim3(64), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_tree_expand(const ExpandArgs &a, hipStream_t st) {
  hipLaunchKernelGGL(tree_expand_kernel, dim3(1), dim3(256), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_tree_select(const SelectArgs &a, hipStream_t st) {
  hipLaunchKernelGGL(tree_select_kernel, dim3(1), dim3(1024), 0, st, a);
  return hipGetLastError();
}

}  // namespace sparrow
