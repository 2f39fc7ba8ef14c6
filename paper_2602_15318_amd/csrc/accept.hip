// Greedy acceptance, plain-ALU lm_head pass and the finalize pass.
//
// Step 1 (this file: any dtype; accept_mfma.hip: bf16 on the matrix cores): logits of the
// B*(n_q+1) verified rows against the whole vocabulary, never written out: every wavefront keeps,
// per row, the best (value, lowest index) of the vocabulary range it owns and writes one
// candidate per row.  Step 2: reduce the candidates to the target's greedy token per row
// (lowest index wins ties), then walk the draft chain / tree from the last accepted token,
// taking the lowest-numbered child whose drafted token equals the target token of the current
// row (lossless greedy acceptance at temperature 0).
#include "accept.hpp"
#include "common.hpp"

namespace sparrow {

constexpr int kGenVW = 4;        // vocabulary rows per wavefront step
constexpr int kGenMC = 8;        // hidden rows per pass
constexpr int kGenBlocks = 512;  // workgroups of 4 wavefronts

template <typename T>
__global__ void __launch_bounds__(256) lm_head_generic_kernel(AcceptArgs a) {
  constexpr int PER = Elem<T>::kPer16B;
  const int lane = threadIdx.x % 64;
  const int gw = blockIdx.x * 4 + threadIdx.x / 64;   // global wavefront = candidate slot
  const int n_w = gridDim.x * 4;
  const int per = (a.V + n_w - 1) / n_w;
  const int v0 = min(a.V, gw * per), v1 = min(a.V, v0 + per);
  const T *Wm = (const T *)a.lm_head;
  const T *Hd = (const T *)a.hidden;

  for (int r0 = 0; r0 < a.M; r0 += kGenMC) {
    float best[kGenMC];
    int best_i[kGenMC];
#pragma unroll
    for (int r = 0; r < kGenMC; ++r) { best[r] = -INFINITY; best_i[r] = 0x7fffffff; }
    for (int vb = v0; vb < v1; vb += kGenVW) {
      float acc[kGenVW][kGenMC];
#pragma unroll
      for (int j = 0; j < kGenVW; ++j)
#pragma unroll
        for (int r = 0; r < kGenMC; ++r) acc[j][r] = 0.f;
      for (int x = lane * PER; x < a.H; x += 64 * PER) {
        float wf[kGenVW][PER];
#pragma unroll
        for (int j = 0; j < kGenVW; ++j) {
          const int v = min(vb + j, v1 - 1);
          u32x4 ww = *(const u32x4 *)(Wm + (int64_t)v * a.H + x);
          Elem<T>::unpack(ww, wf[j]);
        }
#pragma unroll
        for (int r = 0; r < kGenMC; ++r) {
          const int row = min(r0 + r, a.M - 1);
          u32x4 hw = *(const u32x4 *)(Hd + (int64_t)row * a.H + x);
          float hf[PER];
          Elem<T>::unpack(hw, hf);
#pragma unroll
          for (int j = 0; j < kGenVW; ++j)
#pragma unroll
            for (int e = 0; e < PER; ++e) acc[j][r] = fmaf(wf[j][e], hf[e], acc[j][r]);
        }
      }
#pragma unroll
      for (int j = 0; j < kGenVW; ++j) {
        const int v = vb + j;
#pragma unroll
        for (int r = 0; r < kGenMC; ++r) {
          const float s = wave_sum(acc[j][r]);
          if (v < v1 && s > best[r]) { best[r] = s; best_i[r] = v; }   // ascending v: lowest wins
          if (a.logits != nullptr && lane == 0 && v < v1 && r0 + r < a.M)
            a.logits[(int64_t)(r0 + r) * a.V + v] = s;
        }
      }
    }
    if (lane == 0) {
#pragma unroll
      for (int r = 0; r < kGenMC; ++r) {
        if (r0 + r < a.M) {
          a.cand_val[(int64_t)(r0 + r) * a.n_cand + gw] = best[r];
          a.cand_idx[(int64_t)(r0 + r) * a.n_cand + gw] = best_i[r];
        }
      }
    }
  }
}

// One workgroup of 16 wavefronts: wavefront w reduces the candidates of rows w, w+16, ... (64 lanes
// stride over the row's candidates, then a butterfly), then one thread per sequence walks the
// chain / tree.
__global__ void __launch_bounds__(1024) accept_finalize_kernel(AcceptArgs a) {
  __shared__ int32_t tgt[kAcceptMaxRows];
  __shared__ int32_t dr_s[kAcceptMaxRows], par_s[kAcceptMaxRows];
  const int tid = threadIdx.x;
  const int w = tid >> 6, lane = tid & 63;
  // draft tokens and parents of every sequence into LDS while the candidates are being reduced:
  // the walk below is a chain of dependent reads and should not pay a memory round trip each
  if (tid < a.B * a.n_q) {
    const int j = tid % a.n_q, b = tid / a.n_q;
    dr_s[tid] = a.draft_ids[tid];
    par_s[tid] = a.parent ? a.parent[(int64_t)b * a.parent_stride + j] : j - 1;
  }
  // two rows per wavefront at a time (rows r and r + 16): their candidate loads are in flight
  // together, and the 64-lane argmax runs on the vector ALU (maximum, then the lowest index
  // among the lanes that hold it)
  constexpr int kU = 16;                                 // independent loads in flight per lane and row
  for (int r0 = w; r0 < a.M; r0 += 32) {
    float bv[2];
    int bi[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) { bv[h] = -INFINITY; bi[h] = 0x7fffffff; }
    for (int c0 = lane; c0 < a.n_cand; c0 += 64 * kU) {
      float v[2][kU];
      int i[2][kU];
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int r = min(r0 + 16 * h, a.M - 1);         // the second row may not exist: a valid duplicate
        const float *cv = a.cand_val + (int64_t)r * a.n_cand;
        const int32_t *ci = a.cand_idx + (int64_t)r * a.n_cand;
#pragma unroll
        for (int u = 0; u < kU; ++u) {
          const int c = c0 + 64 * u;
          const bool in = c < a.n_cand;
          v[h][u] = in ? cv[c] : -INFINITY;
          i[h][u] = in ? ci[c] : 0x7fffffff;
        }
      }
#pragma unroll
      for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int u = 0; u < kU; ++u)
          if (v[h][u] > bv[h] || (v[h][u] == bv[h] && i[h][u] < bi[h])) { bv[h] = v[h][u]; bi[h] = i[h][u]; }
    }
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int r = r0 + 16 * h;
      const float wv = wave_max_valu(bv[h]);
      const int wi = wave_min_valu(bv[h] == wv ? bi[h] : 0x7fffffff);
      if (lane == 0 && r < a.M) { tgt[r] = wi; a.target_ids[r] = wi; }
    }
  }
  __syncthreads();
  if (tid < a.B) {
    const int b = tid;
    const int32_t *t = tgt + b * (a.n_q + 1);
    const int32_t *dr = dr_s + b * a.n_q, *par = par_s + b * a.n_q;
    int32_t *path = a.accept_path + (int64_t)b * a.n_q;
    int cur = -1, len = 0;
    // every accepted node has a larger index than its parent: at most n_q steps
    for (;;) {
      const int tok = t[cur + 1];
      int next = -1;
      for (int j = cur + 1; j < a.n_q; ++j) {
        if (par[j] == cur && dr[j] == tok) { next = j; break; }
      }
      if (next < 0) break;
      path[len++] = next;
      cur = next;
    }
    a.accept_len[b] = len;
    a.bonus_id[b] = t[cur + 1];
    for (int j = len; j < a.n_q; ++j) path[j] = -1;
  }
}

hipError_t launch_lm_head_generic(int dtype, const AcceptArgs &a, hipStream_t st) {
  const int blocks = a.n_cand / 4;
  if (dtype == SPARROW_F32)
    hipLaunchKernelGGL(lm_head_generic_kernel<float>, dim3(blocks), dim3(256), 0, st, a);
  else
    hipLaunchKernelGGL(lm_head_generic_kernel<bf16_t>, dim3(blocks), dim3(256), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_accept_finalize(const AcceptArgs &a, hipStream_t st) {
  hipLaunchKernelGGL(accept_finalize_kernel, dim3(1), dim3(1024), 0, st, a);
  return hipGetLastError();
}

int generic_num_candidates(int V) {
  int blocks = kGenBlocks;
  while (blocks > 1 && blocks * 4 * kGenVW > V) blocks /= 2;
  return blocks * 4;
}

}  // namespace sparrow
