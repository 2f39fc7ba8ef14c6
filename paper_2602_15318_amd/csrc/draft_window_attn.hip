// Draft model's text-anchored window attention (VATA, Eq. 2): one query per sequence attends
// only to the `window` most recent text positions.  The kernel walks the precomputed
// text-position index, so keys and values at visual positions are never addressed.
//
// The whole job is at most a few hundred KB, so it is latency-bound: a single launch, one
// workgroup of 16 wavefronts per (sequence, query head): the job is too small to be bandwidth-bound, so the work is
// spread over as many compute units as there are heads and each re-reads its KV head's window from L2.
// A group of LPT lanes owns one token (each lane one 16-byte slice of the K and V rows); every
// lane group keeps its own online-softmax stream (m, l, o), streams are merged once at the end
// (lane groups by shuffles, wavefronts through LDS).  Up to 8 gathered tokens per lane group are
// in flight at a time.
#include <type_traits>

#include "common.hpp"
#include "draft_window_attn.hpp"

namespace sparrow {

constexpr int kDraftWaves = 16;
constexpr int kDraftRows = 1;     // query heads per workgroup
constexpr int kDraftUnroll = 8;   // tokens in flight per lane group

template <typename T, int D>
__global__ void __launch_bounds__(kDraftWaves * 64)
draft_window_attn_kernel(DraftArgs a, DraftTable tab) {
  constexpr int PER = Elem<T>::kPer16B;       // elements per 16-byte slice
  constexpr int LPT = D / PER;                // lanes per token
  constexpr int TPW = 64 / LPT;               // tokens per wavefront per step
  constexpr int STEP = kDraftWaves * TPW;     // tokens per workgroup per step
  __shared__ float Om[kDraftWaves][kDraftRows][D];
  __shared__ float Mm[kDraftWaves][kDraftRows];
  __shared__ float Lm[kDraftWaves][kDraftRows];

  const int b = blockIdx.x, c = blockIdx.y, rb = blockIdx.z;
  const int g = a.Hq / a.Hkv;
  const int r0 = rb * kDraftRows;                 // first head of the group handled here
  const int nr = min(kDraftRows, g - r0);
  const int tid = threadIdx.x, w = tid / 64, lane = tid % 64;
  const int sub = lane / LPT, vec = lane % LPT;

  const int n_text = tab.cu_text[b + 1] - tab.cu_text[b];
  const int n = min(n_text, a.window);
  const int32_t *idx = a.text_idx + tab.cu_text[b] + (n_text - n);
  const int64_t tok_base = tab.cu_len[b];
  const T *K = (const T *)a.k + c * a.stride_head + vec * PER;
  const T *V = (const T *)a.v + c * a.stride_head + vec * PER;

  // this lane's slice of the queries (raw storage words; the scale is applied to the scores)
  constexpr bool kBf16 = std::is_same<T, bf16_t>::value;
  u32x4 qw[kDraftRows];
  float qf[kDraftRows][PER];
#pragma unroll
  for (int r = 0; r < kDraftRows; ++r) {
    qw[r] = (u32x4){0u, 0u, 0u, 0u};
    if (r < nr) {
      const int h = c * g + r0 + r;
      qw[r] = *(const u32x4 *)((const T *)a.q + ((int64_t)b * a.Hq + h) * D + vec * PER);
    }
    Elem<T>::unpack(qw[r], qf[r]);
  }

  float m[kDraftRows], l[kDraftRows], acc[kDraftRows][PER];
#pragma unroll
  for (int r = 0; r < kDraftRows; ++r) {
    m[r] = kNegBig; l[r] = 0.f;
#pragma unroll
    for (int u = 0; u < PER; ++u) acc[r][u] = 0.f;
  }

  for (int j0 = w * TPW + sub; j0 < n; j0 += STEP * kDraftUnroll) {
    int pos[kDraftUnroll];
    u32x4 kw[kDraftUnroll], vw[kDraftUnroll];
#pragma unroll
    for (int u = 0; u < kDraftUnroll; ++u) {
      const int j = j0 + u * STEP;
      pos[u] = idx[j < n ? j : n - 1];      // clamped: always a valid text position
    }
#pragma unroll
    for (int u = 0; u < kDraftUnroll; ++u) {
      const int64_t off = (tok_base + pos[u]) * a.stride_tok;
      kw[u] = *(const u32x4 *)(K + off);
      vw[u] = *(const u32x4 *)(V + off);
    }
#pragma unroll
    for (int u = 0; u < kDraftUnroll; ++u) {
      const bool valid = (j0 + u * STEP) < n;
      float kf[PER], vf[PER];
      if (!kBf16) Elem<T>::unpack(kw[u], kf);
      Elem<T>::unpack(vw[u], vf);
#pragma unroll
      for (int r = 0; r < kDraftRows; ++r) {
        float s = 0.f;
        if (kBf16) {   // packed bf16 dot products with fp32 accumulation, no unpacking of K
          typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
          const unsigned qe[4] = {qw[r].x, qw[r].y, qw[r].z, qw[r].w};
          const unsigned ke[4] = {kw[u].x, kw[u].y, kw[u].z, kw[u].w};
#pragma unroll
          for (int e = 0; e < 4; ++e)
            s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, qe[e]),
                                                __builtin_bit_cast(bf16x2, ke[e]), s, false);
        } else {
#pragma unroll
          for (int e = 0; e < PER; ++e) s = fmaf(qf[r][e], kf[e], s);
        }
        s = group_sum<LPT>(s) * a.scale_log2;
        s = valid ? s : -INFINITY;
        const float m_new = fmaxf(m[r], s);
        const float alpha = fast_exp2(m[r] - m_new);
        const float p = fast_exp2(s - m_new);
        l[r] = l[r] * alpha + p;
        m[r] = m_new;
#pragma unroll
        for (int e = 0; e < PER; ++e) acc[r][e] = fmaf(p, vf[e], acc[r][e] * alpha);
      }
    }
  }

  // merge the TPW lane-group streams of this wavefront
  auto merge_with = [&](auto xor_tag) {
    constexpr int O = decltype(xor_tag)::value;
#pragma unroll
    for (int r = 0; r < kDraftRows; ++r) {
      const float m_o = lane_xor<O>(m[r], lane);
      const float l_o = lane_xor<O>(l[r], lane);
      const float m_new = fmaxf(m[r], m_o);
      const float wa = fast_exp2(m[r] - m_new), wb = fast_exp2(m_o - m_new);
      l[r] = l[r] * wa + l_o * wb;
      m[r] = m_new;
#pragma unroll
      for (int e = 0; e < PER; ++e) {
        const float a_o = lane_xor<O>(acc[r][e], lane);
        acc[r][e] = acc[r][e] * wa + a_o * wb;
      }
    }
  };
  if (LPT <= 8) merge_with(std::integral_constant<int, 8>{});
  if (LPT <= 16) merge_with(std::integral_constant<int, 16>{});
  merge_with(std::integral_constant<int, 32>{});
  if (sub == 0) {
#pragma unroll
    for (int r = 0; r < kDraftRows; ++r) {
#pragma unroll
      for (int e = 0; e < PER; ++e) Om[w][r][vec * PER + e] = acc[r][e];
      if (vec == 0) { Mm[w][r] = m[r]; Lm[w][r] = l[r]; }
    }
  }
  __syncthreads();
  // merge the wavefronts: thread -> (row, x)
  for (int e = tid; e < nr * D; e += kDraftWaves * 64) {
    const int r = e / D, x = e % D;
    float mm = kNegBig;
#pragma unroll
    for (int ww = 0; ww < kDraftWaves; ++ww) mm = fmaxf(mm, Mm[ww][r]);
    float ll = 0.f, oo = 0.f;
#pragma unroll
    for (int ww = 0; ww < kDraftWaves; ++ww) {
      const float wt = fast_exp2(Mm[ww][r] - mm);
      ll = fmaf(Lm[ww][r], wt, ll);
      oo = fmaf(Om[ww][r][x], wt, oo);
    }
    const int h = c * g + r0 + r;
    Elem<T>::store((T *)a.out + ((int64_t)b * a.Hq + h) * D + x, oo / ll);
    if (a.lse != nullptr && x == 0) a.lse[(int64_t)b * a.Hq + h] = (mm + fast_log2(ll)) * kLn2;
  }
}

template <typename T, int D>
static hipError_t launch(const DraftArgs &a, const DraftTable &tab, hipStream_t st) {
  const int g = a.Hq / a.Hkv;
  dim3 grid(a.B, a.Hkv, (g + kDraftRows - 1) / kDraftRows);
  hipLaunchKernelGGL((draft_window_attn_kernel<T, D>), grid, dim3(kDraftWaves * 64), 0, st, a, tab);
  return hipGetLastError();
}

hipError_t launch_draft_window_attn(int dtype, const DraftArgs &a, const DraftTable &tab,
                                    hipStream_t st) {
  if (dtype == SPARROW_F32)
    return a.d == 64 ? launch<float, 64>(a, tab, st) : launch<float, 128>(a, tab, st);
  return a.d == 64 ? launch<bf16_t, 64>(a, tab, st) : launch<bf16_t, 128>(a, tab, st);
}

}  // namespace sparrow
