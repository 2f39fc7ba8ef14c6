// Verification attention, plain-ALU partial pass and the split combine pass.
//
// The target scores n_q draft rows against the whole KV cache of their sequence in one pass
// (draft-then-verify loop; dynamic draft trees).  Row i sees every context token and, among the
// draft tokens, itself and its tree ancestors.  The context is cut into splits; each workgroup
// produces, for one (split, KV head, block of 16 rows), the online-softmax partial
//     m = max_t s_t,   l = sum_t 2^(s_t - m),   o = sum_t 2^(s_t - m) v_t
// with s_t = scale * log2(e) * <q, k_t>; the combine pass merges the splits.  All arithmetic is
// fp32, so this version also serves the fp32 configuration (tolerance 1e-5).
#include "common.hpp"
#include "verify_attn.hpp"

namespace sparrow {

constexpr int kGenRows = 16;   // rows (draft row x head of the group) per workgroup
constexpr int kGenTile = 32;   // tokens per LDS tile

template <typename T, int D>
__global__ void __launch_bounds__(256)
verify_partial_generic_kernel(VerifyArgs a, SeqTable tab) {
  constexpr int VPR = D / Elem<T>::kPer16B;   // 16-byte vectors per K/V row
  constexpr int RG = 256 / D;                 // row groups in the PV phase
  constexpr int RPT = kGenRows / RG;          // rows per thread in the PV phase
  __shared__ float Qs[kGenRows][D];
  __shared__ float Ks[kGenTile][D + 1];
  __shared__ float Vs[kGenTile][D];
  __shared__ float Ps[kGenRows][kGenTile];
  __shared__ float As[kGenRows];
  __shared__ unsigned long long Anc[kGenRows];

  const int tid = threadIdx.x;
  const int slot = blockIdx.x, c = blockIdx.y, rb = blockIdx.z;
  const int g = a.Hq / a.Hkv;
  const int R = a.n_q * g;
  const int b = seq_of_slot(tab, a.B, slot);
  const int len = tab.cu_len[b + 1] - tab.cu_len[b];   // L_b + n_q
  const int L = len - a.n_q;
  const int piece = split_len(len, tab.cu_split[b + 1] - tab.cu_split[b]);
  const int t0 = min(len, (slot - tab.cu_split[b]) * piece);
  const int t1 = min(len, t0 + piece);
  const int64_t tok_base = tab.cu_len[b];
  const T *K = (const T *)a.k + c * a.stride_head;
  const T *V = (const T *)a.v + c * a.stride_head;
  const T *Q = (const T *)a.q;

  // Q rows of this block, pre-scaled; rows past R are zero.
  for (int e = tid; e < kGenRows * D; e += 256) {
    int r = e / D, x = e % D;
    int rho = rb * kGenRows + r;
    float qv = 0.f;
    if (rho < R) {
      int i = rho / g, h = c * g + rho % g;
      qv = Elem<T>::load(Q + (((int64_t)b * a.n_q + i) * a.Hq + h) * D + x) * a.scale_log2;
    }
    Qs[r][x] = qv;
  }
  if (tid < kGenRows) {
    int rho = rb * kGenRows + tid;
    Anc[tid] = rho < R ? ancestor_mask(a.parent ? a.parent + (int64_t)b * a.parent_stride : nullptr, rho / g) : 0ull;
  }

  // score phase: thread -> (token tt, row group rg); rows rg and rg + 8
  const int tt = tid % kGenTile, rg = tid / kGenTile;
  float m_run[2] = {kNegBig, kNegBig}, l_run[2] = {0.f, 0.f};
  // PV phase: thread -> (x, row group); rows pr + RG * k
  const int px = tid % D, pr = tid / D;
  float acc[RPT];
#pragma unroll
  for (int k = 0; k < RPT; ++k) acc[k] = 0.f;

  for (int tb = t0; tb < t1; tb += kGenTile) {
    __syncthreads();   // previous tile fully consumed (also orders the Q/Anc stores)
    for (int e = tid; e < kGenTile * VPR; e += 256) {
      int row = e / VPR, vec = e % VPR;
      int tok = tb + row;
      float kf[Elem<T>::kPer16B], vf[Elem<T>::kPer16B];
      if (tok < t1) {
        const int64_t off = (tok_base + tok) * a.stride_tok + vec * Elem<T>::kPer16B;
        u32x4 kw = *(const u32x4 *)(K + off);
        u32x4 vw = *(const u32x4 *)(V + off);
        Elem<T>::unpack(kw, kf);
        Elem<T>::unpack(vw, vf);
      } else {
#pragma unroll
        for (int u = 0; u < Elem<T>::kPer16B; ++u) { kf[u] = 0.f; vf[u] = 0.f; }
      }
#pragma unroll
      for (int u = 0; u < Elem<T>::kPer16B; ++u) {
        Ks[row][vec * Elem<T>::kPer16B + u] = kf[u];
        Vs[row][vec * Elem<T>::kPer16B + u] = vf[u];
      }
    }
    __syncthreads();
    const int tok = tb + tt;
#pragma unroll
    for (int k = 0; k < 2; ++k) {
      const int r = rg + 8 * k;
      float s = 0.f;
#pragma unroll 8
      for (int x = 0; x < D; ++x) s = fmaf(Qs[r][x], Ks[tt][x], s);
      bool ok = tok < t1;
      if (tok >= L) ok = ok && ((Anc[r] >> (tok - L)) & 1ull);
      s = ok ? s : -INFINITY;
      // max / sum over the 32 tokens of the tile = one half of the wavefront
      float mx = s;
#pragma unroll
      for (int o = 16; o >= 1; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
      const float m_new = fmaxf(m_run[k], mx);
      const float p = fast_exp2(s - m_new);
      float ps = p;
#pragma unroll
      for (int o = 16; o >= 1; o >>= 1) ps += __shfl_xor(ps, o, 64);
      const float alpha = fast_exp2(m_run[k] - m_new);
      l_run[k] = l_run[k] * alpha + ps;
      m_run[k] = m_new;
      Ps[r][tt] = p;
      if (tt == 0) As[r] = alpha;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < RPT; ++k) {
      const int r = pr + RG * k;
      float o = acc[k] * As[r];
#pragma unroll 8
      for (int t = 0; t < kGenTile; ++t) o = fmaf(Ps[r][t], Vs[t][px], o);
      acc[k] = o;
    }
  }

  // partial results
#pragma unroll
  for (int k = 0; k < RPT; ++k) {
    const int rho = rb * kGenRows + pr + RG * k;
    if (rho < R) {
      const int i = rho / g, h = c * g + rho % g;
      a.part_o[(((int64_t)slot * a.n_q + i) * a.Hq + h) * D + px] = acc[k];
    }
  }
  if (tt == 0) {
#pragma unroll
    for (int k = 0; k < 2; ++k) {
      const int rho = rb * kGenRows + rg + 8 * k;
      if (rho < R) {
        const int i = rho / g, h = c * g + rho % g;
        float *ml = a.part_ml + (((int64_t)slot * a.n_q + i) * a.Hq + h) * 2;
        ml[0] = m_run[k];
        ml[1] = l_run[k];
      }
    }
  }
}

// Combine: m = max_s m_s, l = sum_s l_s 2^(m_s - m), o = sum_s o_s 2^(m_s - m) / l.
// One workgroup of 4 wavefronts per (row, head); wavefront w takes splits w, w+4, ..., four at a
// time so that all its loads are in flight together; each lane owns D/64 consecutive elements.
template <typename T, int D>
__global__ void __launch_bounds__(256) verify_combine_kernel(VerifyArgs a, SeqTable tab) {
  constexpr int EPL = D / 64;            // elements per lane: 1 or 2
  __shared__ float red_m[4];
  __shared__ float red_l[4];
  __shared__ float red_o[4][D];
  const int row = blockIdx.x;           // b * n_q + i
  const int h = blockIdx.y;
  const int b = row / a.n_q, i = row % a.n_q;
  const int s0 = tab.cu_split[b], s1 = tab.cu_split[b + 1];
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int64_t rh = (int64_t)i * a.Hq + h;
  const int64_t sstride = (int64_t)a.n_q * a.Hq;     // partial rows per split
  // global max over the splits
  float m = kNegBig;
  for (int s = s0 + (int)threadIdx.x; s < s1; s += 256) m = fmaxf(m, a.part_ml[(s * sstride + rh) * 2]);
  m = wave_max(m);
  if (lane == 0) red_m[w] = m;
  __syncthreads();
  m = fmaxf(fmaxf(red_m[0], red_m[1]), fmaxf(red_m[2], red_m[3]));
  float l = 0.f, o[EPL];
#pragma unroll
  for (int e = 0; e < EPL; ++e) o[e] = 0.f;
  for (int sb = s0 + w; sb < s1; sb += 16) {
    float ms[4], ls[4], ov[4][EPL];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int s = min(sb + 4 * u, s1 - 1);
      const int64_t idx = s * sstride + rh;
      ms[u] = a.part_ml[idx * 2];
      ls[u] = a.part_ml[idx * 2 + 1];
#pragma unroll
      for (int e = 0; e < EPL; ++e) ov[u][e] = a.part_o[idx * D + lane * EPL + e];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const float wgt = (sb + 4 * u < s1) ? fast_exp2(ms[u] - m) : 0.f;
      l = fmaf(ls[u], wgt, l);
#pragma unroll
      for (int e = 0; e < EPL; ++e) o[e] = fmaf(ov[u][e], wgt, o[e]);
    }
  }
  if (lane == 0) red_l[w] = l;
#pragma unroll
  for (int e = 0; e < EPL; ++e) red_o[w][lane * EPL + e] = o[e];
  __syncthreads();
  if (threadIdx.x < D) {
    const int x = threadIdx.x;
    const float lt = red_l[0] + red_l[1] + red_l[2] + red_l[3];
    const float ot = red_o[0][x] + red_o[1][x] + red_o[2][x] + red_o[3][x];
    Elem<T>::store((T *)a.out + ((int64_t)row * a.Hq + h) * D + x, ot / lt);
    if (a.lse != nullptr && x == 0) a.lse[(int64_t)row * a.Hq + h] = (m + fast_log2(lt)) * kLn2;
  }
}

template <typename T, int D>
static hipError_t launch_partial(const VerifyArgs &a, const SeqTable &tab, hipStream_t st) {
  const int g = a.Hq / a.Hkv;
  const int R = a.n_q * g;
  dim3 grid(a.n_slots, a.Hkv, (R + kGenRows - 1) / kGenRows);
  hipLaunchKernelGGL((verify_partial_generic_kernel<T, D>), grid, dim3(256), 0, st, a, tab);
  return hipGetLastError();
}

hipError_t launch_verify_partial_generic(int dtype, const VerifyArgs &a, const SeqTable &tab,
                                         hipStream_t st) {
  if (dtype == SPARROW_F32) {
    return a.d == 64 ? launch_partial<float, 64>(a, tab, st) : launch_partial<float, 128>(a, tab, st);
  }
  return a.d == 64 ? launch_partial<bf16_t, 64>(a, tab, st) : launch_partial<bf16_t, 128>(a, tab, st);
}

template <typename T, int D>
static hipError_t launch_comb(const VerifyArgs &a, const SeqTable &tab, hipStream_t st) {
  dim3 grid(a.B * a.n_q, a.Hq);
  hipLaunchKernelGGL((verify_combine_kernel<T, D>), grid, dim3(256), 0, st, a, tab);
  return hipGetLastError();
}

hipError_t launch_verify_combine(int dtype, const VerifyArgs &a, const SeqTable &tab,
                                 hipStream_t st) {
  if (dtype == SPARROW_F32) {
    return a.d == 64 ? launch_comb<float, 64>(a, tab, st) : launch_comb<float, 128>(a, tab, st);
  }
  return a.d == 64 ? launch_comb<bf16_t, 64>(a, tab, st) : launch_comb<bf16_t, 128>(a, tab, st);
}

}  // namespace sparrow
