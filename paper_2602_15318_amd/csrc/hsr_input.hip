// Input side of the draft model: hidden-state-reuse projection (Eq. 1) and the draft layer's
// RMSNorm / QKV / rotary step with the K/V append.  gfx950.
//
// Both are skinny GEMMs (at most 64 activation rows against a 51 MB and a 33 MB weight matrix at
// Qwen2.5-VL-7B shape), bound by the weight stream like lm_head and built the same way:
//   - one workgroup per tile of 16 weight rows (grid.y = blocks of 16 activation rows);
//   - wavefront w owns the 512-wide k-slices w, w + NW, ...: every load instruction reads the
//     slice of one weight row (1 KB contiguous), 16 loads in flight, staged through a private,
//     XOR-swizzled 16 KB LDS buffer into the A operand of v_mfma_f32_16x16x32_bf16; the B operand
//     is the wavefront's slice of the activation rows, held in registers;
//   - the partial sums of the wavefronts meet in LDS and wavefront 0 runs the epilogue.
// For the QKV step the tile's 16 weight rows are features f..f+7 and f+d/2..f+d/2+7 of one head,
// so both halves of every rotary pair sit in the same tile (lanes l and l^32 of the result);
// RMSNorm is folded in: gamma multiplies the activations on their way into the B operand, the
// row's 1/rms (from the squares each wavefront sees in its own slices) scales the result.
// Other shapes and fp32 run plain-ALU kernels (one wavefront per output feature or rotary pair).
#include "common.hpp"
#include "hsr_input.hpp"

namespace sparrow {

namespace {

constexpr int kSlice = 512;               // k elements per wavefront slice (1 KB of bf16)

// ---------------------------------------------------------------------------------------------
// shared main loop over TPW tiles of 16 weight rows: leaves in wavefront 0 the tiles' results,
// out[tp][i] = D[4*c4 + i][n] = sum over K of W[wrow(tp, 4*c4 + i)][k] * x[row0 + n][k], lane =
// n + 16*c4; *ssq = sum of x[row0 + n][k]^2 (kNorm).  SPW = slices per wavefront (K / 512 / NW).
// XLoad: x(m, k) -> pointer to 8 consecutive bf16 of activation row m at column k (k % 8 == 0).
// ---------------------------------------------------------------------------------------------
template <int NW, int SPW, int TPW, bool kNorm, class WRow, class XLoad>
__device__ __forceinline__ void skinny_tile(const bf16_t *W, int K, WRow wrow, XLoad xload,
                                            const bf16_t *gamma, int row0, int M,
                                            unsigned char *smem, f32x4 *out, float *ssq_out) {
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = lane & 15, c4 = lane >> 4;
  unsigned char *stg = smem + w * 16384;
  f32x4 *red = reinterpret_cast<f32x4 *>(smem + NW * 16384);          // [TPW][NW][64]
  float *ssq_lds = reinterpret_cast<float *>(smem + NW * 16384 + TPW * NW * 1024);   // [NW][16]

  u32x4 buf[16];
  // phase p = (slice p / TPW of this wavefront, tile p % TPW)
  auto issue = [&](int p) {
    const int s = w + (p / TPW) * NW, tp = p % TPW;
#pragma unroll
    for (int r = 0; r < 16; ++r)
      buf[r] = __builtin_nontemporal_load(
          (const u32x4 *)(W + (int64_t)wrow(tp, r) * K + kSlice * s + 8 * lane));
  };
  const int m = row0 + n;
  const bool m_ok = m < M;
  bf16x8 hreg[16];
  float ssq = 0.f;
  auto load_x = [&](int s) {
    // all loads first (raw activations, and gamma if the norm is folded in), then the conversion
    // in place: the raw registers become the B operands
    u32x4 xr[16], gr[16];
#pragma unroll
    for (int ks = 0; ks < 16; ++ks) {
      const int k = kSlice * s + 32 * ks + 8 * c4;
      xr[ks] = *(const u32x4 *)xload(m_ok ? m : 0, k);
      if (kNorm) gr[ks] = *(const u32x4 *)(gamma + k);
    }
    if (kNorm) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int ks = 0; ks < 16; ++ks) {
      u32x4 v = xr[ks];
      if (!m_ok) v = (u32x4){0u, 0u, 0u, 0u};
      if (kNorm) {
        float xf[8], gf[8];
        Elem<bf16_t>::unpack(v, xf);
        Elem<bf16_t>::unpack(gr[ks], gf);
#pragma unroll
        for (int e = 0; e < 8; ++e) ssq = fmaf(xf[e], xf[e], ssq);
        v = (u32x4){pack_bf16x2(xf[0] * gf[0], xf[1] * gf[1]), pack_bf16x2(xf[2] * gf[2], xf[3] * gf[3]),
                    pack_bf16x2(xf[4] * gf[4], xf[5] * gf[5]), pack_bf16x2(xf[6] * gf[6], xf[7] * gf[7])};
      }
      hreg[ks] = __builtin_bit_cast(bf16x8, v);
      // one k-step at a time: unpacked, all 16 would need as many registers as the kernel has
      if (kNorm) __builtin_amdgcn_sched_barrier(0);
    }
  };

  issue(0);
  load_x(w);
  f32x4 acc[TPW][2];
#pragma unroll
  for (int tp = 0; tp < TPW; ++tp) acc[tp][0] = acc[tp][1] = (f32x4){0.f, 0.f, 0.f, 0.f};
  const int a_base = n * 1024;            // A read: tile row n, 16-byte chunk 4*ks + c4
#pragma unroll
  for (int p = 0; p < SPW * TPW; ++p) {
    const int tp = p % TPW;
    // lane l of load r holds chunk l of row r; stored at chunk (l & ~15) | ((l & 15) ^ r) so that
    // the A reads (16 rows, same chunk) spread over all banks
#pragma unroll
    for (int r = 0; r < 16; ++r)
      *reinterpret_cast<u32x4 *>(stg + r * 1024 + (((lane & ~15) | ((lane & 15) ^ r)) << 4)) = buf[r];
    if (p + 1 < SPW * TPW) issue(p + 1);
#pragma unroll
    for (int ks = 0; ks < 16; ks += 2) {
      const int ch0 = 4 * ks + c4, ch1 = ch0 + 4;
      const bf16x8 a0 = *reinterpret_cast<const bf16x8 *>(stg + a_base + (((ch0 & ~15) | ((ch0 & 15) ^ n)) << 4));
      const bf16x8 a1 = *reinterpret_cast<const bf16x8 *>(stg + a_base + (((ch1 & ~15) | ((ch1 & 15) ^ n)) << 4));
      acc[tp][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, hreg[ks], acc[tp][0], 0, 0, 0);
      acc[tp][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, hreg[ks + 1], acc[tp][1], 0, 0, 0);
    }
    // next slice of the activations once the last tile of this slice is done
    if (tp == TPW - 1 && p + 1 < SPW * TPW) load_x(w + ((p + 1) / TPW) * NW);
  }
#pragma unroll
  for (int tp = 0; tp < TPW; ++tp) red[(tp * NW + w) * 64 + lane] = acc[tp][0] + acc[tp][1];
  if (kNorm) {
    ssq += lane_xor<16>(ssq, lane);
    ssq += lane_xor<32>(ssq, lane);       // all four k-chunk lanes of row n now hold the slice sum
    if (c4 == 0) ssq_lds[w * 16 + n] = ssq;
  }
  __syncthreads();
  if (w == 0) {
#pragma unroll
    for (int tp = 0; tp < TPW; ++tp) {
      f32x4 sum = red[(tp * NW) * 64 + lane];
#pragma unroll
      for (int ww = 1; ww < NW; ++ww) sum += red[(tp * NW + ww) * 64 + lane];
      out[tp] = sum;
    }
    if (kNorm) {
      float s2 = 0.f;
#pragma unroll
      for (int ww = 0; ww < NW; ++ww) s2 += ssq_lds[ww * 16 + n];
      *ssq_out = s2;
    }
  }
}

constexpr int skinny_lds_bytes(int NW, int TPW) { return NW * 16384 + TPW * NW * 1024 + NW * 64; }

// ---------------------------------------------------------------------------------------------
// Eq. 1: z = FC(e (+) h)
// ---------------------------------------------------------------------------------------------
template <int NW, int SPW>
__global__ void __launch_bounds__(NW * 64)
hsr_fc_mfma_kernel(HsrFcArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tile = blockIdx.x, row0 = blockIdx.y * 16;
  const int H = a.H;
  const bf16_t *E = (const bf16_t *)a.embed, *Hp = (const bf16_t *)a.h_prev;
  const int lane = threadIdx.x & 63, n = lane & 15, c4 = lane >> 4;
  // the token id of this lane's activation row (clamped into the table)
  const int m = row0 + n;
  int tok = m < a.M ? a.token_ids[m] : 0;
  tok = min(max(tok, 0), a.vocab - 1);
  auto wrow = [&](int, int r) { return tile * 16 + r; };
  // a slice lies entirely in one half of the concatenation (H is a multiple of the slice width)
  auto xload = [&](int mm, int k) -> const bf16_t * {
    return k < H ? E + (int64_t)tok * H + k : Hp + (int64_t)mm * H + (k - H);
  };
  float unused;
  f32x4 r;
  skinny_tile<NW, SPW, 1, false>((const bf16_t *)a.w, 2 * H, wrow, xload, nullptr, row0, a.M, smem,
                                 &r, &unused);
  if (threadIdx.x < 64 && m < a.M) {
    const int f = tile * 16 + 4 * c4;
    float b[4] = {0.f, 0.f, 0.f, 0.f};
    if (a.bias != nullptr) {
      const u32x2 bw = *(const u32x2 *)((const bf16_t *)a.bias + f);
      b[0] = bf16lo_to_f32(bw.x); b[1] = bf16hi_to_f32(bw.x);
      b[2] = bf16lo_to_f32(bw.y); b[3] = bf16hi_to_f32(bw.y);
    }
    const u32x2 o = {pack_bf16x2(r[0] + b[0], r[1] + b[1]), pack_bf16x2(r[2] + b[2], r[3] + b[3])};
    *(u32x2 *)((bf16_t *)a.z + (int64_t)m * H + f) = o;
  }
}

// ---------------------------------------------------------------------------------------------
// draft layer input: RMSNorm, QKV, rotary embedding, scatter
// ---------------------------------------------------------------------------------------------
template <int NW, int SPW>
__global__ void __launch_bounds__(NW * 64)
draft_qkv_mfma_kernel(DraftQkvArgs a) {
  constexpr int TPW = 2;        // tiles per workgroup: blockIdx.x and blockIdx.x + gridDim.x
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int row0 = blockIdx.y * 16;
  const int H = a.H, d = a.d, half = d >> 1;
  const int tiles_per_head = d >> 4;
  const int lane = threadIdx.x & 63, n = lane & 15, c4 = lane >> 4;
  const int m = row0 + n;
  const bool m_ok = m < a.M;
  const bf16_t *Z = (const bf16_t *)a.z;
  // tile -> (head, group j of 8 features); tile row r: feature 8j + (r & 7) of the head's first
  // half for r < 8, its rotary partner (+ d/2) for r >= 8
  int hd[TPW], j[TPW];
#pragma unroll
  for (int tp = 0; tp < TPW; ++tp) {
    const int tile = blockIdx.x + tp * gridDim.x;
    hd[tp] = tile / tiles_per_head;
    j[tp] = tile - hd[tp] * tiles_per_head;
  }
  auto wrow = [&](int tp, int r) { return hd[tp] * d + 8 * j[tp] + (r & 7) + (r >> 3) * half; };
  auto xload = [&](int mm, int k) -> const bf16_t * { return Z + (int64_t)mm * H + k; };
  // lane (n, c4), entry i of a tile's result: tile row 4*c4 + i -> feature f0 + i of half `hi`
  const int hi = c4 >> 1;
  // epilogue operands, fetched ahead of the weight stream: bias, the token's rotary row, its
  // cache row (the table is a kernel argument, read with uniform indices)
  u32x2 bw[TPW];
  f32x4 cs[TPW], sn[TPW];
#pragma unroll
  for (int tp = 0; tp < TPW; ++tp) {
    const int f0 = 8 * j[tp] + 4 * (c4 & 1);
    bw[tp] = (u32x2){0u, 0u};
    if (a.bias != nullptr) bw[tp] = *(const u32x2 *)((const bf16_t *)a.bias + hd[tp] * d + hi * half + f0);
    cs[tp] = *(const f32x4 *)(a.rope_cos + (int64_t)(m_ok ? m : 0) * half + f0);
    sn[tp] = *(const f32x4 *)(a.rope_sin + (int64_t)(m_ok ? m : 0) * half + f0);
  }
  int kv_row = 0;
#pragma unroll
  for (int mm = 0; mm < 16; ++mm) {
    const int r = a.kv_rows[min(row0 + mm, kHsrMaxRows - 1)];
    if (n == mm) kv_row = r;
  }

  float ssq = 0.f;
  f32x4 res[TPW];
  skinny_tile<NW, SPW, TPW, true>((const bf16_t *)a.w, H, wrow, xload, (const bf16_t *)a.gamma,
                                  row0, a.M, smem, res, &ssq);
  if (threadIdx.x >= 64) return;
  const float rstd = __builtin_amdgcn_rsqf(ssq / (float)H + a.eps);
#pragma unroll
  for (int tp = 0; tp < TPW; ++tp) {
    const int f0 = 8 * j[tp] + 4 * (c4 & 1);
    const float b[4] = {bf16lo_to_f32(bw[tp].x), bf16hi_to_f32(bw[tp].x),
                        bf16lo_to_f32(bw[tp].y), bf16hi_to_f32(bw[tp].y)};
    const bool is_v = hd[tp] >= a.Hq + a.Hkv;
    float o[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float y = fmaf(res[tp][i], rstd, b[i]);
      const float partner = lane_xor<32>(y, lane);      // the other half of the rotary pair
      o[i] = y;
      if (!is_v) o[i] = hi ? fmaf(partner, sn[tp][i], y * cs[tp][i]) : fmaf(-partner, sn[tp][i], y * cs[tp][i]);
    }
    if (!m_ok) continue;
    const u32x2 ow = {pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3])};
    const int feat = hi * half + f0;
    if (hd[tp] < a.Hq) {
      *(u32x2 *)((bf16_t *)a.q_out + ((int64_t)m * a.Hq + hd[tp]) * d + feat) = ow;
    } else {
      const int c = is_v ? hd[tp] - a.Hq - a.Hkv : hd[tp] - a.Hq;
      bf16_t *base = (bf16_t *)(is_v ? a.v_cache : a.k_cache);
      *(u32x2 *)(base + (int64_t)kv_row * a.stride_tok + (int64_t)c * a.stride_head + feat) = ow;
    }
  }
}

// ---------------------------------------------------------------------------------------------
// One activation row (the chain draft's one new token per step), bf16: no matrix cores, no LDS.
// A wavefront owns one output feature (FC) or one rotary pair of a head (QKV).  It issues every
// load of its weight row(s) at once (KS loads of 1 KB, each contiguous), then fetches the
// activation row (14 KB at most, shared by all wavefronts through L2), multiplies and reduces
// across its lanes on the vector ALU.  With ~100 registers per lane a compute unit holds 16 such
// wavefronts, i.e. ~200 KB of weight loads in flight, against 112 KB for the matrix-core kernel
// whose 16 KB of LDS staging per wavefront allows one workgroup per compute unit; at one row the
// matrix cores have nothing to offer (16 x fewer products than a tile holds).
// ---------------------------------------------------------------------------------------------
template <int KS>             // K / 512: 14 or 16 for Eq. 1 (K = 2H)
__global__ void __launch_bounds__(256)
hsr_fc_gemv_kernel(HsrFcArgs a) {
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
  const int lane = threadIdx.x & 63;
  const int nfeat = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int H = a.H;
  if (nfeat >= H) return;
  const bf16_t *W = (const bf16_t *)a.w + (int64_t)nfeat * (2 * H) + 8 * lane;
  u32x4 wv[KS];
#pragma unroll
  for (int s = 0; s < KS; ++s) wv[s] = __builtin_nontemporal_load((const u32x4 *)(W + kSlice * s));
  const int tok = min(max(a.token_ids[0], 0), a.vocab - 1);
  const bf16_t *E = (const bf16_t *)a.embed + (int64_t)tok * H + 8 * lane;
  const bf16_t *Hp = (const bf16_t *)a.h_prev + 8 * lane;
  u32x4 xv[KS];
#pragma unroll
  for (int s = 0; s < KS; ++s)     // the first KS / 2 slices meet the embedding, the rest the hidden state
    xv[s] = *(const u32x4 *)(s < KS / 2 ? E + kSlice * s : Hp + kSlice * (s - KS / 2));
  float acc = 0.f;
#pragma unroll
  for (int s = 0; s < KS; ++s) {
    const unsigned int w4[4] = {wv[s].x, wv[s].y, wv[s].z, wv[s].w};
    const unsigned int x4[4] = {xv[s].x, xv[s].y, xv[s].z, xv[s].w};
#pragma unroll
    for (int e = 0; e < 4; ++e)
      acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w4[e]), __builtin_bit_cast(bf16x2, x4[e]),
                                            acc, false);
  }
  acc = wave_sum_valu(acc);
  if (lane == 0) {
    const float b = a.bias != nullptr ? bf16_to_f32(((const bf16_t *)a.bias)[nfeat]) : 0.f;
    ((bf16_t *)a.z)[nfeat] = f32_to_bf16(acc + b);
  }
}

template <int KS>             // H / 512: 7 or 8
__global__ void __launch_bounds__(256)
draft_qkv_gemv_kernel(DraftQkvArgs a) {
  const int lane = threadIdx.x & 63;
  const int half = a.d >> 1;
  const int pair = blockIdx.x * 4 + (threadIdx.x >> 6);      // (head, feature of the first half)
  const int n_heads = a.Hq + 2 * a.Hkv;
  if (pair >= n_heads * half) return;
  const int hd = pair / half, f = pair - hd * half;
  const int H = a.H;
  const bf16_t *W0 = (const bf16_t *)a.w + ((int64_t)hd * a.d + f) * H + 8 * lane;
  const bf16_t *W1 = W0 + (int64_t)half * H;
  u32x4 w0[KS], w1[KS];
#pragma unroll
  for (int s = 0; s < KS; ++s) {
    w0[s] = __builtin_nontemporal_load((const u32x4 *)(W0 + kSlice * s));
    w1[s] = __builtin_nontemporal_load((const u32x4 *)(W1 + kSlice * s));
  }
  // epilogue operands ahead of the arithmetic
  const bool is_v = hd >= a.Hq + a.Hkv;
  float b0 = 0.f, b1 = 0.f;
  if (a.bias != nullptr) {
    b0 = bf16_to_f32(((const bf16_t *)a.bias)[hd * a.d + f]);
    b1 = bf16_to_f32(((const bf16_t *)a.bias)[hd * a.d + f + half]);
  }
  const float cs = a.rope_cos[f], sn = a.rope_sin[f];
  const bf16_t *Z = (const bf16_t *)a.z + 8 * lane, *G = (const bf16_t *)a.gamma + 8 * lane;
  float s0 = 0.f, s1 = 0.f, ssq = 0.f;
#pragma unroll
  for (int s = 0; s < KS; ++s) {
    float xf[8], gf[8], a0[8], a1[8];
    Elem<bf16_t>::unpack(*(const u32x4 *)(Z + kSlice * s), xf);
    Elem<bf16_t>::unpack(*(const u32x4 *)(G + kSlice * s), gf);
    Elem<bf16_t>::unpack(w0[s], a0);
    Elem<bf16_t>::unpack(w1[s], a1);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float u = xf[e] * gf[e];
      ssq = fmaf(xf[e], xf[e], ssq);
      s0 = fmaf(a0[e], u, s0);
      s1 = fmaf(a1[e], u, s1);
    }
  }
  s0 = wave_sum_valu(s0); s1 = wave_sum_valu(s1); ssq = wave_sum_valu(ssq);
  if (lane != 0) return;
  const float rstd = __builtin_amdgcn_rsqf(ssq / (float)H + a.eps);
  const float y0 = fmaf(s0, rstd, b0), y1 = fmaf(s1, rstd, b1);
  float o0 = y0, o1 = y1;
  if (!is_v) {
    o0 = y0 * cs - y1 * sn;
    o1 = y1 * cs + y0 * sn;
  }
  bf16_t *dst;
  if (hd < a.Hq) {
    dst = (bf16_t *)a.q_out + (int64_t)hd * a.d;
  } else {
    const int c = is_v ? hd - a.Hq - a.Hkv : hd - a.Hq;
    dst = (bf16_t *)(is_v ? a.v_cache : a.k_cache) + (int64_t)a.kv_rows[0] * a.stride_tok +
          (int64_t)c * a.stride_head;
  }
  dst[f] = f32_to_bf16(o0);
  dst[f + half] = f32_to_bf16(o1);
}

// ---------------------------------------------------------------------------------------------
// plain-ALU versions: any dtype, any H.  One wavefront per output feature (FC) or rotary pair.
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256)
hsr_fc_generic_kernel(HsrFcArgs a) {
  const int lane = threadIdx.x & 63;
  const int nfeat = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (nfeat >= a.H) return;
  const int H = a.H;
  const T *W = (const T *)a.w + (int64_t)nfeat * 2 * H;
  for (int row0 = 0; row0 < a.M; row0 += 16) {
    float acc[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    for (int k = lane; k < 2 * H; k += 64) {
      const float wv = Elem<T>::load(W + k);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = row0 + r;
        if (m < a.M) {
          float x;
          if (k < H) {
            const int tok = min(max(a.token_ids[m], 0), a.vocab - 1);
            x = Elem<T>::load((const T *)a.embed + (int64_t)tok * H + k);
          } else {
            x = Elem<T>::load((const T *)a.h_prev + (int64_t)m * H + (k - H));
          }
          acc[r] = fmaf(wv, x, acc[r]);
        }
      }
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const float s = wave_sum(acc[r]);
      const int m = row0 + r;
      if (lane == 0 && m < a.M) {
        const float b = a.bias != nullptr ? Elem<T>::load((const T *)a.bias + nfeat) : 0.f;
        Elem<T>::store((T *)a.z + (int64_t)m * H + nfeat, s + b);
      }
    }
  }
}

template <typename T>
__global__ void __launch_bounds__(256)
draft_qkv_generic_kernel(DraftQkvArgs a) {
  const int lane = threadIdx.x & 63;
  const int half = a.d >> 1;
  const int pair = blockIdx.x * 4 + (threadIdx.x >> 6);      // (head, feature of the first half)
  const int n_heads = a.Hq + 2 * a.Hkv;
  if (pair >= n_heads * half) return;
  const int hd = pair / half, f = pair - hd * half;
  const int H = a.H;
  const T *W0 = (const T *)a.w + ((int64_t)hd * a.d + f) * H;
  const T *W1 = W0 + (int64_t)half * H;
  const bool is_v = hd >= a.Hq + a.Hkv;
  for (int m = 0; m < a.M; ++m) {
    const T *z = (const T *)a.z + (int64_t)m * H;
    float s0 = 0.f, s1 = 0.f, ssq = 0.f;
    for (int k = lane; k < H; k += 64) {
      const float x = Elem<T>::load(z + k);
      const float u = x * Elem<T>::load((const T *)a.gamma + k);
      ssq = fmaf(x, x, ssq);
      s0 = fmaf(Elem<T>::load(W0 + k), u, s0);
      s1 = fmaf(Elem<T>::load(W1 + k), u, s1);
    }
    s0 = wave_sum(s0); s1 = wave_sum(s1); ssq = wave_sum(ssq);
    if (lane != 0) continue;
    const float rstd = 1.0f / sqrtf(ssq / (float)H + a.eps);
    float y0 = s0 * rstd, y1 = s1 * rstd;
    if (a.bias != nullptr) {
      y0 += Elem<T>::load((const T *)a.bias + hd * a.d + f);
      y1 += Elem<T>::load((const T *)a.bias + hd * a.d + f + half);
    }
    float o0 = y0, o1 = y1;
    if (!is_v) {
      const float cs = a.rope_cos[(int64_t)m * half + f], sn = a.rope_sin[(int64_t)m * half + f];
      o0 = y0 * cs - y1 * sn;
      o1 = y1 * cs + y0 * sn;
    }
    T *dst;
    if (hd < a.Hq) {
      dst = (T *)a.q_out + ((int64_t)m * a.Hq + hd) * a.d;
    } else {
      const int c = is_v ? hd - a.Hq - a.Hkv : hd - a.Hq;
      dst = (T *)(is_v ? a.v_cache : a.k_cache) + (int64_t)a.kv_rows[m] * a.stride_tok +
            (int64_t)c * a.stride_head;
    }
    Elem<T>::store(dst + f, o0);
    Elem<T>::store(dst + f + half, o1);
  }
}

template <auto kKern, class Args>
hipError_t launch_skinny(int lds, dim3 grid, int threads, const Args &a, hipStream_t st) {
  // more than 64 KB of dynamic LDS has to be allowed once per kernel
  static const hipError_t attr = hipFuncSetAttribute(
      (const void *)kKern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
  if (attr != hipSuccess) return attr;
  hipLaunchKernelGGL(kKern, grid, dim3(threads), lds, st, a);
  return hipGetLastError();
}

}  // namespace

// The matrix-core kernels are instantiated for 7 and 8 slices of 512 (H = 3584, 4096).
bool hsr_mfma_supported(int dtype, int H) {
  return dtype == SPARROW_BF16 && (H == 7 * kSlice || H == 8 * kSlice);
}

hipError_t launch_hsr_fc(int dtype, const HsrFcArgs &a, hipStream_t st) {
  const int rbs = (a.M + 15) / 16;
  if (hsr_mfma_supported(dtype, a.H) && a.M == 1) {      // one row: a wavefront per output feature
    const dim3 grid((a.H + 3) / 4);
    if (a.H == 7 * kSlice) hipLaunchKernelGGL(hsr_fc_gemv_kernel<14>, grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL(hsr_fc_gemv_kernel<16>, grid, dim3(256), 0, st, a);
    return hipGetLastError();
  }
  if (hsr_mfma_supported(dtype, a.H)) {
    const dim3 grid(a.H / 16, rbs);
    // K = 2H: two slices per wavefront
    if (a.H == 7 * kSlice) return launch_skinny<hsr_fc_mfma_kernel<7, 2>>(skinny_lds_bytes(7, 1), grid, 7 * 64, a, st);
    if (a.H == 8 * kSlice) return launch_skinny<hsr_fc_mfma_kernel<8, 2>>(skinny_lds_bytes(8, 1), grid, 8 * 64, a, st);
  }
  const dim3 grid((a.H + 3) / 4);
  if (dtype == SPARROW_BF16) hipLaunchKernelGGL(hsr_fc_generic_kernel<bf16_t>, grid, dim3(256), 0, st, a);
  else hipLaunchKernelGGL(hsr_fc_generic_kernel<float>, grid, dim3(256), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_draft_qkv(int dtype, const DraftQkvArgs &a, hipStream_t st) {
  const int rbs = (a.M + 15) / 16;
  const int n_heads = a.Hq + 2 * a.Hkv;
  if (hsr_mfma_supported(dtype, a.H) && a.M == 1) {      // one row: a wavefront per rotary pair
    const dim3 grid((n_heads * (a.d / 2) + 3) / 4);
    if (a.H == 7 * kSlice) hipLaunchKernelGGL(draft_qkv_gemv_kernel<7>, grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL(draft_qkv_gemv_kernel<8>, grid, dim3(256), 0, st, a);
    return hipGetLastError();
  }
  if (hsr_mfma_supported(dtype, a.H)) {
    // two tiles per workgroup (d / 16 tiles per head: an even number): 144 workgroups at 36 heads
    // of 128 stay within one round on 256 compute units
    const dim3 grid(n_heads * (a.d / 16) / 2, rbs);
    if (a.H == 7 * kSlice) return launch_skinny<draft_qkv_mfma_kernel<7, 1>>(skinny_lds_bytes(7, 2), grid, 7 * 64, a, st);
    if (a.H == 8 * kSlice) return launch_skinny<draft_qkv_mfma_kernel<8, 1>>(skinny_lds_bytes(8, 2), grid, 8 * 64, a, st);
  }
  const dim3 grid((n_heads * (a.d / 2) + 3) / 4);
  if (dtype == SPARROW_BF16) hipLaunchKernelGGL(draft_qkv_generic_kernel<bf16_t>, grid, dim3(256), 0, st, a);
  else hipLaunchKernelGGL(draft_qkv_generic_kernel<float>, grid, dim3(256), 0, st, a);
  return hipGetLastError();
}

}  // namespace sparrow
