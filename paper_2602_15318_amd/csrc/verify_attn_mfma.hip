// Verification attention, matrix-core partial pass: bf16, head_dim 128, gfx950.
//
// One workgroup (8 wavefronts) owns one (context split, KV head, block of 64 rows); a row is a
// (draft row, query head of the group) pair, so all rows of a block share the K/V stream.
// The workgroup runs two token streams (wavefronts 0-3 and 4-7) that take alternate 32-token
// tiles; within a stream wavefront w owns rows 16w..16w+15 of the block, so rows are never merged
// between wavefronts and the two streams are merged once, through LDS, at the end.
// K/V tiles travel HBM -> registers (coalesced 16-byte loads, several tiles in flight) -> LDS
// (XOR-swizzled 16-byte chunks, double buffered per stream) and are read by the four wavefronts
// of the stream.
//
// Per tile and wavefront, with v_mfma_f32_16x16x32_bf16 (A: 16 x 32, lane = row + 16*kchunk;
// B: 32 x 16, lane = column + 16*kchunk; D: 16 x 16, lane = column + 16*(row/4), 4 rows each):
//   S^T = K Q^T   A = K rows from LDS (ds_read_b128), B = Q^T kept in registers.
//                 A lane then holds, for its query row, the scores of tokens 4c+0..3 (c = lane/16)
//                 of each 16-token sub-tile: the row max needs two cross-lane steps only.
//   O^T += V^T P^T  B = P^T straight from the score registers (k index = the lane's own eight
//                 tokens), A = V^T through the transposing LDS read ds_read_b64_tr_b16.
// The online-softmax state (m, l) and the rescale factor are per lane (= per query row).
#include "common.hpp"
#include "verify_attn.hpp"
#ifndef SPARROW_EXP
#define SPARROW_EXP 0
#endif

namespace sparrow {

namespace {

constexpr int kTile = 32;                 // tokens per tile
constexpr int kRowBytes = 256;            // one K or V row of a head: 128 bf16
constexpr int kTileBytes = kTile * kRowBytes;
constexpr int kPrefetch = 3;              // tiles per stream in flight in registers
constexpr int kRowsPerWG = 64;
constexpr int kStreams = 2;

// Swizzle of the 16-byte chunk index by the token row: a bijection on 0..15 per row whose upper
// three bits differ for rows 0..7, so a half-wavefront of transposing reads (8 rows x 32 bytes)
// and a quarter-wavefront of 16-byte reads (16 rows, same chunk) each cover all banks once.
__device__ __forceinline__ int swz(int row) { return ((row & 7) << 1) | ((row >> 3) & 1); }

__device__ __forceinline__ bf16x8 lds_read_b128(const unsigned char *p) {
  return *reinterpret_cast<const bf16x8 *>(p);
}

__device__ __forceinline__ bf16x4 lds_read_tr(const unsigned char *p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4bf16((__attribute__((address_space(3))) bf16x4 *)p);
}

// max / sum over the four lanes l, l^16, l^32, l^48 (the four k-chunk lanes of one query row),
// with the gfx950 row-swap instructions (no LDS round trip).
__device__ __forceinline__ float quad_max(float v) {
  auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  v = fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
  r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float quad_sum(float v) {
  auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  v = __uint_as_float(r[0]) + __uint_as_float(r[1]);
  r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

__global__ void __launch_bounds__(256 * kStreams)
verify_partial_mfma_kernel(VerifyArgs a, SeqTable tab) {
  // [stream][buf][K,V]; after the main loop the first 32 KB + 2 KB are reused for the stream merge
  __shared__ __attribute__((aligned(16))) unsigned char lds[kStreams][2][2][kTileBytes];

#ifdef SPARROW_TRACE
  long long tr[40]; int ntr = 0;
#define TR() do { if (ntr < 40) tr[ntr++] = wall_clock64(); } while (0)
#else
#define TR() do {} while (0)
#endif
  TR();
  const int tid = threadIdx.x & 255, strm = threadIdx.x >> 8;
  const int w = tid >> 6, lane = tid & 63;
  const int n = lane & 15, c4 = lane >> 4;
  const int slot = blockIdx.x, c = blockIdx.y, rb = blockIdx.z;
  const int g = a.Hq / a.Hkv;
  const int R = a.n_q * g;
  const int b = seq_of_slot(tab, a.B, slot);
  const int len = tab.cu_len[b + 1] - tab.cu_len[b];
  const int L = len - a.n_q;
  const int t0 = (slot - tab.cu_split[b]) * a.chunk;
  const int t1 = min(len, t0 + a.chunk);
  const int n_tiles = (t1 - t0 + kTile - 1) / kTile;          // of the workgroup
  const int n_pairs = (n_tiles + kStreams - 1) / kStreams;    // loop trips, same for both streams
  const int64_t tok_base = tab.cu_len[b];
  const bf16_t *Kg = (const bf16_t *)a.k + c * a.stride_head;
  const bf16_t *Vg = (const bf16_t *)a.v + c * a.stride_head;

  // ---- this lane's query row
  const int rho = rb * kRowsPerWG + 16 * w + n;
  const bool row_ok = rho < R;
  const bool wave_active = (rb * kRowsPerWG + 16 * w) < R;
  const int i_row = row_ok ? rho / g : 0;
  const int h = row_ok ? c * g + rho % g : 0;

  // ---- tile loader: thread -> rows (tid/16) and (tid/16 + 16), 16-byte chunk tid%16
  const int ld_row = tid >> 4, ld_ch = tid & 15;
  u32x4 stage[kPrefetch][4];
  auto issue = [&](int tile, u32x4 *st) {   // tile: index within the workgroup's split
    const int tb = t0 + tile * kTile;
    const int ra = min(tb + ld_row, t1 - 1), rb2 = min(tb + ld_row + 16, t1 - 1);
    const int64_t oa = (tok_base + ra) * a.stride_tok + ld_ch * 8;
    const int64_t ob = (tok_base + rb2) * a.stride_tok + ld_ch * 8;
    st[0] = __builtin_nontemporal_load((const u32x4 *)(Kg + oa));
    st[1] = __builtin_nontemporal_load((const u32x4 *)(Kg + ob));
    st[2] = __builtin_nontemporal_load((const u32x4 *)(Vg + oa));
    st[3] = __builtin_nontemporal_load((const u32x4 *)(Vg + ob));
  };
  const int st_off_a = ld_row * kRowBytes + ((ld_ch ^ swz(ld_row)) << 4);
  const int st_off_b = st_off_a + 16 * kRowBytes;   // row + 16 has the same swizzle
  auto stash = [&](int buf, const u32x4 *st) {
    *reinterpret_cast<u32x4 *>(&lds[strm][buf][0][st_off_a]) = st[0];
    *reinterpret_cast<u32x4 *>(&lds[strm][buf][0][st_off_b]) = st[1];
    *reinterpret_cast<u32x4 *>(&lds[strm][buf][1][st_off_a]) = st[2];
    *reinterpret_cast<u32x4 *>(&lds[strm][buf][1][st_off_b]) = st[3];
  };

  // ---- Q^T operand (B of the score MFMA): lane (n, c4) holds Q[row][32*ks + 8*c4 .. +8]
  bf16x8 qreg[4];
  {
    const int64_t qrow = row_ok ? ((int64_t)b * a.n_q + i_row) * a.Hq + h : 0;   // clamped, zeroed below
    const bf16_t *qp = (const bf16_t *)a.q + qrow * 128 + 8 * c4;
    u32x4 qv[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) qv[ks] = *(const u32x4 *)(qp + 32 * ks);
    // Every vector-memory operation from here to the end of the main loop is unconditional, so
    // the number of loads in flight is a compile-time constant at every wait.
#pragma unroll
    for (int p = 0; p < kPrefetch; ++p) issue(kStreams * p + strm, stage[p]);
    // Q was requested before the 4*kPrefetch tile loads and loads retire in order: wait until at
    // most those are outstanding (vmcnt = 12, no wait on the other counters).
    static_assert(kPrefetch == 3, "the immediate below encodes vmcnt(4 * kPrefetch)");
    __builtin_amdgcn_s_waitcnt(0x0F7C);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      if (!row_ok) qv[ks] = (u32x4){0u, 0u, 0u, 0u};
      qreg[ks] = __builtin_bit_cast(bf16x8, qv[ks]);
    }
  }
  // draft rows this row may attend (bit j <=> draft row j); only needed if the split reaches them
  unsigned long long anc = 0ull;
  if (row_ok && t1 > L) anc = ancestor_mask(a.parent, i_row);

  TR();
  // LDS read offsets
  const int k_off = n * kRowBytes;                 // + subtile*16 rows, chunk (4*ks + c4) ^ swz(n)
  const int k_swz = swz(n);
  const int s16 = lane & 15;                       // source lane index within the 16-lane group
  const int v_row = 4 * c4 + (s16 >> 2);           // token within a 16-token sub-tile
  const int v_swz = swz(v_row);
  const int v_off = v_row * kRowBytes + ((s16 & 1) << 3);   // + chunk (2*mt + ((s16>>1)&1)) ^ swz
  const int v_chb = (s16 >> 1) & 1;

  float m_run = kNegBig, l_run = 0.f;
  f32x4 o_acc[8];
#pragma unroll
  for (int mt = 0; mt < 8; ++mt) o_acc[mt] = (f32x4){0.f, 0.f, 0.f, 0.f};

  auto compute = [&](int tile, int buf) {
    const unsigned char *Ks = &lds[strm][buf][0][0];
    const unsigned char *Vs = &lds[strm][buf][1][0];
    const int tb = t0 + tile * kTile;
    // all LDS reads of the tile are issued up front: K operands first, V operands land while the
    // scores and the softmax are computed
    bf16x8 ka[2][4];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int ks = 0; ks < 4; ++ks)
        ka[j][ks] = lds_read_b128(Ks + j * 16 * kRowBytes + k_off + (((4 * ks + c4) ^ k_swz) << 4));
    bf16x4 va[8], vb[8];
#pragma unroll
    for (int mt = 0; mt < 8; ++mt) {
      const int ch = ((2 * mt + v_chb) ^ v_swz) << 4;
      va[mt] = lds_read_tr(Vs + v_off + ch);
      vb[mt] = lds_read_tr(Vs + 16 * kRowBytes + v_off + ch);
    }
    f32x4 s[2] = {(f32x4){0.f, 0.f, 0.f, 0.f}, (f32x4){0.f, 0.f, 0.f, 0.f}};
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      s[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[0][ks], qreg[ks], s[0], 0, 0, 0);
      s[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[1][ks], qreg[ks], s[1], 0, 0, 0);
    }
    // scale, mask, online softmax (per lane = per query row)
    float sc[8];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int i = 0; i < 4; ++i) sc[4 * j + i] = s[j][i] * a.scale_log2;
    if (tb + kTile > min(t1, L)) {   // wavefront-uniform: tile touches the split end or draft rows
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int tok = tb + 16 * j + 4 * c4 + i;
          const int dj = tok - L;
          const bool vis = (dj < 0) | (((anc >> (dj & 63)) & 1ull) != 0ull);
          sc[4 * j + i] = ((tok < t1) & vis) ? sc[4 * j + i] : -INFINITY;
        }
    }
    float mx = fmaxf(fmaxf(fmaxf(sc[0], sc[1]), fmaxf(sc[2], sc[3])),
                     fmaxf(fmaxf(sc[4], sc[5]), fmaxf(sc[6], sc[7])));
    mx = quad_max(mx);
    const float m_new = fmaxf(m_run, mx);
    const float alpha = fast_exp2(m_run - m_new);
    m_run = m_new;
    float psum = 0.f;
    bf16x8 pb;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float p = fast_exp2(sc[e] - m_new);
      psum += p;
      pb[e] = (__bf16)p;
    }
    l_run = l_run * alpha + psum;
#pragma unroll
    for (int mt = 0; mt < 8; ++mt) {
      o_acc[mt] *= alpha;
      const bf16x8 vt = __builtin_shufflevector(va[mt], vb[mt], 0, 1, 2, 3, 4, 5, 6, 7);
      o_acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vt, pb, o_acc[mt], 0, 0, 0);
    }
  };

  // ---- main loop: unrolled by the prefetch depth so the staging registers are static.  Loads and
  // LDS stores also run for tiles past the end of the split (rows clamped to the last token, data
  // unused); only the compute is skipped for them.
  for (int base = 0; base < n_pairs; base += kPrefetch) {
#pragma unroll
    for (int p = 0; p < kPrefetch; ++p) {
      const int pair = base + p;
      const int tile = kStreams * pair + strm;
      const int buf = pair & 1;
#ifndef SPARROW_EXP
#define SPARROW_EXP 0
#endif
      if (!(SPARROW_EXP & 2)) stash(buf, stage[p]);
      if (!(SPARROW_EXP & 4)) issue(tile + kStreams * kPrefetch, stage[p]);
      TR();
      __syncthreads();
      TR();
      if (!(SPARROW_EXP & 1)) if (tile < n_tiles && wave_active) compute(tile, buf);
      TR();
    }
  }

  TR();
  // ---- merge the two streams (stream 1 -> LDS -> stream 0) and write the split's partials
  l_run = quad_sum(l_run);
  __syncthreads();                      // all tile reads done: LDS is free
  f32x4 *mo = reinterpret_cast<f32x4 *>(&lds[0][0][0][0]);           // [w][mt][lane]
  float *mm = reinterpret_cast<float *>(&lds[0][0][0][0] + 4 * 8 * 64 * 16);   // [w][lane][m,l]
  if (strm == 1) {
#pragma unroll
    for (int mt = 0; mt < 8; ++mt) mo[(w * 8 + mt) * 64 + lane] = o_acc[mt];
    mm[(w * 64 + lane) * 2] = m_run;
    mm[(w * 64 + lane) * 2 + 1] = l_run;
  }
  __syncthreads();
  if (strm == 0 && row_ok) {
    const float m1 = mm[(w * 64 + lane) * 2], l1 = mm[(w * 64 + lane) * 2 + 1];
    const float m_new = fmaxf(m_run, m1);
    const float a0 = fast_exp2(m_run - m_new), a1 = fast_exp2(m1 - m_new);
    const int64_t pidx = ((int64_t)slot * a.n_q + i_row) * a.Hq + h;
    float *po = a.part_o + pidx * 128 + 4 * c4;
#pragma unroll
    for (int mt = 0; mt < 8; ++mt) {
      const f32x4 o1 = mo[(w * 8 + mt) * 64 + lane];
      *reinterpret_cast<f32x4 *>(po + 16 * mt) = o_acc[mt] * a0 + o1 * a1;
    }
    if (c4 == 0) {
      a.part_ml[pidx * 2] = m_new;
      a.part_ml[pidx * 2 + 1] = l_run * a0 + l1 * a1;
    }
  }
  TR();
#ifdef SPARROW_TRACE
  if (a.lse && (threadIdx.x & 63) == 0 && blockIdx.y == 0 && (blockIdx.x == 0 || blockIdx.x == 30)) {
    long long *dst = (long long *)a.lse + ((blockIdx.x ? 1 : 0) * 8 + (threadIdx.x >> 6)) * 40;
    for (int i = 0; i < 40; ++i) dst[i] = i < ntr ? tr[i] : 0;
  }
#endif
}


}  // namespace

bool verify_partial_mfma_supported(int dtype, int head_dim) {
  return dtype == SPARROW_BF16 && head_dim == 128;
}

hipError_t launch_verify_partial_mfma(const VerifyArgs &a, const SeqTable &tab, hipStream_t st) {
  const int R = a.n_q * (a.Hq / a.Hkv);
  dim3 grid(a.n_slots, a.Hkv, (R + kRowsPerWG - 1) / kRowsPerWG);
  hipLaunchKernelGGL(verify_partial_mfma_kernel, grid, dim3(256 * kStreams), 0, st, a, tab);
  return hipGetLastError();
}

}  // namespace sparrow
