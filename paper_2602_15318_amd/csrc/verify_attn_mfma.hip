// Verification attention, matrix-core partial pass: bf16, head_dim 128, gfx950.
//
// One workgroup (4 wavefronts) owns one (context split, KV head, block of 64 rows); a row is a
// (draft row, query head of the group) pair, so all rows of a block share the K/V stream.
// K/V tiles of 32 tokens travel HBM -> registers (coalesced 16-byte loads, several tiles in
// flight) -> LDS (XOR-swizzled 16-byte chunks, double buffered) and are then read by all four
// wavefronts; wavefront w owns rows 16w..16w+15 of the block, so nothing is merged between
// wavefronts.
//
// Per tile and wavefront, with v_mfma_f32_16x16x32_bf16 (A: 16 x 32, lane = row + 16*kchunk;
// B: 32 x 16, lane = column + 16*kchunk; D: 16 x 16, lane = column + 16*(row/4), 4 rows each):
//   S^T = K Q^T   A = K rows from LDS (ds_read_b128), B = Q^T kept in registers.
//                 A lane then holds, for its query row, the scores of tokens 4c+0..3 (c = lane/16)
//                 of each 16-token sub-tile: row max / sum need two cross-lane steps only.
//   O^T += V^T P^T  B = P^T straight from the score registers (k index = the lane's own eight
//                 tokens), A = V^T through the transposing LDS read ds_read_b64_tr_b16.
// The online-softmax state (m, l) and the rescale factor are per lane (= per query row).
#include "common.hpp"
#include "verify_attn.hpp"

namespace sparrow {

namespace {

constexpr int kTile = 32;                 // tokens per tile
constexpr int kRowBytes = 256;            // one K or V row of a head: 128 bf16
constexpr int kTileBytes = kTile * kRowBytes;
constexpr int kPrefetch = 3;              // tiles in flight in registers
constexpr int kRowsPerWG = 64;

typedef __attribute__((address_space(3))) unsigned char lds_byte;

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

__global__ void __launch_bounds__(256)
verify_partial_mfma_kernel(VerifyArgs a, SeqTable tab) {
  __shared__ __attribute__((aligned(16))) unsigned char lds[2][2][kTileBytes];  // [buf][K,V]

  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
  const int n = lane & 15, c4 = lane >> 4;
  const int slot = blockIdx.x, c = blockIdx.y, rb = blockIdx.z;
  const int g = a.Hq / a.Hkv;
  const int R = a.n_q * g;
  const int b = seq_of_slot(tab, a.B, slot);
  const int len = tab.cu_len[b + 1] - tab.cu_len[b];
  const int L = len - a.n_q;
  const int t0 = (slot - tab.cu_split[b]) * a.chunk;
  const int t1 = min(len, t0 + a.chunk);
  const int n_tiles = (t1 - t0 + kTile - 1) / kTile;
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
  auto issue = [&](int tile, u32x4 *st) {
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
    *reinterpret_cast<u32x4 *>(&lds[buf][0][st_off_a]) = st[0];
    *reinterpret_cast<u32x4 *>(&lds[buf][0][st_off_b]) = st[1];
    *reinterpret_cast<u32x4 *>(&lds[buf][1][st_off_a]) = st[2];
    *reinterpret_cast<u32x4 *>(&lds[buf][1][st_off_b]) = st[3];
  };

#pragma unroll
  for (int p = 0; p < kPrefetch; ++p)
    if (p < n_tiles) issue(p, stage[p]);

  // ---- Q^T operand (B of the score MFMA): lane (n, c4) holds Q[row][32*ks + 8*c4 .. +8]
  bf16x8 qreg[4];
  {
    const bf16_t *qp = (const bf16_t *)a.q + (((int64_t)b * a.n_q + i_row) * a.Hq + h) * 128 + 8 * c4;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      u32x4 v = {0u, 0u, 0u, 0u};
      if (row_ok) v = *(const u32x4 *)(qp + 32 * ks);
      qreg[ks] = __builtin_bit_cast(bf16x8, v);
    }
  }
  // draft rows this row may attend (bit j <=> draft row j); only needed if the split reaches them
  unsigned long long anc = 0ull;
  if (row_ok && t1 > L) anc = ancestor_mask(a.parent, i_row);

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
    const unsigned char *Ks = &lds[buf][0][0];
    const unsigned char *Vs = &lds[buf][1][0];
    const int tb = t0 + tile * kTile;
    f32x4 s[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      s[j] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const bf16x8 ka = lds_read_b128(Ks + j * 16 * kRowBytes + k_off + (((4 * ks + c4) ^ k_swz) << 4));
        s[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka, qreg[ks], s[j], 0, 0, 0);
      }
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
          bool ok = tok < t1;
          if (tok >= L) ok = ok && ((anc >> (tok - L)) & 1ull);
          sc[4 * j + i] = ok ? sc[4 * j + i] : -INFINITY;
        }
    }
    float mx = sc[0];
#pragma unroll
    for (int e = 1; e < 8; ++e) mx = fmaxf(mx, sc[e]);
    mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
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
      const int ch = ((2 * mt + v_chb) ^ v_swz) << 4;
      const bf16x4 va = lds_read_tr(Vs + v_off + ch);
      const bf16x4 vb = lds_read_tr(Vs + 16 * kRowBytes + v_off + ch);
      const bf16x8 vt = __builtin_shufflevector(va, vb, 0, 1, 2, 3, 4, 5, 6, 7);
      o_acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vt, pb, o_acc[mt], 0, 0, 0);
    }
  };

  // ---- main loop: unrolled by the prefetch depth so the staging registers are static
  for (int base = 0; base < n_tiles; base += kPrefetch) {
#pragma unroll
    for (int p = 0; p < kPrefetch; ++p) {
      const int tile = base + p;
      if (tile < n_tiles) {            // uniform over the workgroup
        const int buf = tile & 1;
        stash(buf, stage[p]);
        if (tile + kPrefetch < n_tiles) issue(tile + kPrefetch, stage[p]);
        __syncthreads();
        if (wave_active) compute(tile, buf);
      }
    }
  }

  // ---- partial results of this split
  l_run += __shfl_xor(l_run, 16, 64);
  l_run += __shfl_xor(l_run, 32, 64);
  if (row_ok) {
    const int64_t pidx = ((int64_t)slot * a.n_q + i_row) * a.Hq + h;
    float *po = a.part_o + pidx * 128 + 4 * c4;
#pragma unroll
    for (int mt = 0; mt < 8; ++mt) *reinterpret_cast<f32x4 *>(po + 16 * mt) = o_acc[mt];
    if (c4 == 0) {
      a.part_ml[pidx * 2] = m_run;
      a.part_ml[pidx * 2 + 1] = l_run;
    }
  }
}

}  // namespace

bool verify_partial_mfma_supported(int dtype, int head_dim) {
  return dtype == SPARROW_BF16 && head_dim == 128;
}

hipError_t launch_verify_partial_mfma(const VerifyArgs &a, const SeqTable &tab, hipStream_t st) {
  const int R = a.n_q * (a.Hq / a.Hkv);
  dim3 grid(a.n_slots, a.Hkv, (R + kRowsPerWG - 1) / kRowsPerWG);
  hipLaunchKernelGGL(verify_partial_mfma_kernel, grid, dim3(256), 0, st, a, tab);
  return hipGetLastError();
}

}  // namespace sparrow
