// Greedy acceptance, matrix-core lm_head pass: bf16, gfx950.
//
// logits[r, v] = sum_x hidden[r, x] * W[v, x] for the B*(n_q+1) verified rows r against the whole
// vocabulary; 1.09 GB of weights for Qwen2.5-VL-7B, read exactly once, so the pass is bound by HBM
// and organised around the weight stream:
//   - one persistent workgroup (8 wavefronts) per compute unit; the 16 hidden rows of the current
//     row block sit in LDS (XOR-swizzled 16-byte chunks) for the whole pass;
//   - the vocabulary is cut into tiles of 16 rows, dealt round-robin to all wavefronts of the chip
//     (at any moment the chip reads one contiguous region of W);
//   - a wavefront streams its tile's rows straight from HBM into the A operand of
//     v_mfma_f32_16x16x32_bf16 (lane = row + 16*kchunk: 16 rows x 64 contiguous bytes per load),
//     16 loads (16 KB) in flight per wavefront, double buffered in registers; B = hidden^T from LDS;
//   - logits never leave the registers: every lane keeps the best (value, lowest index) of the
//     vocabulary rows it has seen for its column; one candidate per (wavefront, row) is written at
//     the end and reduced by the finalize kernel.
// More than 16 rows (trees, batches) are handled as several row blocks, each a full pass over W.
#include "accept.hpp"
#include "common.hpp"

namespace sparrow {

namespace {

constexpr int kLmWaves = 8;               // wavefronts per workgroup
constexpr int kLmBlocks = 256;            // one workgroup per compute unit
constexpr int kLmChunk = 16;              // k-steps (of 32 elements) per register buffer

__global__ void __launch_bounds__(kLmWaves * 64)
lm_head_mfma_kernel(AcceptArgs a, int row0) {
  extern __shared__ __attribute__((aligned(16))) unsigned char hid[];   // [16 rows][H] bf16, swizzled

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int n = lane & 15, c4 = lane >> 4;
  const int H = a.H, V = a.V;
  const int row_bytes = H * 2;
  const int gw = blockIdx.x * kLmWaves + w;              // global wavefront = candidate slot
  const int n_waves = gridDim.x * kLmWaves;
  const int n_vt = (V + 15) / 16;                        // vocabulary tiles
  const int my_tiles = n_vt > gw ? (n_vt - gw + n_waves - 1) / n_waves : 0;
  const int chunks_per_tile = H / (32 * kLmChunk);
  const int nq = my_tiles * chunks_per_tile;             // register-buffer chunks of this wavefront
  const bf16_t *Wm = (const bf16_t *)a.lm_head;

  // A-operand loads of chunk q: tile gw + (q / cpt) * n_waves, k-steps (q % cpt) * 16 .. +16.
  // Unconditional (rows clamped to the last vocabulary row, chunk index clamped to the last chunk)
  // so that the number of loads in flight is static.
  auto issue = [&](int q, u32x4 *buf) {
    const int qq = min(q, max(nq - 1, 0));
    const int j = qq / chunks_per_tile, cidx = qq - j * chunks_per_tile;
    const int v = min((gw + j * n_waves) * 16 + n, V - 1);
    const bf16_t *p = Wm + (int64_t)v * H + cidx * (32 * kLmChunk) + 8 * c4;
#pragma unroll
    for (int s = 0; s < kLmChunk; ++s) buf[s] = __builtin_nontemporal_load((const u32x4 *)(p + 32 * s));
  };
  u32x4 bufA[kLmChunk], bufB[kLmChunk];
  issue(0, bufA);

  // hidden rows row0 .. row0+15 -> LDS (rows past M are zero)
  {
    const int cpr = H / 8;                               // 16-byte chunks per row
    for (int e = tid; e < 16 * cpr; e += kLmWaves * 64) {
      const int r = e / cpr, ch = e - r * cpr;
      u32x4 v = {0u, 0u, 0u, 0u};
      if (row0 + r < a.M) v = *(const u32x4 *)((const bf16_t *)a.hidden + (int64_t)(row0 + r) * H + 8 * ch);
      *reinterpret_cast<u32x4 *>(hid + r * row_bytes + (((ch & ~15) | ((ch & 15) ^ r)) << 4)) = v;
    }
  }
  __syncthreads();

  const unsigned char *hrow = hid + n * row_bytes;
  float best = -INFINITY;
  int best_i = 0x7fffffff;
  f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};

  auto compute = [&](int q, const u32x4 *buf) {
    const int j = q / chunks_per_tile, cidx = q - j * chunks_per_tile;
#pragma unroll
    for (int s = 0; s < kLmChunk; s += 2) {
      const int ch0 = 4 * (cidx * kLmChunk + s) + c4, ch1 = ch0 + 4;
      const bf16x8 b0 = *reinterpret_cast<const bf16x8 *>(hrow + (((ch0 & ~15) | ((ch0 & 15) ^ n)) << 4));
      const bf16x8 b1 = *reinterpret_cast<const bf16x8 *>(hrow + (((ch1 & ~15) | ((ch1 & 15) ^ n)) << 4));
      acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, buf[s]), b0, acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, buf[s + 1]), b1, acc1, 0, 0, 0);
    }
    if (cidx == chunks_per_tile - 1) {     // tile finished: lane holds logits of rows 4*c4 + i, column n
      const int vbase = (gw + j * n_waves) * 16 + 4 * c4;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float lg = acc0[i] + acc1[i];
        if (vbase + i < V && lg > best) { best = lg; best_i = vbase + i; }   // ascending: lowest wins
      }
      acc0 = (f32x4){0.f, 0.f, 0.f, 0.f};
      acc1 = (f32x4){0.f, 0.f, 0.f, 0.f};
    }
  };

  for (int q = 0; q < nq; q += 2) {
    issue(q + 1, bufB);
    compute(q, bufA);
    issue(q + 2, bufA);
    if (q + 1 < nq) compute(q + 1, bufB);
  }

  // best over the four lanes of a column (lanes n, n+16, n+32, n+48): lowest index on equal value
#pragma unroll
  for (int o = 16; o <= 32; o <<= 1) {
    const float ov = __shfl_xor(best, o, 64);
    const int oi = __shfl_xor(best_i, o, 64);
    if (ov > best || (ov == best && oi < best_i)) { best = ov; best_i = oi; }
  }
  if (c4 == 0 && row0 + n < a.M) {
    a.cand_val[(int64_t)(row0 + n) * a.n_cand + gw] = best;
    a.cand_idx[(int64_t)(row0 + n) * a.n_cand + gw] = best_i;
  }
}

}  // namespace

bool lm_head_mfma_supported(int dtype, int M, int H, int V) {
  (void)M; (void)V;
  // rows of W must split into whole register chunks, and the 16 hidden rows must fit in LDS
  return dtype == SPARROW_BF16 && H % (32 * kLmChunk) == 0 && 16 * H * 2 <= 144 * 1024;
}

int accept_num_candidates(int, int, int, int) { return kLmBlocks * kLmWaves; }

hipError_t launch_lm_head_mfma(const AcceptArgs &a, hipStream_t st) {
  const int lds = 16 * a.H * 2;
  static const hipError_t attr = hipFuncSetAttribute(
      (const void *)lm_head_mfma_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 144 * 1024);
  if (attr != hipSuccess) return attr;
  for (int row0 = 0; row0 < a.M; row0 += 16) {
    hipLaunchKernelGGL(lm_head_mfma_kernel, dim3(kLmBlocks), dim3(kLmWaves * 64), lds, st, a, row0);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace sparrow
