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
// More than 16 rows (trees, batches): the k-split kernel takes 32 rows per pass over W, the
// fallback kernel 16.
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
        if (a.logits != nullptr && vbase + i < V && row0 + n < a.M)
          a.logits[(int64_t)(row0 + n) * V + vbase + i] = lg;
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


// ------------------------------------------------------------------------------------------------
// k-split version, used when hidden = NW * 512 with NW <= 16 (3584 -> 7 wavefronts): the fast path.
//
// A workgroup of NW wavefronts owns groups of 64 consecutive vocabulary rows (4 MFMA tiles);
// wavefront w owns the k-slice [512 w, 512 w + 512) of every row: its slice of the 16 hidden rows
// lives in registers for the whole pass (16 B operands), and every load instruction of the
// wavefront reads 1 KB that is contiguous in memory (the slice of one weight row), so the
// workgroup as a whole sweeps 448 KB of W front to back.  The 16-row tile goes registers -> LDS
// (private 16 KB per wavefront, XOR swizzled) -> A operands.  The wavefronts' partial logits of a
// group are summed through LDS; wavefront g < 4 then owns the argmax bookkeeping of tile g.
constexpr int kKsGroup = 4;               // vocabulary tiles (of 16 rows) per group

// NB = blocks of 16 hidden rows handled in one pass over W (1 or 2); the vocabulary group is
// kKsGroup / NB tiles so that the partial logits held in registers stay at 16 per lane.
// halves = 2 (33 to 64 hidden rows): ONE pass over W for two blocks of 32 rows.  The workgroups
// form pairs that stream the same vocabulary tiles, one for rows row0 .. row0+31, the other for
// rows row0+32 .. row0+63; the two of a pair have indices 8 apart, i.e. they run at the same time
// on the same XCD (workgroups are handed to the 8 XCDs round-robin), so the second fetch of a
// weight tile is served by that XCD's L2 and HBM still sees the weights once.  (Only the speed
// depends on that placement.)
template <int NW, int NB>
__global__ void __launch_bounds__(NW * 64)
lm_head_ksplit_kernel(AcceptArgs a, int row0_arg, int halves) {
  const int half = halves == 2 ? ((int)blockIdx.x >> 3) & 1 : 0;
  const int wg = halves == 2 ? ((int)blockIdx.x >> 4) * 8 + ((int)blockIdx.x & 7) : (int)blockIdx.x;
  const int n_wg = (int)gridDim.x / halves;            // streams of vocabulary tiles
  const int row0 = row0_arg + 32 * half;
  constexpr int G = kKsGroup / NB;          // vocabulary tiles per group
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  // [NW][16 KB] staging, then [NW][G][64] f32x4 partial logits
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = lane & 15, c4 = lane >> 4;
  const int H = a.H, V = a.V;
  const bf16_t *Wm = (const bf16_t *)a.lm_head;
  unsigned char *stg = smem + w * 16384;
  f32x4 *red = reinterpret_cast<f32x4 *>(smem + NW * 16384);

  // Vocabulary tiles (16 rows) are dealt round-robin to the workgroups one by one, so that the
  // workgroups' shares differ by at most one tile (9,504 tiles over 256 workgroups: 38 against a
  // mean of 37.1; dealt in groups of four tiles it was 40 against 37.1, and the kernel ends with
  // its slowest workgroup); a workgroup still reduces its tiles in groups of G, the last group
  // possibly short.
  const int n_vt = (V + 15) / 16;
  const int n_tiles = n_vt > wg ? (n_vt - wg + n_wg - 1) / n_wg : 0;

  // tile t of this workgroup -> first vocabulary row
  auto tile_row0 = [&](int t) { return (wg + t * n_wg) * 16; };
  // 16 loads of 1 KB: load r = the k-slice of row r of the tile (rows clamped to the last row).
  // Issued unconditionally (tile index clamped) so that the number of loads in flight is static.
  // one tile (16 KB per wavefront, 112 KB per compute unit) in flight: the weight stream already
  // saturates HBM with that, a second tile in flight measured 2 us slower
  constexpr int kBufs = 1;
  u32x4 buf[kBufs][16];
  auto issue = [&](int t, u32x4 *bp) {
    const int v0 = tile_row0(min(t, max(n_tiles - 1, 0)));
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int v = min(v0 + r, V - 1);
      bp[r] = __builtin_nontemporal_load((const u32x4 *)(Wm + (int64_t)v * H + 512 * w + 8 * lane));
    }
  };
  issue(0, buf[0]);
  if (kBufs == 2) issue(1, buf[1]);

  // B operands: lane (n, c4) holds hidden[row0 + 16 nb + n][512 w + 32 ks + 8 c4 .. +8], ks = 0..15
  bf16x8 hreg[NB][16];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    const int row = row0 + 16 * nb + n;
    const bool ok = row < a.M;
    // Rows past M (padding of the last block) take the data of valid rows, row % M: their results
    // are never stored, and every lane then fetches a row of its own -- the paired workgroups of
    // the 33-to-64-row pass keep in step only if their prologues take the same time (with all
    // padding lanes on one row the pass took 330 us at 33 rows, with this 229 us)
    const bf16_t *hp = (const bf16_t *)a.hidden + (int64_t)(ok ? row : row % a.M) * H + 512 * w + 8 * c4;
#pragma unroll
    for (int ks = 0; ks < 16; ++ks) hreg[nb][ks] = __builtin_bit_cast(bf16x8, *(const u32x4 *)(hp + 32 * ks));
  }

  // staging: lane i of load r holds chunk i (16 bytes) of row r; stored at chunk position
  // (i & ~15) | ((i & 15) ^ r) so that the A-operand reads (16 rows, same chunk) hit all banks
  const int a_base = n * 1024;      // A read: row n, chunk 4 ks + c4
  float best[NB];
  int best_i[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) { best[nb] = -INFINITY; best_i[nb] = 0x7fffffff; }
  auto tile_step = [&](int t, u32x4 *bp) {
#pragma unroll
    for (int r = 0; r < 16; ++r)
      *reinterpret_cast<u32x4 *>(stg + r * 1024 + (((lane & ~15) | ((lane & 15) ^ r)) << 4)) = bp[r];
    issue(t + kBufs, bp);
    f32x4 acc[NB][2];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      acc[nb][0] = (f32x4){0.f, 0.f, 0.f, 0.f};
      acc[nb][1] = (f32x4){0.f, 0.f, 0.f, 0.f};
    }
#pragma unroll
    for (int ks = 0; ks < 16; ks += 2) {
      const int ch0 = 4 * ks + c4, ch1 = ch0 + 4;
      const bf16x8 a0 = *reinterpret_cast<const bf16x8 *>(stg + a_base + (((ch0 & ~15) | ((ch0 & 15) ^ n)) << 4));
      const bf16x8 a1 = *reinterpret_cast<const bf16x8 *>(stg + a_base + (((ch1 & ~15) | ((ch1 & 15) ^ n)) << 4));
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        acc[nb][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, hreg[nb][ks], acc[nb][0], 0, 0, 0);
        acc[nb][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, hreg[nb][ks + 1], acc[nb][1], 0, 0, 0);
      }
    }
    const int g = t % G;
    // the tile's partial logits go to LDS at once ([row block][wavefront][tile of the group]: G * NB
    // = 4 slots per wavefront whatever NB), not into registers held for the whole group
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) red[((nb * NW + w) * G + g) * 64 + lane] = acc[nb][0] + acc[nb][1];
    if (g == G - 1 || t == n_tiles - 1) {     // uniform over the workgroup
      // sum the group's partial logits over the wavefronts; wavefront w <= g takes tile w of the
      // group (the last group may hold fewer than G tiles)
      __syncthreads();
      if (w <= g) {
        const int vbase = tile_row0(t - g + w) + 4 * c4;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
          f32x4 sum = red[((nb * NW + 0) * G + w) * 64 + lane];
#pragma unroll
          for (int ww = 1; ww < NW; ++ww) sum += red[((nb * NW + ww) * G + w) * 64 + lane];
#pragma unroll
          for (int i = 0; i < 4; ++i)
            if (vbase + i < V && sum[i] > best[nb]) { best[nb] = sum[i]; best_i[nb] = vbase + i; }
          if (a.logits != nullptr) {
            const int row = row0 + 16 * nb + n;
#pragma unroll
            for (int i = 0; i < 4; ++i)
              if (vbase + i < V && row < a.M) a.logits[(int64_t)row * V + vbase + i] = sum[i];
          }
        }
      }
      __syncthreads();   // reads done before the next partials are written
    }
  };
  // (unrolled by the number of register buffers so that each step names its own)
  for (int t = 0; t < n_tiles; t += kBufs) {
    tile_step(t, buf[0]);
    if (kBufs == 2 && t + 1 < n_tiles) tile_step(t + 1, buf[kBufs - 1]);
  }

  // a pair's workgroup leaves neutral candidates for the rows of the other half in its slots
  if (halves == 2) {
    const int other0 = row0_arg + 32 * (1 - half);
    for (int e = tid; e < 32 * kKsGroup; e += NW * 64) {
      const int row = other0 + e / kKsGroup;
      if (row < a.M) {
        const int slot = blockIdx.x * kKsGroup + e % kKsGroup;
        a.cand_val[(int64_t)row * a.n_cand + slot] = -INFINITY;
        a.cand_idx[(int64_t)row * a.n_cand + slot] = 0x7fffffff;
      }
    }
  }
  // candidates: wavefronts 0..G-1 hold, per lane, the best of tiles g = w over all groups; the
  // workgroup always fills kKsGroup candidate slots (the others stay at -inf)
  if (w < kKsGroup) {
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      float bv = best[nb];
      int bi = best_i[nb];
#pragma unroll
      for (int o = 16; o <= 32; o <<= 1) {
        const float ov = __shfl_xor(bv, o, 64);
        const int oi = __shfl_xor(bi, o, 64);
        if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
      }
      const int row = row0 + 16 * nb + n;
      if (c4 == 0 && row < a.M) {
        const int slot = blockIdx.x * kKsGroup + w;
        a.cand_val[(int64_t)row * a.n_cand + slot] = bv;
        a.cand_idx[(int64_t)row * a.n_cand + slot] = bi;
      }
    }
  }
}

template <int NW, int NB>
hipError_t launch_ksplit_nb(const AcceptArgs &a, int row0, int halves, hipStream_t st) {
  const int lds = NW * 16384 + NW * kKsGroup * 64 * 16;
  static const hipError_t attr = hipFuncSetAttribute(
      (const void *)lm_head_ksplit_kernel<NW, NB>, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
  if (attr != hipSuccess) return attr;
  hipLaunchKernelGGL((lm_head_ksplit_kernel<NW, NB>), dim3(kLmBlocks), dim3(NW * 64), lds, st, a, row0, halves);
  return hipGetLastError();
}

// One pass over W per 64 hidden rows by paired workgroups while more than 32 rows are left, then
// one pass for the last 17 to 32 rows, or for the last 16 or fewer.
template <int NW>
hipError_t launch_ksplit(const AcceptArgs &a, hipStream_t st) {
  for (int row0 = 0; row0 < a.M;) {
    const int left = a.M - row0;
    hipError_t e;
    if (left > 32) { e = launch_ksplit_nb<NW, 2>(a, row0, 2, st); row0 += 64; }
    else if (left > 16) { e = launch_ksplit_nb<NW, 2>(a, row0, 1, st); row0 += 32; }
    else { e = launch_ksplit_nb<NW, 1>(a, row0, 1, st); row0 += 16; }
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

bool ksplit_ok(int H) { return H == 3584 || H == 4096; }

}  // namespace

bool lm_head_mfma_supported(int dtype, int M, int H, int V) {
  (void)M; (void)V;
  // rows of W must split into whole register chunks, and the 16 hidden rows must fit in LDS
  return dtype == SPARROW_BF16 && H % (32 * kLmChunk) == 0 && 16 * H * 2 <= 144 * 1024;
}

int accept_num_candidates(int, int, int H, int) {
  return ksplit_ok(H) ? kLmBlocks * kKsGroup : kLmBlocks * kLmWaves;
}

hipError_t launch_lm_head_mfma(const AcceptArgs &a, hipStream_t st) {
  if (a.H == 3584) return launch_ksplit<7>(a, st);
  if (a.H == 4096) return launch_ksplit<8>(a, st);
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
