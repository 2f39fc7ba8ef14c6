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
#include <algorithm>
#include <type_traits>

#include "common.hpp"
#include "verify_attn.hpp"

namespace sparrow {

namespace {

constexpr int kTile = 32;                 // tokens per tile
constexpr int kRowBytes = 256;            // one K or V row of a head: 128 bf16
constexpr int kTileBytes = kTile * kRowBytes;
constexpr int kSub = 1;                   // 32-token tiles per stream per step
constexpr int kRowsPerWG = 64;
constexpr int kMlFloats = 3;              // per row of a partial: max, sum, output scale
constexpr int kStreams = 2;
constexpr float kSlack = 8.0f;            // log2 units a score may exceed a row's reference point

// Swizzle of the 16-byte chunk index by the token row: chunk c of row r is stored at chunk position
// c ^ ((r & 7) << 1).  Measured with the bank-conflict counter on the three access patterns of this
// kernel (16-byte writes of whole rows, 16-byte reads of 16 rows at one chunk, transposing 8-byte
// reads of 16 rows x 32 bytes): no conflict cycle on any of them.  Variants that also fold bit 3
// of the row in (so that rows r and r + 8 land on different chunks) doubled the cycles of the
// 16-byte operand reads -- two thirds of the kernel's LDS cycles were bank conflicts with it.
__device__ __forceinline__ int swz(int row) { return (row & 7) << 1; }

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

// kQT = 16-row tiles per wavefront: 1 serves up to 64 rows per workgroup (chains), 2 and 3 serve
// 128 and 192 (draft trees): the K and V^T operands read from LDS then feed every row tile, and a
// tree of R rows needs a half or a third as many passes over the K/V stream.  Three tiles take
// all 256 registers with one step in flight.
// kPrefetch = steps in flight in registers.  The whole split of a workgroup is only a handful of
// steps at decode-time sizes (7 at 26k context on 256 compute units), so a deep look-ahead turns
// the kernel into "load most of it, then compute": depth 3-4 is slower there, depth 2 wins from
// about four steps on, depth 1 for the shortest splits.
// Per-sequence split length in tokens (split_len of the sequence), worked out by the host so that
// the kernel's way to its first load holds no integer division.
struct PieceTable {
  int32_t piece[SPARROW_MAX_BATCH];
};

template <int kPrefetch, int kQT>
__global__ void __launch_bounds__(256 * kStreams)
verify_partial_mfma_kernel(VerifyArgs a, SeqTable tab, PieceTable pt, int rbs, int flat) {
  // [stream][buf][K,V][kSub tiles]; after the main loop the first 34 KB are reused for the merge
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  constexpr int kStepBytes = kSub * kTileBytes;            // K (or V) rows of one stream step
  auto lds_at = [&](int strm_, int buf, int kv) {
    return lds + ((strm_ * 2 + buf) * 2 + kv) * kStepBytes;
  };

  // wavefront-uniform indices as scalars, so that everything derived from them (which rows are
  // live, whether a step touches the split end) is decided by scalar branches
  const int wave_id = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int strm = wave_id >> 2, w = wave_id & 3;
  const int tid = threadIdx.x & 255, lane = threadIdx.x & 63;
  const int n = lane & 15, c4 = lane >> 4;
  // Workgroup -> (sequence, KV head, split of the sequence, row block).  Workgroups are handed to
  // the 8 XCDs round-robin by their linear index and gridDim.x is a multiple of 8, so x & 7 is
  // the XCD; the row blocks of one split stream the same K/V and get x values that are equal
  // modulo 8 and adjacent in that XCD's order: they run at the same time on one XCD and all but
  // the first fetch of a tile hit its L2.  (Only the speed depends on the round-robin placement.)
  // Two grid shapes:
  //  - (x, KV head, sequence): everything the first K/V load needs comes from ONE round of scalar
  //    loads of the arguments (the sequence's table entries are addressed by blockIdx.z) and no
  //    division -- at decode-time sizes the whole kernel lasts ~13 us and every dependent round
  //    trip before the first load shows.  x is sized for the sequence with the most splits; the
  //    XCD of a split is rotated by its global number, so that the splits of all heads and
  //    sequences together are dealt evenly to the XCDs.
  //  - flat (x only; for ragged batches, where the first shape would launch mostly padding):
  //    x enumerates (global split, KV head) and the sequence is searched in the split table.
  const int xj = blockIdx.x >> 3, xcd = blockIdx.x & 7;
  const int bz = blockIdx.z;               // (0 on the flat grid: no need to wait for `flat` to know it)
  const int cl0_z = tab.cu_len[bz], cl1_z = tab.cu_len[bz + 1];
  const int cs0_z = tab.cu_split[bz], cs1_z = tab.cu_split[bz + 1];
  const int piece_z = pt.piece[bz];
  // an empty statement that takes these values as scalar-register inputs: the compiler has to
  // have all of them loaded here, which makes it issue their loads together, ahead of the
  // branches below, instead of one round per use
  asm volatile("" ::"s"(rbs), "s"(flat), "s"(cl0_z), "s"(cl1_z), "s"(cs0_z), "s"(cs1_z), "s"(piece_z),
               "s"(a.k), "s"(a.v), "s"(a.stride_tok), "s"(a.stride_head), "s"(a.n_q), "s"(a.n_slots),
               "s"(a.Hkv));
  int rb = 0, sq = xj;
  if (rbs > 1) { rb = xj % rbs; sq = xj / rbs; }
  int b = bz, c, s_loc;
  int cl0 = cl0_z, len = cl1_z - cl0_z, cs0 = cs0_z, ns = cs1_z - cs0_z, piece = piece_z;
  if (flat) {
    const int grp = sq * 8 + xcd;                          // global split + n_slots * KV head
    if (grp >= a.n_slots * a.Hkv) return;                  // padding of the last round of 8
    const int gslot = grp % a.n_slots;
    c = grp / a.n_slots;
    b = seq_of_slot(tab, a.B, gslot);
    cl0 = tab.cu_len[b]; len = tab.cu_len[b + 1] - cl0;
    cs0 = tab.cu_split[b]; ns = tab.cu_split[b + 1] - cs0;
    piece = pt.piece[b];
    s_loc = gslot - cs0;
  } else {
    c = blockIdx.y;
    s_loc = sq * 8 + ((xcd - (cs0 + a.n_slots * c)) & 7);  // split within the sequence
    if (s_loc >= ns) return;                               // padding of the grid (uniform)
  }
  const int slot = cs0 + s_loc;
  const int L = len - a.n_q;
  const int t0 = min(len, s_loc * piece);
  const int t1 = min(len, t0 + piece);
  const int n_tiles = (t1 - t0 + kTile - 1) / kTile;                    // of the workgroup
  const int n_steps = (n_tiles + kStreams * kSub - 1) / (kStreams * kSub);   // loop trips
  // K/V of this sequence and head; a token row is addressed by a 32-bit byte offset from here
  // (the host checks that a sequence's K/V spans less than 2 GB)
  const int64_t seq_off = (int64_t)cl0 * a.stride_tok + (int64_t)c * a.stride_head;
  const unsigned char *Kg = (const unsigned char *)((const bf16_t *)a.k + seq_off);
  const unsigned char *Vg = (const unsigned char *)((const bf16_t *)a.v + seq_off);
  const unsigned int row_bytes = (unsigned int)a.stride_tok * 2u;

  // ---- loader: in step `st` stream `strm` owns tiles (st*kStreams + strm)*kSub .. +kSub, i.e.
  // 32*kSub consecutive tokens; thread -> rows tid/16 + 16 j, 16-byte chunk tid%16.  Rows past
  // the end of the split are clamped to its last token (loaded, never used), so every load is
  // unconditional and the number of loads in flight is a compile-time constant at every wait.
  const int ld_row = tid >> 4, ld_ch = tid & 15;
  constexpr int kLd = 2 * kSub;                       // 16-row slabs per step (per K and per V)
  u32x4 stage[kPrefetch][2 * kLd];
  auto issue = [&](int st, u32x4 *sg) {
    const int tb = t0 + (st * kStreams + strm) * kSub * kTile;
#pragma unroll
    for (int j = 0; j < kLd; ++j) {
      const int r = min(tb + ld_row + 16 * j, t1 - 1);
      const unsigned int o = (unsigned int)r * row_bytes + (unsigned int)ld_ch * 16u;
      sg[j] = __builtin_nontemporal_load((const u32x4 *)(Kg + o));
      sg[kLd + j] = __builtin_nontemporal_load((const u32x4 *)(Vg + o));
    }
  };
  // row r of the step lands at byte r*256 + ((chunk ^ swz(r)) * 16); swz depends on r mod 16 only
  const int st_off = ld_row * kRowBytes + ((ld_ch ^ swz(ld_row)) << 4);
  auto stash = [&](int buf, const u32x4 *sg) {
    unsigned char *kb = lds_at(strm, buf, 0), *vb = lds_at(strm, buf, 1);
#pragma unroll
    for (int j = 0; j < kLd; ++j) {
      *reinterpret_cast<u32x4 *>(kb + st_off + 16 * j * kRowBytes) = sg[j];
      *reinterpret_cast<u32x4 *>(vb + st_off + 16 * j * kRowBytes) = sg[kLd + j];
    }
  };

  // ---- first step, then Q^T (B operand of the score MFMA: lane (n, c4) holds
  // Q[row][32*ks + 8*c4 .. +8]), then the rest of the look-ahead.
  issue(0, stage[0]);
  __builtin_amdgcn_sched_barrier(0);      // the first step is on its way before anything else is worked out

  const int g = a.Hq / a.Hkv;
  const int R = a.n_q * g;
  const int rbs64 = (R + kRowsPerWG - 1) / kRowsPerWG;     // 64-row units of the partial layout
  // ---- this lane's query rows: one per row tile
  bool row_ok[kQT];
  int i_row[kQT], h[kQT];
  int n_act = 0;                                  // row tiles of this wavefront that hold rows
#pragma unroll
  for (int qt = 0; qt < kQT; ++qt) {
    const int rho = (rb * kQT + qt) * kRowsPerWG + 16 * w + n;
    row_ok[qt] = rho < R;
    if ((rb * kQT + qt) * kRowsPerWG + 16 * w < R) n_act = qt + 1;
    i_row[qt] = row_ok[qt] ? rho / g : 0;
    h[qt] = row_ok[qt] ? c * g + rho % g : 0;
  }

  bf16x8 qreg[kQT][4];
  {
    u32x4 qv[kQT][4];
#pragma unroll
    for (int qt = 0; qt < kQT; ++qt) {
      // rows past R read row 0 (in bounds) and are zeroed below
      const int64_t qrow = row_ok[qt] ? ((int64_t)b * a.n_q + i_row[qt]) * a.Hq + h[qt] : 0;
      const bf16_t *qp = (const bf16_t *)a.q + qrow * 128 + 8 * c4;
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) qv[qt][ks] = *(const u32x4 *)(qp + 32 * ks);
    }
    // The memory pipeline of a compute unit serves requests in issue order and a wavefront
    // issues all its loads back to back: without this barrier the look-ahead of the wavefronts
    // that issue first would queue ahead of the FIRST step of the others (measured: 3 us of
    // skew between the two streams).
    if (kPrefetch > 1) __syncthreads();
#pragma unroll
    for (int p = 1; p < kPrefetch; ++p) issue(p, stage[p]);
    // Loads retire in order: Q (and the first step before it) have landed once at most the
    // loads issued after Q are outstanding (other counters untouched).
    constexpr int kAfterQ = (kPrefetch - 1) * 2 * kLd;
    static_assert(kAfterQ < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt(0x0F70 | (kAfterQ & 15) | ((kAfterQ >> 4) << 14));
#pragma unroll
    for (int qt = 0; qt < kQT; ++qt)
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        if (!row_ok[qt]) qv[qt][ks] = (u32x4){0u, 0u, 0u, 0u};
        qreg[qt][ks] = __builtin_bit_cast(bf16x8, qv[qt][ks]);
      }
  }
  // draft rows a row may attend (bit j <=> draft row j); only needed if the split reaches them
  unsigned long long anc[kQT];
#pragma unroll
  for (int qt = 0; qt < kQT; ++qt) {
    anc[qt] = 0ull;
    if (t1 > L) {                                            // uniform over the workgroup
      anc[qt] = ancestor_mask_wave(a.parent ? a.parent + (int64_t)b * a.parent_stride : nullptr, a.n_q,
                                   i_row[qt], lane);
      if (!row_ok[qt]) anc[qt] = 0ull;
    }
  }

  // LDS read offsets
  const int k_off = n * kRowBytes;                 // + 16-row slab, chunk (4*ks + c4) ^ swz(n)
  const int k_swz = swz(n);
  const int s16 = lane & 15;                       // source lane index within the 16-lane group
  const int v_row = 4 * c4 + (s16 >> 2);           // token within a 16-token slab
  const int v_swz = swz(v_row);
  const int v_off = v_row * kRowBytes + ((s16 & 1) << 3);   // + chunk (2*mt + ((s16>>1)&1)) ^ swz
  const int v_chb = (s16 >> 1) & 1;

  float m_run[kQT];
  f32x4 l_acc[kQT];       // running sum of a row's exponentials, the same value in all 4 entries
  f32x4 o_acc[kQT][8];
  constexpr bool kMfmaRowSum = true;
  bf16x8 ones;
#pragma unroll
  for (int e = 0; e < 8; ++e) ones[e] = (__bf16)1.0f;
#pragma unroll
  for (int qt = 0; qt < kQT; ++qt) {
    m_run[qt] = kNegBig;
    l_acc[qt] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int mt = 0; mt < 8; ++mt) o_acc[qt][mt] = (f32x4){0.f, 0.f, 0.f, 0.f};
  }

  // One step of one stream: 32*kSub tokens against the wavefront's 16 rows, one joint softmax
  // update (a single running-max / rescale for the whole step).
  auto compute = [&](int st, int buf, auto na_tag) {
    constexpr int NA = decltype(na_tag)::value;   // live row tiles (the leading ones)
    const unsigned char *Ks = lds_at(strm, buf, 0);
    const unsigned char *Vs = lds_at(strm, buf, 1);
    const int tb = t0 + (st * kStreams + strm) * kSub * kTile;
    f32x4 s[NA][kLd];
    // Tree instances raise the wavefront's priority for their MFMA phases: the other wavefront of
    // the SIMD is then in its softmax, and the matrix pipe stays fed (-3 % on the 60-node tree).
    constexpr bool kPrio = kQT > 1;
    if (kPrio) __builtin_amdgcn_s_setprio(1);
#pragma unroll
    for (int j = 0; j < kLd; ++j) {
      bf16x8 ka[4];
#pragma unroll
      for (int ks = 0; ks < 4; ++ks)
        ka[ks] = lds_read_b128(Ks + j * 16 * kRowBytes + k_off + (((4 * ks + c4) ^ k_swz) << 4));
#pragma unroll
      for (int qt = 0; qt < NA; ++qt) s[qt][j] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < 4; ++ks)
#pragma unroll
        for (int qt = 0; qt < NA; ++qt)
          s[qt][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[ks], qreg[qt][ks], s[qt][j], 0, 0, 0);
    }
    // mask, online softmax (per lane = per query row).  Scores stay unscaled until the exponent:
    // exp2(s * scale_log2 - m) is one fused multiply-add per score (scale_log2 > 0, so the
    // maximum can be taken before scaling).
    if (kPrio) __builtin_amdgcn_s_setprio(0);
    const bool edge = tb + kSub * kTile > min(t1, L);   // uniform: split end or draft rows in reach
    if (kQT > 1) __builtin_amdgcn_sched_barrier(0);     // keep the V^T reads below the softmax
    bf16x8 pb[NA][kSub];
#pragma unroll
    for (int qt = 0; qt < NA; ++qt) {
      float sc[4 * kLd];
#pragma unroll
      for (int j = 0; j < kLd; ++j)
#pragma unroll
        for (int i = 0; i < 4; ++i) sc[4 * j + i] = s[qt][j][i];
      if (edge) {
        // (an opaque copy of the step's first token: without it the compiler works the token
        // numbers, their distances to L and the shift counts out on EVERY step, ahead of the
        // branch -- some 20 vector instructions per row tile that all but one step throw away)
        int tb_e = tb;
        asm volatile("" : "+s"(tb_e));
#pragma unroll
        for (int j = 0; j < kLd; ++j)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int tok = tb_e + 16 * j + 4 * c4 + i;
            const int dj = tok - L;
            const bool vis = (dj < 0) | (((anc[qt] >> (dj & 63)) & 1ull) != 0ull);
            sc[4 * j + i] = ((tok < t1) & vis) ? sc[4 * j + i] : -INFINITY;
          }
      }
      float mx = sc[0];
#pragma unroll
      for (int e = 1; e < 4 * kLd; ++e) mx = fmaxf(mx, sc[e]);
      mx *= a.scale_log2;
      // The reference point m of a row moves only when some score of the wavefront's tile lies
      // more than kSlack above it (exponentials then stay below 2^kSlack, far from overflow, and
      // softmax does not depend on the reference point): the cross-lane maximum, the rescale
      // factor and the 32 accumulator multiplies are skipped for almost every tile.
      if (__builtin_amdgcn_ballot_w64(mx > m_run[qt] + kSlack) != 0ull) {
        const float m_new = fmaxf(m_run[qt], quad_max(mx));
        const float alpha = fast_exp2(m_run[qt] - m_new);
        m_run[qt] = m_new;
        if (kMfmaRowSum) l_acc[qt] *= alpha; else l_acc[qt][0] *= alpha;
#pragma unroll
        for (int mt = 0; mt < 8; ++mt) o_acc[qt][mt] *= alpha;
      }
#pragma unroll
      for (int u = 0; u < kSub; ++u) {
        float psum = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float p = fast_exp2(fmaf(sc[8 * u + e], a.scale_log2, -m_run[qt]));
          if (!kMfmaRowSum) psum += p;
          pb[qt][u][e] = (__bf16)p;
        }
        // row sums on the matrix cores: every row of ones . P^T is the sum over the 32 tokens
        // (kMfmaRowSum off: per-lane sums on the vector ALU, merged across the four lanes at the end)
        if (kMfmaRowSum)
          l_acc[qt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, pb[qt][u], l_acc[qt], 0, 0, 0);
        else
          l_acc[qt][0] += psum;
      }
    }
    if (kQT > 1) __builtin_amdgcn_sched_barrier(0);
    if (kPrio) __builtin_amdgcn_s_setprio(1);
#pragma unroll
    for (int mt = 0; mt < 8; ++mt) {
      const int ch = ((2 * mt + v_chb) ^ v_swz) << 4;
      if (kQT > 1 && mt == 4) __builtin_amdgcn_sched_barrier(0);    // at most 4 d-tiles of V^T in flight
#pragma unroll
      for (int u = 0; u < kSub; ++u) {
        const bf16x4 va = lds_read_tr(Vs + (2 * u) * 16 * kRowBytes + v_off + ch);
        const bf16x4 vb = lds_read_tr(Vs + (2 * u + 1) * 16 * kRowBytes + v_off + ch);
        const bf16x8 vt = __builtin_shufflevector(va, vb, 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
        for (int qt = 0; qt < NA; ++qt)
          o_acc[qt][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vt, pb[qt][u], o_acc[qt][mt], 0, 0, 0);
      }
    }
    if (kPrio) __builtin_amdgcn_s_setprio(0);
  };

  // A wavefront with a partly filled set of row tiles computes all of them (the empty ones on a zero
  // query): a second, one-tile instance of the step in the same kernel costs more registers than
  // the kernel has.
  auto run = [&](int st, int buf) {
    if (n_act > 0) compute(st, buf, std::integral_constant<int, kQT>{});
  };

  // ---- main loop, unrolled by the prefetch depth so that the staging registers are static.
  // Look-ahead loads past the end of the split are clamped duplicates of its last rows.
  int base = 0;
  for (; base + kPrefetch <= n_steps; base += kPrefetch) {
#pragma unroll
    for (int p = 0; p < kPrefetch; ++p) {
      const int st = base + p;
      const int buf = st & 1;
      stash(buf, stage[p]);
      issue(st + kPrefetch, stage[p]);
      __syncthreads();
      if ((st * kStreams + strm) * kSub < n_tiles) run(st, buf);
    }
  }
  // remainder (n_steps % kPrefetch trips): everything it needs is already in flight
#pragma unroll
  for (int p = 0; p < kPrefetch - 1; ++p) {
    const int st = base + p;
    if (st < n_steps) {                    // uniform over the workgroup
      const int buf = st & 1;
      stash(buf, stage[p]);
      __syncthreads();
      if ((st * kStreams + strm) * kSub < n_tiles) run(st, buf);
    }
  }

  // ---- merge the two streams (stream 1 -> LDS -> stream 0) and write the split's partials in
  // register layout: [slot][kv head][row block][wavefront][pair of d-tiles][lane] x 8 halves, so
  // that every store instruction writes 1 KB of contiguous memory.
  f32x4 *mo = reinterpret_cast<f32x4 *>(lds);                                  // [w][mt][lane]
  float *mm = reinterpret_cast<float *>(lds + 4 * 8 * 64 * 16);                // [w][lane][m,l]
#pragma unroll
  for (int qt = 0; qt < kQT; ++qt) {
    const float l_mine = kMfmaRowSum ? l_acc[qt][0] : quad_sum(l_acc[qt][0]);
    __syncthreads();                    // all tile reads (and the previous merge) done: LDS is free
    if (strm == 1) {
#pragma unroll
      for (int mt = 0; mt < 8; ++mt) mo[(w * 8 + mt) * 64 + lane] = o_acc[qt][mt];
      mm[(w * 64 + lane) * 2] = m_run[qt];
      mm[(w * 64 + lane) * 2 + 1] = l_mine;
    }
    __syncthreads();
    if (strm == 0 && qt < n_act) {
      const float m1 = mm[(w * 64 + lane) * 2], l1 = mm[(w * 64 + lane) * 2 + 1];
      const float m_new = fmaxf(m_run[qt], m1);
      const float a0 = fast_exp2(m_run[qt] - m_new), a1 = fast_exp2(m1 - m_new);
      // unit = (split, KV head, block of 64 rows).  The split's output is stored normalised
      // (o / l: a convex combination of V rows, of the magnitude of V) in fp16, two d-tiles per
      // 16-byte store; m, l and a per-row power-of-two scale c in fp32.  c is 1 unless the row's
      // largest |o / l| would leave the fp16 range (|V| beyond 16384), then o / (l c) is stored.
      const int64_t unit = ((int64_t)slot * a.Hkv + c) * rbs64 + rb * kQT + qt;
      const float l_tot = l_mine * a0 + l1 * a1;
      const float inv_l = l_tot > 0.f ? 1.0f / l_tot : 0.f;
      const float s0 = a0 * inv_l, s1 = a1 * inv_l;
      float amax = 0.f;
#pragma unroll
      for (int mt = 0; mt < 8; ++mt) {
        o_acc[qt][mt] = o_acc[qt][mt] * s0 + mo[(w * 8 + mt) * 64 + lane] * s1;
#pragma unroll
        for (int i = 0; i < 4; ++i) amax = fmaxf(amax, fabsf(o_acc[qt][mt][i]));
      }
      amax = quad_max(amax);                       // over the row's 128 values
      float cscale = 1.0f, inv_c = 1.0f;
      if (amax > 16384.f) {                        // exponent of amax / 16384, rounded up
        const int e = (int)((__float_as_uint(amax) >> 23) & 0xff) - 127 - 13;
        cscale = __uint_as_float((unsigned int)(127 + e) << 23);
        inv_c = __uint_as_float((unsigned int)(127 - e) << 23);
      }
      u32x4 *po = reinterpret_cast<u32x4 *>(a.part_o) + (unit * 4 + w) * (4 * 64) + lane;
#pragma unroll
      for (int pr = 0; pr < 4; ++pr) {
        const f32x4 x = o_acc[qt][2 * pr] * inv_c, y = o_acc[qt][2 * pr + 1] * inv_c;
        __builtin_nontemporal_store((u32x4){pack_f16x2(x[0], x[1]), pack_f16x2(x[2], x[3]),
                                            pack_f16x2(y[0], y[1]), pack_f16x2(y[2], y[3])}, &po[pr * 64]);
      }
      if (c4 == 0) {
        float *pml = a.part_ml + (unit * kRowsPerWG + 16 * w + n) * kMlFloats;
        __builtin_nontemporal_store(m_new, &pml[0]);
        __builtin_nontemporal_store(l_tot, &pml[1]);
        __builtin_nontemporal_store(cscale, &pml[2]);
      }
    }
  }
}

// Combine for the tiled partial layout above.  One workgroup of 16 wavefronts per (sequence, KV
// head, 16-row tile, 16-wide d tile); wavefront ws merges splits ws, ws+16, ... with 4 splits (8
// bytes per lane each) in flight at a time, so the usual 64 splits cost one memory round trip; the
// running results are merged through LDS.  The pass is bound by its dependent chain (launch, one
// load round trip, the exponentials, the LDS merge, the store), not by bytes: measured per C5 layer
// with 4 wavefronts x 16 splits and two d-tiles per workgroup 20.6 us, one d-tile 19.0 us, 8 x 8
// 18.7 us, 16 x 4 18.5 us.
constexpr int kCombInFlight = 4;

// kCombWaves = 16 for the decode-time case (one sequence cut into ~64 splits); 8 or 4 when no
// sequence of the call has more than 32 or 16 splits (draft trees, batches), where 16 wavefronts
// per output tile would mostly find nothing to merge.
template <int kCombWaves>
__global__ void __launch_bounds__(64 * kCombWaves)
verify_combine_tiled_kernel(VerifyArgs a, SeqTable tab, int rbs, int g) {
  __shared__ f32x4 xo[kCombWaves][64];
  __shared__ float xm[kCombWaves][64], xl[kCombWaves][64];
  const int b = blockIdx.z;
  const int s0 = tab.cu_split[b], s1 = tab.cu_split[b + 1];
  // all scalar arguments in one round of loads (see the partial pass)
  asm volatile("" ::"s"(rbs), "s"(g), "s"(s0), "s"(s1), "s"(a.n_q), "s"(a.Hq), "s"(a.Hkv), "s"(a.part_o),
               "s"(a.part_ml), "s"(a.out), "s"(a.lse));
  const int unit_in_seq = blockIdx.x;            // (c * rbs + rb) * 4 + wq
  const int wq = unit_in_seq & 3, crb = unit_in_seq >> 2;
  int rb = 0, c = crb;
  if (rbs > 1) { rb = crb % rbs; c = crb / rbs; }
  const int mt = blockIdx.y;                     // d-tile: half (mt & 1) of the stored pair mt >> 1
  const int ws = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int n = lane & 15, c4 = lane >> 4;
  const int R = a.n_q * g;
  if (rb * kRowsPerWG + 16 * wq >= R) return;    // tile without rows (uniform)
  const u32x2 *po = reinterpret_cast<const u32x2 *>(a.part_o);
  float m_run = kNegBig, l_run = 0.f;
  f32x4 o = {0.f, 0.f, 0.f, 0.f};
  for (int sb = s0 + ws; sb < s1; sb += kCombWaves * kCombInFlight) {
    float ms[kCombInFlight], ls[kCombInFlight], cs[kCombInFlight];
    u32x2 pa[kCombInFlight];
#pragma unroll
    for (int u = 0; u < kCombInFlight; ++u) {
      const int s = min(sb + kCombWaves * u, s1 - 1);
      const int64_t unit = ((int64_t)s * a.Hkv + c) * rbs + rb;
      const float *pml = a.part_ml + (unit * kRowsPerWG + 16 * wq + n) * kMlFloats;
      ms[u] = __builtin_nontemporal_load(&pml[0]);
      ls[u] = __builtin_nontemporal_load(&pml[1]);
      cs[u] = __builtin_nontemporal_load(&pml[2]);
      pa[u] = __builtin_nontemporal_load(&po[((((unit * 4 + wq) * 4 + (mt >> 1)) * 64 + lane) << 1) + (mt & 1)]);
    }
    float mx = m_run;
#pragma unroll
    for (int u = 0; u < kCombInFlight; ++u) if (sb + kCombWaves * u < s1) mx = fmaxf(mx, ms[u]);
    const float alpha = fast_exp2(m_run - mx);
    m_run = mx;
    l_run *= alpha; o *= alpha;
#pragma unroll
    for (int u = 0; u < kCombInFlight; ++u) {
      // weight of the split: its share of the softmax denominator (its output is normalised)
      const float wgt = (sb + kCombWaves * u < s1) ? fast_exp2(ms[u] - mx) * ls[u] : 0.f;
      l_run += wgt;
      o += unpack_f16x4(pa[u].x, pa[u].y) * (wgt * cs[u]);
    }
  }
  xo[ws][lane] = o;
  xm[ws][lane] = m_run; xl[ws][lane] = l_run;
  __syncthreads();
  if (ws == 0) {
    float m = xm[0][lane];
#pragma unroll
    for (int k = 1; k < kCombWaves; ++k) m = fmaxf(m, xm[k][lane]);
    float l = 0.f;
    f32x4 r = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int k = 0; k < kCombWaves; ++k) {
      const float wgt = fast_exp2(xm[k][lane] - m);
      l = fmaf(xl[k][lane], wgt, l);
      r += xo[k][lane] * wgt;
    }
    const int rho = rb * kRowsPerWG + 16 * wq + n;
    if (rho < R) {
      const int i_row = rho / g, h = c * g + rho % g;
      const int64_t orow = ((int64_t)b * a.n_q + i_row) * a.Hq + h;
      const float inv = 1.0f / l;
      bf16_t *out = (bf16_t *)a.out + orow * 128 + 16 * mt + 4 * c4;
      u32x2 w0 = {pack_bf16x2(r[0] * inv, r[1] * inv), pack_bf16x2(r[2] * inv, r[3] * inv)};
      *reinterpret_cast<u32x2 *>(out) = w0;
      if (a.lse != nullptr && mt == 0 && c4 == 0) a.lse[orow] = (m + fast_log2(l)) * kLn2;
    }
  }
}

}  // namespace

bool verify_partial_mfma_supported(int dtype, int head_dim) {
  return dtype == SPARROW_BF16 && head_dim == 128;
}

// Floats of workspace per (split, KV head, row block) unit of the tiled partial layout.
int64_t verify_mfma_unit_floats_o() { return 4 * 4 * 64 * 4; }   // 16 KB: 64 rows x 128 halves
int64_t verify_mfma_unit_floats_ml() { return kRowsPerWG * kMlFloats; }

// Row blocks (workgroups per split and KV head) for R rows: blocks of three 64-row tiles unless
// blocks of two leave fewer empty tiles (7 tiles: 2+2+2+1 beats 3+3+1, measured).
int verify_mfma_row_blocks(int R) {
  const int tiles = (R + kRowsPerWG - 1) / kRowsPerWG;
  const int rbs3 = (tiles + 2) / 3, rbs2 = (tiles + 1) / 2;
  return rbs3 * 3 - tiles <= rbs2 * 2 - tiles ? rbs3 : rbs2;
}

hipError_t launch_verify_partial_mfma(const VerifyArgs &a, const SeqTable &tab, hipStream_t st) {
  const int R = a.n_q * (a.Hq / a.Hkv);
  const int rbs = verify_mfma_row_blocks(R);
  PieceTable pt;
  int max_ns = 0;
  for (int b = 0; b < SPARROW_MAX_BATCH; ++b) {
    const int ns = b < a.B ? tab.cu_split[b + 1] - tab.cu_split[b] : 0;
    pt.piece[b] = ns > 0 ? split_len(tab.cu_len[b + 1] - tab.cu_len[b], ns) : 0;
    if (ns > max_ns) max_ns = ns;
  }
  // grid shape: one x range per (KV head, sequence) unless that would launch mostly padding
  const int x3d = (max_ns + 7) / 8 * 8;
  const int flat = (int64_t)a.n_slots * 4 < (int64_t)x3d * a.B * 3;      // fewer than 3/4 of the slots real
  dim3 grid(x3d * rbs, a.Hkv, a.B), block(256 * kStreams);
  if (flat) grid = dim3((a.n_slots * a.Hkv + 7) / 8 * 8 * rbs, 1, 1);
  constexpr int kLdsBytes = kStreams * 2 * 2 * kSub * kTileBytes;
  static_assert(kLdsBytes <= 64 * 1024, "beyond 64 KB the kernel needs the dynamic-LDS attribute");
  const int steps = (a.chunk / kTile + kStreams * kSub - 1) / (kStreams * kSub);   // of a full split
  const int tiles = (R + kRowsPerWG - 1) / kRowsPerWG;
  const int qt = (tiles + rbs - 1) / rbs;
  if (qt == 3)      // a second tile in flight does not fit the registers (and the step is compute-bound)
    hipLaunchKernelGGL((verify_partial_mfma_kernel<1, 3>), grid, block, kLdsBytes, st, a, tab, pt, rbs, flat);
  else if (qt == 2 && steps <= 10)
    hipLaunchKernelGGL((verify_partial_mfma_kernel<1, 2>), grid, block, kLdsBytes, st, a, tab, pt, rbs, flat);
  else if (qt == 2)
    hipLaunchKernelGGL((verify_partial_mfma_kernel<2, 2>), grid, block, kLdsBytes, st, a, tab, pt, rbs, flat);
  else if (steps <= 3)       // (a second step in flight pays from 4 steps on: -0.15 us at the 7 steps of a 26k chain)
    hipLaunchKernelGGL((verify_partial_mfma_kernel<1, 1>), grid, block, kLdsBytes, st, a, tab, pt, rbs, flat);
  else
    hipLaunchKernelGGL((verify_partial_mfma_kernel<2, 1>), grid, block, kLdsBytes, st, a, tab, pt, rbs, flat);
  return hipGetLastError();
}

hipError_t launch_verify_combine_mfma(const VerifyArgs &a, const SeqTable &tab, hipStream_t st) {
  const int R = a.n_q * (a.Hq / a.Hkv);
  const int rbs = (R + kRowsPerWG - 1) / kRowsPerWG;
  dim3 grid(a.Hkv * rbs * 4, 8, a.B);
  int max_ns = 0;
  for (int b = 0; b < a.B; ++b) max_ns = std::max(max_ns, tab.cu_split[b + 1] - tab.cu_split[b]);
  if (max_ns > 32)
    hipLaunchKernelGGL(verify_combine_tiled_kernel<16>, grid, dim3(64 * 16), 0, st, a, tab, rbs, a.Hq / a.Hkv);
  else if (max_ns > 16)
    hipLaunchKernelGGL(verify_combine_tiled_kernel<8>, grid, dim3(64 * 8), 0, st, a, tab, rbs, a.Hq / a.Hkv);
  else
    hipLaunchKernelGGL(verify_combine_tiled_kernel<4>, grid, dim3(64 * 4), 0, st, a, tab, rbs, a.Hq / a.Hkv);
  return hipGetLastError();
}

}  // namespace sparrow
