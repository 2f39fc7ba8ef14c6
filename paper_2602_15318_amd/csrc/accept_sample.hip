// Stochastic (temperature > 0) tree acceptance on the logits stored by the lm_head pass.
//
//   logit_stats_kernel   the whole chip reads the M x V logits once (grid M x 64 chunks): per
//                        chunk the max and the sum of exponentials of logits / T, and per block of
//                        256 tokens the sum of exponentials relative to the chunk's max;
//   accept_sample_kernel one workgroup per sequence walks the tree: at the current node it merges
//                        the row's 64 chunk statistics, evaluates the children's probabilities
//                        in parallel, lets one thread apply the sequential rejection rule
//                        (u * S <= p[x] accepts; a rejected token is struck out and its mass leaves
//                        S), and, when no child is accepted, draws the bonus token from what is
//                        left by inverse CDF in vocabulary order: a scan over the row's block
//                        sums (struck-out tokens taken out), then a search inside the one block
//                        that holds the target -- the only 256 logits of the row it reads.
// Exponentials are exp2 of logits pre-multiplied by log2(e) / T in fp32; sums across blocks fp64.
#include "accept.hpp"
#include "common.hpp"

namespace sparrow {

namespace {

constexpr int kStatThreads = 256;
constexpr int kWalkThreads = 1024;
constexpr int kBonusBlock = 256;              // tokens per block of the bonus draw
constexpr int kBonusMaxBlocks = kSampleMaxVocab / kBonusBlock;

// Philox4x32 with 10 rounds (Salmon et al., SC'11): round (c0, c1, c2, c3), key (k0, k1) ->
// (hi(M1 c2) ^ c1 ^ k0, lo(M1 c2), hi(M0 c0) ^ c3 ^ k1, lo(M0 c0)); the key grows by the Weyl
// constants after every round.  Only the first output word is used here.
__device__ __forceinline__ unsigned int philox4x32_10_word0(unsigned int c0, unsigned int c1,
                                                            unsigned int c2, unsigned int c3,
                                                            unsigned int k0, unsigned int k1) {
#pragma unroll
  for (int round = 0; round < 10; ++round) {
    const unsigned int h0 = __umulhi(0xD2511F53u, c0), l0 = 0xD2511F53u * c0;
    const unsigned int h1 = __umulhi(0xCD9E8D57u, c2), l1 = 0xCD9E8D57u * c2;
    const unsigned int n0 = h1 ^ c1 ^ k0, n2 = h0 ^ c3 ^ k1;
    c0 = n0; c1 = l1; c2 = n2; c3 = l0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return c0;
}
// The uniform that decides node j of sequence b (j = -1: the bonus draw): the caller's, or the
// top 24 bits of the Philox block (offset, b, j) under the key `seed`, times 2^-24.
__device__ __forceinline__ float uniform_of(const SampleArgs &a, int b, int j) {
  if (j >= 0 && a.u_accept != nullptr) return a.u_accept[(int64_t)b * a.n_q + j];
  if (j < 0 && a.u_bonus != nullptr) return a.u_bonus[b];
  const unsigned int w = philox4x32_10_word0((unsigned int)a.offset, (unsigned int)(a.offset >> 32),
                                             (unsigned int)b, j >= 0 ? (unsigned int)j : 0xFFFFFFFFu,
                                             (unsigned int)a.seed, (unsigned int)(a.seed >> 32));
  return (float)(w >> 8) * (1.0f / 16777216.0f);
}

// A wavefront owns whole blocks of 256 tokens (blocks b0 + w, b0 + w + 4, ... of the chunk), a lane
// four consecutive tokens of each: the chunk is read once, 16 bytes per lane, and stays in
// registers for the maximum and for the sums.
constexpr int kStatBlocksPerWave = kBonusMaxBlocks / kStatChunks / (kStatThreads / 64);   // 16

__global__ void __launch_bounds__(kStatThreads)
logit_stats_kernel(SampleArgs a) {
  __shared__ float red[kStatThreads / 64];
  constexpr int kWaves = kStatThreads / 64;
  const int c = blockIdx.x, r = blockIdx.y;
  const int n_blk = (a.V + kBonusBlock - 1) / kBonusBlock;
  const int bpc = (n_blk + kStatChunks - 1) / kStatChunks;          // blocks per chunk
  const int b0 = min(n_blk, c * bpc), b1 = min(n_blk, b0 + bpc);
  const float *lg = a.logits + (int64_t)r * a.V;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  // scaled logits of this lane: x[k][i] = token (b0 + w + 4 k) * 256 + 4 lane + i, kNegBig past V
  float x[kStatBlocksPerWave][4];
  const bool row_aligned = (((int64_t)r * a.V) & 3) == 0;           // 16-byte loads possible
#pragma unroll
  for (int k = 0; k < kStatBlocksPerWave; ++k) {
    const int ib = b0 + w + kWaves * k;
    const int v = ib * kBonusBlock + 4 * lane;
#pragma unroll
    for (int i = 0; i < 4; ++i) x[k][i] = kNegBig;
    if (ib < b1) {
      if (row_aligned && v + 3 < a.V) {
        const f32x4 q = *reinterpret_cast<const f32x4 *>(lg + v);
#pragma unroll
        for (int i = 0; i < 4; ++i) x[k][i] = q[i] * a.inv_temp_log2;
      } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (v + i < a.V) x[k][i] = lg[v + i] * a.inv_temp_log2;
      }
    }
  }
  float m = kNegBig;
#pragma unroll
  for (int k = 0; k < kStatBlocksPerWave; ++k)
#pragma unroll
    for (int i = 0; i < 4; ++i) m = fmaxf(m, x[k][i]);
  m = wave_max_valu(m);
  if (lane == 0) red[w] = m;
  __syncthreads();
  m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  __syncthreads();
  // block sums relative to the chunk's max
  float s = 0.f;
#pragma unroll
  for (int k = 0; k < kStatBlocksPerWave; ++k) {
    const int ib = b0 + w + kWaves * k;
    if (ib < b1) {                              // uniform over the wavefront
      const int v = ib * kBonusBlock + 4 * lane;
      float t = 0.f;
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (v + i < a.V) t += fast_exp2(x[k][i] - m);
      t = wave_sum_valu(t);
      if (lane == 0) a.blk_sum[(int64_t)r * n_blk + ib] = t;
      s += t;                                   // the same value in every lane
    }
  }
  if (lane == 0) red[w] = s;
  __syncthreads();
  if (threadIdx.x == 0) {
    float *o = a.stats + ((int64_t)r * kStatChunks + c) * 2;
    o[0] = m;                                   // kNegBig and sum 0 for an empty chunk
    o[1] = red[0] + red[1] + red[2] + red[3];
  }
}

__global__ void __launch_bounds__(kWalkThreads)
accept_sample_kernel(SampleArgs a) {
  __shared__ float cand_p[SPARROW_MAX_NQ];      // probability of child j's token, -1 if not a child
  __shared__ float cand_u[SPARROW_MAX_NQ];      // the uniform that decides child j
  __shared__ int struck[SPARROW_MAX_NQ];        // tokens rejected at the current node
  __shared__ int sh_next, sh_nstruck;
  __shared__ float sh_S, sh_m, sh_Z;
  __shared__ double wave_tot[kWalkThreads / 64];
  __shared__ int sh_owner, sh_last, sh_pick, sh_blk;
  __shared__ double sh_excl;
  __shared__ double blk_tot[kBonusMaxBlocks];   // sum of the live exponentials of 256 tokens
  __shared__ float chunk_m[kStatChunks];        // max of every chunk of the current row
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int n_q = a.n_q, V = a.V;
  const int32_t *dr = a.draft_ids + (int64_t)b * n_q;
  int32_t *path = a.accept_path + (int64_t)b * n_q;
  for (int i = tid; i < n_q; i += kWalkThreads) path[i] = -1;
  int cur = -1, len = 0;
  // at most n_q + 1 levels: cur strictly increases along a path
  for (int level = 0; level <= n_q; ++level) {
    const int64_t row = (int64_t)b * (n_q + 1) + cur + 1;
    const float *lg = a.logits + row * V;
    // ---- row statistics from the 64 chunk partials (wavefront 0)
    if (w == 0) {
      const float pm = a.stats[(row * kStatChunks + lane) * 2];
      const float ps = a.stats[(row * kStatChunks + lane) * 2 + 1];
      const float m = wave_max(pm);
      const float Z = wave_sum(ps * fast_exp2(pm - m));
      chunk_m[lane] = pm;
      if (lane == 0) { sh_m = m; sh_Z = Z; }
    }
    __syncthreads();
    const float m = sh_m, Z = sh_Z;
    // ---- children of cur and the probabilities of their tokens
    if (tid < n_q) {
      const int pj = a.parent ? a.parent[(int64_t)b * a.parent_stride + tid] : tid - 1;
      const int x = dr[tid];
      float p = -1.f;
      if (pj == cur && x >= 0 && x < V) p = fast_exp2(lg[x] * a.inv_temp_log2 - m) / Z;
      cand_p[tid] = p;
      cand_u[tid] = uniform_of(a, b, tid);
    }
    __syncthreads();
    if (tid == 0) {
      float S = 1.f;
      int next = -1, ns = 0;
      for (int j = 0; j < n_q && next < 0; ++j) {
        const float p = cand_p[j];
        if (p < 0.f) continue;
        const int x = dr[j];
        bool gone = false;
        for (int k = 0; k < ns; ++k) gone |= struck[k] == x;
        if (gone || p == 0.f) continue;
        if (cand_u[j] * S <= p) next = j;
        else { S -= p; struck[ns++] = x; }
      }
      sh_next = next; sh_S = S; sh_nstruck = ns;
      sh_owner = kWalkThreads; sh_last = -1; sh_pick = -1;
    }
    __syncthreads();
    const int next = sh_next;
    if (next >= 0) {
      if (tid == 0) path[len] = next;
      ++len;
      cur = next;
      __syncthreads();          // cand_p / struck are rewritten at the next level
      continue;
    }
    // ---- bonus token: inverse CDF over what is left of the row's distribution.  The sums of
    // the row's 256-token blocks come from the statistics pass (relative to their chunk's max);
    // rescaled to the row's max, minus the struck-out tokens, they are scanned in fp64 (fp32
    // inside a block, whose sum is a small part of the mass), so the draw is decided by the fp32
    // exponentials alone (~1e-7 of the remaining mass).  Only the block that holds the target
    // is read from the logits.
    const int ns = sh_nstruck;
    const double target = (double)uniform_of(a, b, -1) * (double)sh_S * (double)Z;   // unnormalised units
    auto weight = [&](int v) {
      bool gone = false;
      for (int k = 0; k < ns; ++k) gone |= struck[k] == v;
      return gone ? 0.f : fast_exp2(lg[v] * a.inv_temp_log2 - m);
    };
    // the 4 weights of this lane in block ib (0 past the end of the vocabulary)
    auto lane_weights = [&](int ib, float *e) {
      const int v = ib * kBonusBlock + 4 * lane;
#pragma unroll
      for (int i = 0; i < 4; ++i) e[i] = (v + i < V) ? weight(v + i) : 0.f;
    };
    const int n_blk = (V + kBonusBlock - 1) / kBonusBlock;
    const int bpc = (n_blk + kStatChunks - 1) / kStatChunks;
    const float *bs = a.blk_sum + row * n_blk;
    for (int ib = tid; ib < n_blk; ib += kWalkThreads)
      blk_tot[ib] = (double)bs[ib] * (double)fast_exp2(chunk_m[ib / bpc] - m);
    __syncthreads();
    if (tid == 0) {                  // struck-out tokens leave their blocks
      for (int k = 0; k < ns; ++k) {
        const int x = struck[k];
        const double left = blk_tot[x / kBonusBlock] - (double)fast_exp2(lg[x] * a.inv_temp_log2 - m);
        blk_tot[x / kBonusBlock] = left > 0.0 ? left : 0.0;
      }
    }
    __syncthreads();
    // scan over the block sums: thread t owns blocks [t*bp, (t+1)*bp)
    const int bp = (n_blk + kWalkThreads - 1) / kWalkThreads;
    double local = 0.0;
    int last_blk = -1;
    for (int i = 0; i < bp; ++i) {
      const int ib = tid * bp + i;
      if (ib < n_blk) {
        local += blk_tot[ib];
        if (blk_tot[ib] > 0.0) last_blk = ib;
      }
    }
    if (last_blk >= 0) atomicMax(&sh_last, last_blk);      // last live block of the row
    double incl = local;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const double up = __shfl_up(incl, o, 64);
      if (lane >= o) incl += up;
    }
    if (lane == 63) wave_tot[w] = incl;
    __syncthreads();
    double base = 0.0;
    for (int k = 0; k < w; ++k) base += wave_tot[k];
    incl += base;
    if (local > 0.0 && incl >= target) atomicMin(&sh_owner, tid);
    __syncthreads();
    if (tid == sh_owner) {           // which of this thread's blocks holds the target
      double run = incl - local;
      int blk = -1;
      for (int i = 0; i < bp && blk < 0; ++i) {
        const int ib = tid * bp + i;
        if (ib < n_blk && blk_tot[ib] > 0.0) {
          if (run + blk_tot[ib] >= target) blk = ib; else run += blk_tot[ib];
        }
      }
      if (blk < 0) {                 // rounding between the two summation orders: last live block
        for (int i = bp - 1; i >= 0 && blk < 0; --i) {
          const int ib = tid * bp + i;
          if (ib < n_blk && blk_tot[ib] > 0.0) blk = ib;
        }
        run = -1.0e300;              // nothing in blk reaches the target: its last live token
      }
      sh_blk = blk;
      sh_excl = run;
    }
    __syncthreads();
    if (w == 0 && (sh_owner < kWalkThreads || sh_last >= 0)) {
      // the block that holds the target; if rounding left the row's total a hair below the
      // target, the last live block with nothing to find: its last live token is taken
      const bool owned = sh_owner < kWalkThreads;
      const int ib = owned ? sh_blk : sh_last;
      const double excl0 = owned ? sh_excl : -1.0e300;
      float e[4];
      lane_weights(ib, e);
      const float mine = (e[0] + e[1]) + (e[2] + e[3]);
      float li = mine;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const float up = __shfl_up(li, o, 64);
        if (lane >= o) li += up;
      }
      double run = excl0 + (double)(li - mine);
      int found = -1, lastp = -1;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if (e[i] > 0.f) {
          lastp = ib * kBonusBlock + 4 * lane + i;
          run += (double)e[i];
          if (found < 0 && run >= target) found = lastp;
        }
      }
      // first lane that found its element wins (vocabulary order = lane order)
      const unsigned long long hit = __builtin_amdgcn_ballot_w64(found >= 0);
      int pick;
      if (hit != 0ull) {
        pick = __shfl(found, __builtin_ctzll(hit), 64);
      } else {                       // a hair below the target after rounding: last live token
        pick = lastp;
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) pick = max(pick, __shfl_xor(pick, o, 64));
      }
      if (lane == 0) sh_pick = pick;
    }
    __syncthreads();
    if (tid == 0) {
      a.bonus_id[b] = max(sh_pick, 0);
      a.accept_len[b] = len;
    }
    return;
  }
  // only reachable with a malformed tree (the walk did not end within n_q + 1 levels)
  if (tid == 0) { a.accept_len[b] = len; a.bonus_id[b] = 0; }
}

// Acceptance against a SAMPLED draft: the children of a node were drawn from the draft's
// distribution q (row of draft_q), and child j with token x is accepted with probability
// min(1, (R[x] / S) / q[x]), where R is the residual of the target's p after the rejections so far
// at this node (R <- max(R - S q, 0) on every rejection, S its sum); the bonus token comes from R.
// One workgroup per sequence.  R is never stored: a token's residual after k rejections follows
// from its p, its q and the k sums S_0 .. S_{k-1}, so a rejection costs one pass over the row
// (logits and q) for the next sum, which also leaves the sums per block of 256 tokens in LDS for
// the bonus draw: scan over the blocks, then a search inside the block that holds the target.
constexpr int kMaxRejections = SPARROW_MAX_NQ;

__global__ void __launch_bounds__(kWalkThreads)
accept_sample_q_kernel(SampleArgs a) {
  __shared__ int dr_s[SPARROW_MAX_NQ], par_s[SPARROW_MAX_NQ];
  __shared__ float S_s[kMaxRejections + 1];     // residual sums at the current node
  __shared__ double blk_tot[kBonusMaxBlocks];   // sums of the current residual per 256 tokens
  __shared__ double wave_tot[kWalkThreads / 64];
  __shared__ float sh_m;
  __shared__ int sh_owner, sh_last, sh_pick, sh_blk;
  __shared__ double sh_excl;
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int n_q = a.n_q, V = a.V;
  int32_t *path = a.accept_path + (int64_t)b * n_q;
  for (int i = tid; i < n_q; i += kWalkThreads) {
    path[i] = -1;
    dr_s[i] = a.draft_ids[(int64_t)b * n_q + i];
    par_s[i] = a.parent ? a.parent[(int64_t)b * a.parent_stride + i] : i - 1;
  }
  __syncthreads();
  const int n_blk = (V + kBonusBlock - 1) / kBonusBlock;
  int cur = -1, len = 0;
  for (int level = 0; level <= n_q; ++level) {
    const int64_t row = (int64_t)b * (n_q + 1) + cur + 1;
    const float *lg = a.logits + row * V;
    const float *q = a.draft_q + row * V;
    const bool aligned = ((row * V) & 3) == 0;                // 16-byte loads possible on this row
    if (w == 0) {                                             // row maximum and sum from the chunk partials
      const float pm = a.stats[(row * kStatChunks + lane) * 2];
      const float ps = a.stats[(row * kStatChunks + lane) * 2 + 1];
      const float m = wave_max(pm);
      const float Z = wave_sum(ps * fast_exp2(pm - m));
      if (lane == 0) { sh_m = m; S_s[0] = Z; }
    }
    __syncthreads();
    const float m = sh_m;
    int k = 0;                                                // rejections at this node so far
    // residual of token v after k rejections (unnormalised: p = exp2(..) / S_0)
    auto residual = [&](float lv, float qv, int kk) {
      float r = fast_exp2(lv * a.inv_temp_log2 - m);
      for (int i = 0; i < kk; ++i) r = fmaxf(r - S_s[i] * qv, 0.f);
      return r;
    };
    // one pass over the row: sums of the residual after kk rejections per block of 256 tokens
    // (into blk_tot) and in total (returned to every thread)
    auto block_sums = [&](int kk) {
      double mine = 0.0;
      for (int ib = w; ib < n_blk; ib += kWalkThreads / 64) {
        const int v = ib * kBonusBlock + 4 * lane;
        float lv[4], qv[4];
        if (aligned && v + 3 < V) {
          const f32x4 l4 = *reinterpret_cast<const f32x4 *>(lg + v);
          const f32x4 q4 = *reinterpret_cast<const f32x4 *>(q + v);
#pragma unroll
          for (int i = 0; i < 4; ++i) { lv[i] = l4[i]; qv[i] = q4[i]; }
        } else {
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            lv[i] = v + i < V ? lg[v + i] : 0.f;
            qv[i] = v + i < V ? q[v + i] : 0.f;
          }
        }
        float t = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (v + i < V) t += residual(lv[i], qv[i], kk);
        t = wave_sum_valu(t);
        if (lane == 0) blk_tot[ib] = (double)t;
        mine += (double)t;                                    // the same value in every lane
      }
      if (lane == 0) wave_tot[w] = mine;
      __syncthreads();
      double tot = 0.0;
      for (int i = 0; i < kWalkThreads / 64; ++i) tot += wave_tot[i];
      __syncthreads();                                        // wave_tot is reused by the scan
      return tot;
    };
    int next = -1;
    bool sums_current = false;                                // blk_tot holds the sums of residual k
    for (int j = cur + 1; j < n_q && next < 0; ++j) {         // uniform: par_s / dr_s are shared
      if (par_s[j] != cur) continue;
      const int x = dr_s[j];
      if (x < 0 || x >= V) continue;
      const float qx = q[x];
      const float r = residual(lg[x], qx, k);
      if (r > 0.f && uniform_of(a, b, j) * qx * S_s[k] <= r) { next = j; break; }
      if (k == kMaxRejections) continue;                      // (cannot happen: at most n_q children)
      const double tot = block_sums(k + 1);                   // rejected: the next residual's sum
      if (tid == 0) S_s[k + 1] = (float)tot;
      __syncthreads();
      ++k;
      sums_current = true;
    }
    if (next >= 0) {
      if (tid == 0) path[len] = next;
      ++len;
      cur = next;
      __syncthreads();                                        // S_s is rewritten at the next level
      continue;
    }
    // ---- bonus token: inverse CDF of the residual after k rejections, in vocabulary order
    if (!sums_current) (void)block_sums(k);
    if (tid == 0) { sh_owner = kWalkThreads; sh_last = -1; sh_pick = -1; }
    __syncthreads();
    const double target = (double)uniform_of(a, b, -1) * (double)S_s[k];
    const int bp = (n_blk + kWalkThreads - 1) / kWalkThreads;
    double local = 0.0;
    int last_blk = -1;
    for (int i = 0; i < bp; ++i) {
      const int ib = tid * bp + i;
      if (ib < n_blk) {
        local += blk_tot[ib];
        if (blk_tot[ib] > 0.0) last_blk = ib;
      }
    }
    if (last_blk >= 0) atomicMax(&sh_last, last_blk);
    double incl = local;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const double up = __shfl_up(incl, o, 64);
      if (lane >= o) incl += up;
    }
    if (lane == 63) wave_tot[w] = incl;
    __syncthreads();
    double base = 0.0;
    for (int i = 0; i < w; ++i) base += wave_tot[i];
    incl += base;
    if (local > 0.0 && incl >= target) atomicMin(&sh_owner, tid);
    __syncthreads();
    if (tid == sh_owner) {                                    // which of this thread's blocks
      double run = incl - local;
      int blk = -1;
      for (int i = 0; i < bp && blk < 0; ++i) {
        const int ib = tid * bp + i;
        if (ib < n_blk && blk_tot[ib] > 0.0) {
          if (run + blk_tot[ib] >= target) blk = ib; else run += blk_tot[ib];
        }
      }
      if (blk < 0) {                                          // rounding between the two orders of summation
        for (int i = bp - 1; i >= 0 && blk < 0; --i) {
          const int ib = tid * bp + i;
          if (ib < n_blk && blk_tot[ib] > 0.0) blk = ib;
        }
        run = -1.0e300;
      }
      sh_blk = blk;
      sh_excl = run;
    }
    __syncthreads();
    if (w == 0 && (sh_owner < kWalkThreads || sh_last >= 0)) {
      const bool owned = sh_owner < kWalkThreads;
      const int ib = owned ? sh_blk : sh_last;
      const double excl0 = owned ? sh_excl : -1.0e300;
      float e[4];
      const int v = ib * kBonusBlock + 4 * lane;
#pragma unroll
      for (int i = 0; i < 4; ++i) e[i] = v + i < V ? residual(lg[v + i], q[v + i], k) : 0.f;
      const float mine = (e[0] + e[1]) + (e[2] + e[3]);
      float li = mine;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const float up = __shfl_up(li, o, 64);
        if (lane >= o) li += up;
      }
      double run = excl0 + (double)(li - mine);
      int found = -1, lastp = -1;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if (e[i] > 0.f) {
          lastp = v + i;
          run += (double)e[i];
          if (found < 0 && run >= target) found = lastp;
        }
      }
      const unsigned long long hit = __builtin_amdgcn_ballot_w64(found >= 0);
      int pick;
      if (hit != 0ull) {
        pick = __shfl(found, __builtin_ctzll(hit), 64);
      } else {                                                // a hair below the target: last live token
        pick = lastp;
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) pick = max(pick, __shfl_xor(pick, o, 64));
      }
      if (lane == 0) sh_pick = pick;
    }
    __syncthreads();
    if (tid == 0) {
      a.bonus_id[b] = max(sh_pick, 0);
      a.accept_len[b] = len;
    }
    return;
  }
  if (tid == 0) { a.accept_len[b] = len; a.bonus_id[b] = 0; }   // malformed tree only
}

}  // namespace

hipError_t launch_logit_stats(const SampleArgs &a, hipStream_t st) {
  hipLaunchKernelGGL(logit_stats_kernel, dim3(kStatChunks, a.M), dim3(kStatThreads), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_accept_sample(const SampleArgs &a, hipStream_t st) {
  if (a.draft_q != nullptr)
    hipLaunchKernelGGL(accept_sample_q_kernel, dim3(a.B), dim3(kWalkThreads), 0, st, a);
  else
    hipLaunchKernelGGL(accept_sample_kernel, dim3(a.B), dim3(kWalkThreads), 0, st, a);
  return hipGetLastError();
}

}  // namespace sparrow
