// Internal interface of the acceptance kernels (lm_head GEMM + argmax + greedy walk).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/sparrow.h"

namespace sparrow {

constexpr int kAcceptMaxRows = SPARROW_MAX_ACCEPT_ROWS;

struct AcceptArgs {
  const void *hidden;        // [M, H]
  const void *lm_head;       // [V, H]
  const int32_t *draft_ids;  // [B*n_q]
  const int32_t *parent;     // [n_q] (parent_stride 0) or [B, parent_stride], or nullptr
  int32_t parent_stride;
  int32_t B, n_q, M, H, V;   // M = B*(n_q+1)
  int32_t n_cand;            // argmax candidates per row produced by the GEMM pass
  float *cand_val;           // [M, n_cand]
  int32_t *cand_idx;         // [M, n_cand]
  int32_t *target_ids, *accept_len, *accept_path, *bonus_id;
  float *logits;             // [M, V] or nullptr: the GEMM pass also stores every logit (sampling)
};

// Stochastic acceptance (temperature > 0) on stored logits.
constexpr int kStatChunks = 64;   // partial (max, sum of exponentials) per row
constexpr int kSampleMaxVocab = 1 << 20;   // the bonus draw keeps one fp64 sum per 256 tokens in LDS
struct SampleArgs {
  const float *logits;       // [M, V]
  const int32_t *draft_ids;  // [B*n_q]
  const int32_t *parent;     // [n_q] (parent_stride 0) or [B, parent_stride], or nullptr
  int32_t parent_stride;
  const float *u_accept;     // [B, n_q], or nullptr: generated from (seed, offset)
  const float *u_bonus;      // [B], or nullptr
  const float *draft_q;      // [M, V] draft distribution of every row's children, or nullptr
  uint64_t seed, offset;     // key and counter prefix of the generated uniforms
  float *stats;              // [M, kStatChunks, 2]: max and sum of exponentials per chunk
  float *blk_sum;            // [M, ceil(V / 256)]: sum of exponentials per block, relative to the
                             // max of the block's chunk (chunk = ceil(blocks / 64) blocks)
  int32_t *accept_len, *accept_path, *bonus_id;
  int32_t B, n_q, M, V;
  float inv_temp_log2;       // log2(e) / temperature
};
hipError_t launch_logit_stats(const SampleArgs &a, hipStream_t st);
hipError_t launch_accept_sample(const SampleArgs &a, hipStream_t st);

// Number of per-row argmax candidates the GEMM pass writes (one per wavefront / tile owner).
int accept_num_candidates(int dtype, int M, int H, int V);
bool lm_head_mfma_supported(int dtype, int M, int H, int V);
hipError_t launch_lm_head_generic(int dtype, const AcceptArgs &a, hipStream_t st);
hipError_t launch_lm_head_mfma(const AcceptArgs &a, hipStream_t st);
hipError_t launch_accept_finalize(const AcceptArgs &a, hipStream_t st);

}  // namespace sparrow
