// Internal interface of the dynamic draft-tree kernels: top-k log-probabilities of the draft's
// lm_head rows, level expansion of the candidate pool, final selection.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/sparrow.h"
#include "accept.hpp"

namespace sparrow {

constexpr int kTreeMaxWidth = 16;       // candidates per node and nodes per frontier
constexpr int kTreeMaxPool = 2048;      // width + (depth - 1) * width^2 must fit

struct TopkArgs {
  const float *logits;      // [M, V]
  float *stats;             // [M, kStatChunks, 2] (max, sum of exp2) in the log2 domain, T = 1:
                            // written by the chunk kernel, read by the merge kernel
  float *cand_val;          // [M, kStatChunks, k] chunk-local top-k (decreasing)
  int32_t *cand_idx;
  int32_t *ids;             // [M, k]
  float *logp;              // [M, k] natural-log softmax
  int32_t M, V, k;
};
hipError_t launch_topk(const TopkArgs &a, hipStream_t st);

struct ExpandArgs {
  const int32_t *front_in;  // [n_front] pool indices, or nullptr (root)
  const int32_t *cand_ids;  // [n_front, width]
  const float *cand_logp;
  int32_t *pool_tok, *pool_par;
  float *pool_score;
  int32_t *front_out;       // [width]
  int32_t n_front, width, n_pool;
};
hipError_t launch_tree_expand(const ExpandArgs &a, hipStream_t st);

struct SelectArgs {
  const int32_t *pool_tok, *pool_par;
  const float *pool_score;
  int32_t *parent, *ids, *pool_index;   // [min(total, n_pool)]
  int32_t n_pool, total;
};
hipError_t launch_tree_select(const SelectArgs &a, hipStream_t st);

}  // namespace sparrow
