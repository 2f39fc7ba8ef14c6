// Internal interface of the post-accept commit kernel.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/sparrow.h"

namespace sparrow {

constexpr int kCommitMaxLayers = 64;

struct CommitArgs {
  void *k[kCommitMaxLayers];      // per layer: K and V with the verification layout
  void *v[kCommitMaxLayers];
  int32_t cu_len[SPARROW_MAX_BATCH + 1];   // sequence b owns rows cu_len[b] .. cu_len[b+1]-1
  const int32_t *accept_path;     // [B, n_q]
  const int32_t *accept_len;      // [B]
  const void *hidden;             // [B*(n_q+1), H] or nullptr
  void *next_hidden;              // [B, H]
  int64_t stride_tok, stride_head;   // in elements
  int32_t n_layers, B, n_q, Hkv, d, H, esize;
};

hipError_t launch_kv_commit(const CommitArgs &a, hipStream_t st);

}  // namespace sparrow
