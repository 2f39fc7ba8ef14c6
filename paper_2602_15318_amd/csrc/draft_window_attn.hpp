// Internal interface of the draft window-attention kernel.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/sparrow.h"

namespace sparrow {

struct DraftTable {
  int32_t cu_len[SPARROW_MAX_BATCH + 1];   // token offset of every sequence in k/v
  int32_t cu_text[SPARROW_MAX_BATCH + 1];  // offsets into text_idx
};

struct DraftArgs {
  const void *q, *k, *v;
  const int32_t *text_idx;
  int32_t B, Hq, Hkv, d, window;
  float scale_log2;
  int64_t stride_tok, stride_head;
  void *out;
  float *lse;
};

hipError_t launch_draft_window_attn(int dtype, const DraftArgs &a, const DraftTable &tab,
                                    hipStream_t st);

}  // namespace sparrow
