// Internal interface of the draft's input-side kernels: the hidden-state-reuse projection (Eq. 1)
// and the draft layer's norm / QKV / rotary step with the K/V append.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/sparrow.h"

namespace sparrow {

constexpr int kHsrMaxRows = 64;

// z[m, n] = bias[n] + W[n, 0:H] . embed[token_ids[m], :] + W[n, H:2H] . h_prev[m, :]
struct HsrFcArgs {
  const void *embed;          // [vocab, H]
  const int32_t *token_ids;   // [M]
  const void *h_prev;         // [M, H]
  const void *w;              // [H, 2H]
  const void *bias;           // [H] or nullptr
  void *z;                    // [M, H]
  int32_t M, H, vocab;
};

// u = RMSNorm(z) * gamma; y = W u + bias; rotary embedding on q and k heads; scatter.
struct DraftQkvArgs {
  const void *z;              // [M, H]
  const void *gamma;          // [H]
  const void *w;              // [(Hq + 2 Hkv) d, H], rows: q heads, k heads, v heads
  const void *bias;           // [(Hq + 2 Hkv) d] or nullptr
  const float *rope_cos;      // [M, d/2]
  const float *rope_sin;      // [M, d/2]
  void *q_out;                // [M, Hq, d]
  void *k_cache, *v_cache;    // row r, head c at r*stride_tok + c*stride_head
  int64_t stride_tok, stride_head;
  float eps;
  int32_t M, H, Hq, Hkv, d;
  int32_t kv_rows[kHsrMaxRows];   // cache row that receives the K/V of new token m
};

bool hsr_mfma_supported(int dtype, int H);
hipError_t launch_hsr_fc(int dtype, const HsrFcArgs &a, hipStream_t st);
hipError_t launch_draft_qkv(int dtype, const DraftQkvArgs &a, hipStream_t st);

}  // namespace sparrow
