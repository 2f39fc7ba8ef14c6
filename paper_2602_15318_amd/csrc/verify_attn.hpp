// Internal interface of the verification-attention kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/sparrow.h"

namespace sparrow {

// Per-call schedule, passed to the kernels by value (no device-side schedule buffer, so a call is
// a pure function of its arguments and can be captured in a graph).  The context of every
// sequence is cut into splits of `chunk` tokens; split slots are numbered across sequences.
struct SeqTable {
  int32_t cu_len[SPARROW_MAX_BATCH + 1];    // token offsets (L_b + n_q rows per sequence)
  int32_t cu_split[SPARROW_MAX_BATCH + 1];  // split-slot offsets
};

struct VerifyArgs {
  const void *q, *k, *v;
  const int32_t *parent;  // device, or nullptr for a chain
  int32_t parent_stride;  // 0: one tree [n_q] for all sequences; else sequence b's tree at parent + b*stride
  int32_t B, n_q, Hq, Hkv, d;
  int32_t chunk;          // longest split of the call, in tokens (the kernels derive each
                          // sequence's own split length from SeqTable)
  int32_t n_slots;        // cu_split[B]
  float scale_log2;       // softmax scale * log2(e)
  int64_t stride_tok, stride_head;
  // plain-ALU path: part_o [n_slots, n_q, Hq, d], part_ml [n_slots, n_q, Hq, 2];
  // matrix-core path: tiled per (split, KV head, row block), see verify_attn_mfma.hip
  float *part_o;          // partial outputs (plain-ALU path: unnormalised fp32; matrix-core
                          // path: normalised fp16)
  float *part_ml;         // running max (log2 domain), partial sum
  void *out;              // [B*n_q, Hq, d]
  float *lse;             // [B*n_q, Hq] or nullptr
};

// Token range [t0, t1) of a split: a sequence of `len` rows with `ns` splits is cut into pieces of
// ceil(len / ns) rounded up to a whole 32-token tile (the last piece takes what is left, possibly
// nothing), so that all workgroups of a sequence stream the same number of bytes.
__host__ __device__ __forceinline__ int split_len(int len, int ns) {
  return ((len + ns - 1) / ns + 31) / 32 * 32;
}

// Which sequence owns split slot `slot` (linear scan; B <= SPARROW_MAX_BATCH).
__device__ __forceinline__ int seq_of_slot(const SeqTable &tab, int B, int slot) {
  int b = 0;
  while (b + 1 < B && tab.cu_split[b + 1] <= slot) ++b;
  return b;
}

// Partial pass, plain-ALU version: any supported dtype / head_dim.
hipError_t launch_verify_partial_generic(int dtype, const VerifyArgs &a, const SeqTable &tab,
                                         hipStream_t st);
// Partial pass, matrix-core version: bf16, head_dim 128.
bool verify_partial_mfma_supported(int dtype, int head_dim);
hipError_t launch_verify_partial_mfma(const VerifyArgs &a, const SeqTable &tab, hipStream_t st);
// Workgroups per (split, KV head) for R = n_q * (Hq / Hkv) rows.
int verify_mfma_row_blocks(int R);
// Its partials use a tiled layout of their own: workspace floats per (split, KV head, block of 64
// rows) unit, and the matching combine pass.
int64_t verify_mfma_unit_floats_o();
int64_t verify_mfma_unit_floats_ml();
hipError_t launch_verify_combine_mfma(const VerifyArgs &a, const SeqTable &tab, hipStream_t st);
// Second pass: merge the per-split partials of every (row, head).
hipError_t launch_verify_combine(int dtype, const VerifyArgs &a, const SeqTable &tab,
                                 hipStream_t st);

}  // namespace sparrow
