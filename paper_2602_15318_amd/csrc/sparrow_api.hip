// Host side of the C ABI declared in include/sparrow.h: argument validation, split planning,
// kernel selection and launches.  No device allocation, no synchronisation, no device reads.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <vector>

#include "../../include/sparrow.h"
#include "accept.hpp"
#include "draft_tree.hpp"
#include "draft_window_attn.hpp"
#include "hsr_input.hpp"
#include "kv_commit.hpp"
#include "verify_attn.hpp"

// Library-owned scratch of sparrow_verify_attn_static: one copy per GPU, held from the moment the
// code object is loaded on that GPU until the process ends.  In host code the name `scratch` is
// only a handle for hipGetSymbolAddress; the device address that call yields differs per GPU and
// is what the kernels are given.
static __device__ __align__(256) unsigned char scratch[SPARROW_STATIC_WS_BYTES];

namespace sparrow {
int generic_num_candidates(int V);
hipError_t launch_stream_read(const void *p, size_t bytes, unsigned int *sink, int workgroups,
                              int in_flight, int regions, hipStream_t st);

namespace {
thread_local char g_err[512] = "";

int fail(int code, const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
constexpr int kNumCU = 256;   // MI355X
constexpr int kNumXCD = 8;    // 32 compute units and one L2 each

int check_desc(const sparrow_attn_desc *d) {
  if (!d) return fail(SPARROW_ERR_INVALID_ARG, "desc is NULL");
  if (d->dtype != SPARROW_F32 && d->dtype != SPARROW_BF16)
    return fail(SPARROW_ERR_UNSUPPORTED, "dtype %d is neither SPARROW_F32 nor SPARROW_BF16", d->dtype);
  if (d->n_q_heads <= 0 || d->n_kv_heads <= 0 || d->n_q_heads % d->n_kv_heads != 0)
    return fail(SPARROW_ERR_INVALID_ARG, "n_q_heads %d must be a positive multiple of n_kv_heads %d",
                d->n_q_heads, d->n_kv_heads);
  if (d->head_dim != 64 && d->head_dim != 128)
    return fail(SPARROW_ERR_UNSUPPORTED, "head_dim %d (supported: 64, 128)", d->head_dim);
  const int per = d->dtype == SPARROW_BF16 ? 8 : 4;
  // token-major ([T, Hkv, d]: a token's heads side by side) or head-major ([Hkv, T, d]: a head's
  // tokens side by side; that stride_head covers all tokens is the caller's precondition)
  const bool token_major = d->kv_stride_token >= d->kv_stride_head * d->n_kv_heads;
  const bool head_major = d->kv_stride_head >= d->kv_stride_token;
  if (d->kv_stride_head < d->head_dim || d->kv_stride_head % per != 0 ||
      d->kv_stride_token < d->head_dim || d->kv_stride_token % per != 0 ||
      !(token_major || head_major))
    return fail(SPARROW_ERR_INVALID_ARG,
                "kv strides (token %lld, head %lld) must be multiples of 16 bytes, at least "
                "head_dim, and either stride_token >= n_kv_heads*stride_head (token-major) or "
                "stride_head >= stride_token (head-major)",
                (long long)d->kv_stride_token, (long long)d->kv_stride_head);
  if (!(d->scale >= 0.f) || std::isinf(d->scale))
    return fail(SPARROW_ERR_INVALID_ARG, "scale must be finite and >= 0 (0 = 1/sqrt(head_dim))");
  return SPARROW_OK;
}

float scale_log2_of(const sparrow_attn_desc *d) {
  const float s = d->scale > 0.f ? d->scale : 1.0f / std::sqrt((float)d->head_dim);
  return s * 1.4426950408889634f;
}

// Tokens per context split.  Aim at about one workgroup per compute unit: the split partials are
// pure overhead traffic, so no more splits than it takes to occupy the chip.
int plan_chunk(const sparrow_attn_desc *d, int32_t n_q, int64_t total_tokens, bool mfma) {
  const int R = n_q * (d->n_q_heads / d->n_kv_heads);
  const int rbs = mfma ? verify_mfma_row_blocks(R) : (R + 15) / 16;
  int slots;
  if (mfma) {
    // The row blocks of one (split, KV head) run side by side on one XCD (they share the K/V
    // stream through its L2), one workgroup per compute unit: whole groups per XCD only.
    const int groups_per_xcd = (kNumCU / kNumXCD) / rbs > 0 ? (kNumCU / kNumXCD) / rbs : 1;
    slots = groups_per_xcd * kNumXCD / d->n_kv_heads;
  } else {
    slots = kNumCU / (d->n_kv_heads * rbs);
  }
  if (slots < 1) slots = 1;
  int64_t chunk = (total_tokens + slots - 1) / slots;
  chunk = (int64_t)round_up((size_t)chunk, 32);
  if (chunk < 64) chunk = 64;
  return (int)chunk;
}

// The matrix-core kernel addresses a sequence's K/V rows by 32-bit byte offsets; judged on the
// call's total token count so that the workspace query and the call always agree.
bool use_mfma_verify(const sparrow_attn_desc *d, int64_t total_tokens) {
  return verify_partial_mfma_supported(d->dtype, d->head_dim) &&
         d->kv_stride_token < (1ll << 24) &&
         total_tokens * d->kv_stride_token * 2 < (1ll << 31);
}

// Workspace split: partial outputs first, then (max, sum) pairs, each rounded up to 256 bytes.
void verify_ws_layout(const sparrow_attn_desc *d, int64_t slots, int32_t n_q, bool mfma,
                      size_t *bytes_o, size_t *bytes_ml) {
  if (mfma) {
    const int R = n_q * (d->n_q_heads / d->n_kv_heads);
    const size_t units = (size_t)slots * d->n_kv_heads * ((R + 63) / 64);
    *bytes_o = round_up(units * verify_mfma_unit_floats_o() * sizeof(float), 256);
    *bytes_ml = round_up(units * verify_mfma_unit_floats_ml() * sizeof(float), 256);
  } else {
    const size_t rows = (size_t)slots * n_q * d->n_q_heads;
    *bytes_o = round_up(rows * d->head_dim * sizeof(float), 256);
    *bytes_ml = round_up(rows * 2 * sizeof(float), 256);
  }
}

size_t verify_ws_bytes(const sparrow_attn_desc *d, int64_t max_slots, int32_t n_q, bool mfma) {
  size_t bo, bml;
  verify_ws_layout(d, max_slots, n_q, mfma, &bo, &bml);
  return bo + bml;
}

constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices];

// Device address of `scratch` on the current device (looked up once per device).
int static_scratch(void **out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail(SPARROW_ERR_DEVICE, "hipGetDevice: %s", hipGetErrorString(e));
  if (dev < 0 || dev >= kMaxDevices) return fail(SPARROW_ERR_UNSUPPORTED, "device index %d (0..%d)", dev, kMaxDevices - 1);
  void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (p == nullptr) {
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || p == nullptr)
      return fail(SPARROW_ERR_DEVICE, "hipGetSymbolAddress(scratch) on device %d: %s", dev, hipGetErrorString(e));
    g_scratch_ptr[dev].store(p, std::memory_order_release);   // every thread finds the same address
  }
  *out = p;
  return SPARROW_OK;
}
}  // namespace
}  // namespace sparrow

using namespace sparrow;

extern "C" {

// ------------------------------------------------------------------ draft input side
int sparrow_hsr_fc(int32_t dtype, const void *embed, const int32_t *token_ids, const void *h_prev,
                   const void *w_fc, const void *b_fc, int32_t M, int32_t hidden, int32_t vocab,
                   void *z, void *hip_stream) {
  g_err[0] = 0;
  if (dtype != SPARROW_F32 && dtype != SPARROW_BF16)
    return fail(SPARROW_ERR_UNSUPPORTED, "dtype %d is neither SPARROW_F32 nor SPARROW_BF16", dtype);
  if (M < 0 || hidden <= 0 || vocab <= 0)
    return fail(SPARROW_ERR_INVALID_ARG, "M = %d, hidden = %d, vocab = %d", M, hidden, vocab);
  if (M == 0) return SPARROW_OK;
  if (M > kHsrMaxRows) return fail(SPARROW_ERR_UNSUPPORTED, "M = %d exceeds %d rows", M, kHsrMaxRows);
  if (hidden % 8 != 0) return fail(SPARROW_ERR_UNSUPPORTED, "hidden = %d is not a multiple of 8", hidden);
  if (!embed || !token_ids || !h_prev || !w_fc || !z)
    return fail(SPARROW_ERR_INVALID_ARG, "NULL pointer among embed/token_ids/h_prev/w_fc/z");
  if (!aligned16(embed) || !aligned16(h_prev) || !aligned16(w_fc) || !aligned16(z) ||
      (b_fc && !aligned16(b_fc)))
    return fail(SPARROW_ERR_INVALID_ARG, "embed, h_prev, w_fc, b_fc and z must be 16-byte aligned");
  HsrFcArgs a;
  a.embed = embed; a.token_ids = token_ids; a.h_prev = h_prev; a.w = w_fc; a.bias = b_fc; a.z = z;
  a.M = M; a.H = hidden; a.vocab = vocab;
  const hipError_t e = launch_hsr_fc(dtype, a, (hipStream_t)hip_stream);
  if (e != hipSuccess) return fail(SPARROW_ERR_DEVICE, "hsr_fc launch: %s", hipGetErrorString(e));
  return SPARROW_OK;
}

int sparrow_draft_qkv_append(const sparrow_attn_desc *desc, const void *z, const void *norm_weight,
                             float eps, const void *w_qkv, const void *b_qkv,
                             const float *rope_cos, const float *rope_sin,
                             const int32_t *kv_rows, int32_t M, int32_t hidden, void *q_out,
                             void *k_cache, void *v_cache, void *hip_stream) {
  g_err[0] = 0;
  if (int rc = check_desc(desc)) return rc;
  if (M < 0 || hidden <= 0) return fail(SPARROW_ERR_INVALID_ARG, "M = %d, hidden = %d", M, hidden);
  if (M == 0) return SPARROW_OK;
  if (M > kHsrMaxRows) return fail(SPARROW_ERR_UNSUPPORTED, "M = %d exceeds %d rows", M, kHsrMaxRows);
  if (hidden % 8 != 0) return fail(SPARROW_ERR_UNSUPPORTED, "hidden = %d is not a multiple of 8", hidden);
  if (!(eps >= 0.f) || std::isinf(eps)) return fail(SPARROW_ERR_INVALID_ARG, "eps must be finite and >= 0");
  if (!z || !norm_weight || !w_qkv || !rope_cos || !rope_sin || !kv_rows || !q_out || !k_cache || !v_cache)
    return fail(SPARROW_ERR_INVALID_ARG,
                "NULL pointer among z/norm_weight/w_qkv/rope_cos/rope_sin/kv_rows/q_out/k_cache/v_cache");
  if (!aligned16(z) || !aligned16(norm_weight) || !aligned16(w_qkv) || (b_qkv && !aligned16(b_qkv)) ||
      !aligned16(q_out) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(rope_cos) ||
      !aligned16(rope_sin))
    return fail(SPARROW_ERR_INVALID_ARG,
                "z, norm_weight, w_qkv, b_qkv, rope_cos, rope_sin, q_out and the caches must be 16-byte aligned");
  DraftQkvArgs a;
  for (int m = 0; m < M; ++m) {
    if (kv_rows[m] < 0) return fail(SPARROW_ERR_INVALID_ARG, "kv_rows[%d] = %d is negative", m, kv_rows[m]);
    for (int j = 0; j < m; ++j)
      if (kv_rows[j] == kv_rows[m])
        return fail(SPARROW_ERR_INVALID_ARG, "kv_rows[%d] and kv_rows[%d] name the same cache row %d", j, m, kv_rows[m]);
    a.kv_rows[m] = kv_rows[m];
  }
  for (int m = M; m < kHsrMaxRows; ++m) a.kv_rows[m] = 0;
  a.z = z; a.gamma = norm_weight; a.w = w_qkv; a.bias = b_qkv;
  a.rope_cos = rope_cos; a.rope_sin = rope_sin;
  a.q_out = q_out; a.k_cache = k_cache; a.v_cache = v_cache;
  a.stride_tok = desc->kv_stride_token; a.stride_head = desc->kv_stride_head;
  a.eps = eps; a.M = M; a.H = hidden;
  a.Hq = desc->n_q_heads; a.Hkv = desc->n_kv_heads; a.d = desc->head_dim;
  const hipError_t e = launch_draft_qkv(desc->dtype, a, (hipStream_t)hip_stream);
  if (e != hipSuccess) return fail(SPARROW_ERR_DEVICE, "draft_qkv launch: %s", hipGetErrorString(e));
  return SPARROW_OK;
}

// ------------------------------------------------------------------ post-accept commit
int sparrow_kv_commit(const sparrow_attn_desc *desc, void *const *k_layers, void *const *v_layers,
                      int32_t n_layers, const int32_t *cu_seqlens, int32_t B, int32_t n_q,
                      const int32_t *accept_path, const int32_t *accept_len,
                      const void *hidden_rows, int32_t hidden, void *next_hidden,
                      void *hip_stream) {
  g_err[0] = 0;
  if (int rc = check_desc(desc)) return rc;
  if (n_layers < 0 || B < 0 || n_q < 0)
    return fail(SPARROW_ERR_INVALID_ARG, "n_layers = %d, B = %d, n_q = %d: negative", n_layers, B, n_q);
  if (n_layers > kCommitMaxLayers) return fail(SPARROW_ERR_UNSUPPORTED, "n_layers = %d exceeds %d", n_layers, kCommitMaxLayers);
  if (B > SPARROW_MAX_BATCH) return fail(SPARROW_ERR_UNSUPPORTED, "B = %d exceeds %d", B, SPARROW_MAX_BATCH);
  if (n_q > SPARROW_MAX_NQ) return fail(SPARROW_ERR_UNSUPPORTED, "n_q = %d exceeds %d", n_q, SPARROW_MAX_NQ);
  if (B == 0 || (n_layers == 0 && !hidden_rows)) return SPARROW_OK;
  if (!cu_seqlens || !accept_path || !accept_len)
    return fail(SPARROW_ERR_INVALID_ARG, "NULL pointer among cu_seqlens/accept_path/accept_len");
  if (n_layers > 0 && (!k_layers || !v_layers)) return fail(SPARROW_ERR_INVALID_ARG, "k_layers / v_layers is NULL");
  const int esize = desc->dtype == SPARROW_BF16 ? 2 : 4;
  CommitArgs a;
  memset(&a, 0, sizeof(a));
  for (int l = 0; l < n_layers; ++l) {
    if (!k_layers[l] || !v_layers[l] || !aligned16(k_layers[l]) || !aligned16(v_layers[l]))
      return fail(SPARROW_ERR_INVALID_ARG, "layer %d: K/V pointer NULL or not 16-byte aligned", l);
    a.k[l] = k_layers[l];
    a.v[l] = v_layers[l];
  }
  if (cu_seqlens[0] < 0) return fail(SPARROW_ERR_INVALID_ARG, "cu_seqlens[0] must be >= 0");
  for (int b = 0; b < B; ++b)
    if (cu_seqlens[b + 1] - cu_seqlens[b] < n_q)
      return fail(SPARROW_ERR_INVALID_ARG, "sequence %d has %d rows, fewer than its n_q = %d draft rows",
                  b, cu_seqlens[b + 1] - cu_seqlens[b], n_q);
  for (int b = 0; b <= B; ++b) a.cu_len[b] = cu_seqlens[b];
  if (hidden_rows) {
    if (!next_hidden) return fail(SPARROW_ERR_INVALID_ARG, "hidden_rows given but next_hidden is NULL");
    if (hidden <= 0 || (hidden * esize) % 16 != 0)
      return fail(SPARROW_ERR_UNSUPPORTED, "hidden = %d: rows must be a positive multiple of 16 bytes", hidden);
    if (!aligned16(hidden_rows) || !aligned16(next_hidden))
      return fail(SPARROW_ERR_INVALID_ARG, "hidden_rows and next_hidden must be 16-byte aligned");
  }
  a.accept_path = accept_path; a.accept_len = accept_len;
  a.hidden = hidden_rows; a.next_hidden = next_hidden;
  a.stride_tok = desc->kv_stride_token; a.stride_head = desc->kv_stride_head;
  a.n_layers = n_layers; a.B = B; a.n_q = n_q; a.Hkv = desc->n_kv_heads; a.d = desc->head_dim;
  a.H = hidden; a.esize = esize;
  const hipError_t e = launch_kv_commit(a, (hipStream_t)hip_stream);
  if (e != hipSuccess) return fail(SPARROW_ERR_DEVICE, "kv_commit launch: %s", hipGetErrorString(e));
  return SPARROW_OK;
}

int sparrow_stream_read_shape(const void *dev_ptr, size_t bytes, void *sink, int32_t workgroups,
                              int32_t loads_in_flight, int32_t regions, void *hip_stream) {
  g_err[0] = 0;
  if (bytes == 0) return SPARROW_OK;
  if (!dev_ptr || !sink || !aligned16(dev_ptr) || bytes % 16 != 0)
    return fail(SPARROW_ERR_INVALID_ARG, "stream_read: NULL or misaligned pointer, or bytes not a multiple of 16");
  if (workgroups < 1 || workgroups > 65536)
    return fail(SPARROW_ERR_INVALID_ARG, "stream_read: workgroups = %d (1..65536)", workgroups);
  if (loads_in_flight != 2 && loads_in_flight != 4 && loads_in_flight != 8 && loads_in_flight != 16)
    return fail(SPARROW_ERR_UNSUPPORTED, "stream_read: loads_in_flight = %d (2, 4, 8 or 16)", loads_in_flight);
  const hipError_t e = launch_stream_read(dev_ptr, bytes, (unsigned int *)sink, workgroups, loads_in_flight,
                                          regions != 0, (hipStream_t)hip_stream);
  if (e != hipSuccess) return fail(SPARROW_ERR_DEVICE, "stream_read launch: %s", hipGetErrorString(e));
  return SPARROW_OK;
}

int sparrow_stream_read(const void *dev_ptr, size_t bytes, void *sink, void *hip_stream) {
  return sparrow_stream_read_shape(dev_ptr, bytes, sink, 1024, 8, 0, hip_stream);
}

// ------------------------------------------------------------------ debug aids
// Host copy of `n` int32 at `p`, wherever they live.  Memory the runtime does not know (plain host
// memory; every pointer on a machine without a device) is read in place.
static int host_copy_i32(const int32_t *p, size_t n, hipStream_t st, std::vector<int32_t> *out) {
  out->resize(n);
  if (n == 0) return SPARROW_OK;
  hipPointerAttribute_t attr;
  const hipError_t qa = hipPointerGetAttributes(&attr, p);
  if (qa != hipSuccess) (void)hipGetLastError();          // unknown pointer: clear the sticky error
  const bool on_device = qa == hipSuccess && (attr.type == hipMemoryTypeDevice || attr.type == hipMemoryTypeManaged);
  if (!on_device) {
    memcpy(out->data(), p, n * sizeof(int32_t));
    return SPARROW_OK;
  }
  hipError_t e = hipMemcpyAsync(out->data(), p, n * sizeof(int32_t), hipMemcpyDeviceToHost, st);
  if (e == hipSuccess) e = hipStreamSynchronize(st);
  if (e != hipSuccess) return fail(SPARROW_ERR_DEVICE, "copy to the host: %s", hipGetErrorString(e));
  return SPARROW_OK;
}

int sparrow_debug_validate_parent(const int32_t *parent, int32_t parent_stride, int32_t B,
                                  int32_t n_q, void *hip_stream) {
  g_err[0] = 0;
  if (n_q < 0 || n_q > SPARROW_MAX_NQ) return fail(SPARROW_ERR_INVALID_ARG, "n_q = %d (0..%d)", n_q, SPARROW_MAX_NQ);
  if (!parent || n_q == 0) return SPARROW_OK;             // NULL = chain: nothing to check
  if (parent_stride != 0 && (parent_stride < n_q || B < 0 || B > SPARROW_MAX_BATCH))
    return fail(SPARROW_ERR_INVALID_ARG, "parent_stride = %d (0 or >= n_q = %d), B = %d", parent_stride, n_q, B);
  const int trees = parent_stride == 0 ? 1 : B;
  if (trees == 0) return SPARROW_OK;
  const size_t n = parent_stride == 0 ? (size_t)n_q : (size_t)(trees - 1) * parent_stride + n_q;
  std::vector<int32_t> h;
  if (int rc = host_copy_i32(parent, n, (hipStream_t)hip_stream, &h)) return rc;
  for (int b = 0; b < trees; ++b)
    for (int i = 0; i < n_q; ++i) {
      const int32_t pi = h[(size_t)b * parent_stride + i];
      if (pi < -1 || pi >= i)
        return fail(SPARROW_ERR_INVALID_ARG, "tree %d: parent[%d] = %d is outside [-1, %d)", b, i, pi, i);
    }
  return SPARROW_OK;
}

int sparrow_debug_validate_text_idx(const int32_t *text_idx, const int32_t *cu_seqlens,
                                    const int32_t *cu_text, int32_t B, void *hip_stream) {
  g_err[0] = 0;
  if (B < 0 || B > SPARROW_MAX_BATCH) return fail(SPARROW_ERR_INVALID_ARG, "B = %d (0..%d)", B, SPARROW_MAX_BATCH);
  if (B == 0) return SPARROW_OK;
  if (!text_idx || !cu_seqlens || !cu_text) return fail(SPARROW_ERR_INVALID_ARG, "NULL pointer among text_idx/cu_seqlens/cu_text");
  if (cu_text[0] < 0 || cu_seqlens[0] < 0) return fail(SPARROW_ERR_INVALID_ARG, "cu_text[0] and cu_seqlens[0] must be >= 0");
  for (int b = 0; b < B; ++b)
    if (cu_text[b + 1] <= cu_text[b] || cu_seqlens[b + 1] <= cu_seqlens[b])
      return fail(SPARROW_ERR_INVALID_ARG, "sequence %d: %d text positions in %d tokens", b,
                  cu_text[b + 1] - cu_text[b], cu_seqlens[b + 1] - cu_seqlens[b]);
  std::vector<int32_t> h;
  if (int rc = host_copy_i32(text_idx + cu_text[0], (size_t)(cu_text[B] - cu_text[0]), (hipStream_t)hip_stream, &h)) return rc;
  for (int b = 0; b < B; ++b) {
    const int len = cu_seqlens[b + 1] - cu_seqlens[b];
    int prev = -1;
    for (int j = cu_text[b]; j < cu_text[b + 1]; ++j) {
      const int32_t t = h[(size_t)(j - cu_text[0])];
      if (t <= prev || t >= len)
        return fail(SPARROW_ERR_INVALID_ARG,
                    "sequence %d: text_idx[%d] = %d is not above its predecessor %d or not below the sequence's %d tokens",
                    b, j, t, prev, len);
      prev = t;
    }
  }
  return SPARROW_OK;
}

const char *sparrow_last_error(void) { return g_err; }
const char *sparrow_version(void) { return "0.2"; }

// ------------------------------------------------------------------ draft window attention
size_t sparrow_draft_window_attn_workspace(const sparrow_attn_desc *, int32_t, int32_t) { return 0; }

int sparrow_draft_window_attn(const sparrow_attn_desc *desc, const void *q, const void *k,
                              const void *v, const int32_t *cu_seqlens, const int32_t *text_idx,
                              const int32_t *cu_text, int32_t B, int32_t window, void *out,
                              float *lse, void *workspace, size_t workspace_bytes,
                              void *hip_stream) {
  (void)workspace; (void)workspace_bytes;
  g_err[0] = 0;
  if (int rc = check_desc(desc)) return rc;
  if (B < 0) return fail(SPARROW_ERR_INVALID_ARG, "B = %d is negative", B);
  if (B == 0) return SPARROW_OK;
  if (B > SPARROW_MAX_BATCH) return fail(SPARROW_ERR_UNSUPPORTED, "B = %d exceeds %d", B, SPARROW_MAX_BATCH);
  if (window <= 0) return fail(SPARROW_ERR_INVALID_ARG, "window = %d must be positive", window);
  if (!q || !k || !v || !cu_seqlens || !text_idx || !cu_text || !out)
    return fail(SPARROW_ERR_INVALID_ARG, "NULL pointer among q/k/v/cu_seqlens/text_idx/cu_text/out");
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out))
    return fail(SPARROW_ERR_INVALID_ARG, "q, k, v and out must be 16-byte aligned");
  DraftTable tab;
  memset(&tab, 0, sizeof(tab));
  if (cu_seqlens[0] < 0 || cu_text[0] < 0)
    return fail(SPARROW_ERR_INVALID_ARG, "cu_seqlens[0] and cu_text[0] must be >= 0");
  for (int b = 0; b <= B; ++b) { tab.cu_len[b] = cu_seqlens[b]; tab.cu_text[b] = cu_text[b]; }
  for (int b = 0; b < B; ++b) {
    const int len = cu_seqlens[b + 1] - cu_seqlens[b], nt = cu_text[b + 1] - cu_text[b];
    if (len <= 0) return fail(SPARROW_ERR_INVALID_ARG, "sequence %d has %d tokens", b, len);
    if (nt <= 0)
      return fail(SPARROW_ERR_INVALID_ARG,
                  "sequence %d has no text position: softmax over an empty set is undefined", b);
    if (nt > len)
      return fail(SPARROW_ERR_INVALID_ARG, "sequence %d: %d text positions in %d tokens", b, nt, len);
  }
  DraftArgs a;
  a.q = q; a.k = k; a.v = v; a.text_idx = text_idx;
  a.B = B; a.Hq = desc->n_q_heads; a.Hkv = desc->n_kv_heads; a.d = desc->head_dim;
  a.window = window;
  a.scale_log2 = scale_log2_of(desc);
  a.stride_tok = desc->kv_stride_token; a.stride_head = desc->kv_stride_head;
  a.out = out; a.lse = lse;
  hipError_t e = launch_draft_window_attn(desc->dtype, a, tab, (hipStream_t)hip_stream);
  if (e != hipSuccess) return fail(SPARROW_ERR_DEVICE, "draft_window_attn launch: %s", hipGetErrorString(e));
  return SPARROW_OK;
}

// ------------------------------------------------------------------ verification attention
size_t sparrow_verify_attn_workspace(const sparrow_attn_desc *desc, int32_t B, int32_t n_q,
                                     int64_t total_tokens) {
  if (check_desc(desc) != SPARROW_OK || B <= 0 || n_q <= 0 || total_tokens <= 0) return 0;
  const bool mfma = use_mfma_verify(desc, total_tokens);
  const int chunk = plan_chunk(desc, n_q, total_tokens, mfma);
  const int64_t max_slots = (total_tokens + chunk - 1) / chunk + B;
  return verify_ws_bytes(desc, max_slots, n_q, mfma);
}

int sparrow_verify_attn(const sparrow_attn_desc *desc, const void *q, const void *k,
                        const void *v, const int32_t *cu_seqlens, const int32_t *parent,
                        int32_t B, int32_t n_q, void *out, float *lse, void *workspace,
                        size_t workspace_bytes, void *hip_stream) {
  return sparrow_verify_attn_passes(desc, q, k, v, cu_seqlens, parent, B, n_q, out, lse, workspace,
                                    workspace_bytes, hip_stream, 3);
}

// Shared body.  static_ws: the workspace is the library's own scratch array (looked up here, after
// validation, so that an invalid call never touches the device).
static int verify_body(const sparrow_attn_desc *desc, const void *q, const void *k,
                       const void *v, const int32_t *cu_seqlens, const int32_t *parent,
                       int32_t B, int32_t n_q, void *out, float *lse, void *workspace,
                       size_t workspace_bytes, void *hip_stream, int32_t passes, bool static_ws) {
  g_err[0] = 0;
  if (passes < 1 || passes > 3) return fail(SPARROW_ERR_INVALID_ARG, "passes = %d (1, 2 or 3)", passes);
  if (int rc = check_desc(desc)) return rc;
  if (B < 0 || n_q < 0) return fail(SPARROW_ERR_INVALID_ARG, "B = %d, n_q = %d: negative", B, n_q);
  if (B == 0 || n_q == 0) return SPARROW_OK;
  if (B > SPARROW_MAX_BATCH) return fail(SPARROW_ERR_UNSUPPORTED, "B = %d exceeds %d", B, SPARROW_MAX_BATCH);
  if (n_q > SPARROW_MAX_NQ) return fail(SPARROW_ERR_UNSUPPORTED, "n_q = %d exceeds %d", n_q, SPARROW_MAX_NQ);
  if (!q || !k || !v || !cu_seqlens || !out)
    return fail(SPARROW_ERR_INVALID_ARG, "NULL pointer among q/k/v/cu_seqlens/out");
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out))
    return fail(SPARROW_ERR_INVALID_ARG, "q, k, v and out must be 16-byte aligned");
  if (cu_seqlens[0] < 0) return fail(SPARROW_ERR_INVALID_ARG, "cu_seqlens[0] must be >= 0");
  for (int b = 0; b < B; ++b)
    if (cu_seqlens[b + 1] - cu_seqlens[b] < n_q)
      return fail(SPARROW_ERR_INVALID_ARG, "sequence %d has %d rows, fewer than its n_q = %d draft rows",
                  b, cu_seqlens[b + 1] - cu_seqlens[b], n_q);
  if (parent && desc->parent_stride != 0 && desc->parent_stride < n_q)
    return fail(SPARROW_ERR_INVALID_ARG, "parent_stride = %d must be 0 (one shared tree) or at least n_q = %d",
                desc->parent_stride, n_q);
  const int64_t total = (int64_t)cu_seqlens[B] - cu_seqlens[0];   // the figure the workspace query is given
  const bool mfma = use_mfma_verify(desc, total);
  // Splits per sequence in proportion to its length (at least one), within the budget of about one
  // workgroup per compute unit that plan_chunk aims at; each sequence is then cut into equal
  // pieces, so that every workgroup of the call streams about the same number of bytes.
  const int chunk0 = plan_chunk(desc, n_q, total, mfma);
  const int slot_budget = (int)((total + chunk0 - 1) / chunk0);
  SeqTable tab;
  memset(&tab, 0, sizeof(tab));
  for (int b = 0; b <= B; ++b) tab.cu_len[b] = cu_seqlens[b];
  int chunk = 0;
  {
    int ns[SPARROW_MAX_BATCH];
    int used = 0;
    for (int b = 0; b < B; ++b) {
      const int len = cu_seqlens[b + 1] - cu_seqlens[b];
      ns[b] = (int)((int64_t)len * slot_budget / (total > 0 ? total : 1));
      if (ns[b] < 1) ns[b] = 1;
      used += ns[b];
    }
    // hand the slots lost to rounding down to the sequences with the longest pieces
    while (used < slot_budget) {
      int worst = 0;
      double worst_len = -1.0;
      for (int b = 0; b < B; ++b) {
        const double piece = (double)(cu_seqlens[b + 1] - cu_seqlens[b]) / ns[b];
        if (piece > worst_len) { worst_len = piece; worst = b; }
      }
      ++ns[worst];
      ++used;
    }
    for (int b = 0; b < B; ++b) {
      const int len = cu_seqlens[b + 1] - cu_seqlens[b];
      tab.cu_split[b + 1] = tab.cu_split[b] + ns[b];
      const int piece = split_len(len, ns[b]);
      if (piece > chunk) chunk = piece;
    }
  }
  const int n_slots = tab.cu_split[B];
  const size_t need = verify_ws_bytes(desc, n_slots, n_q, mfma);
  if (static_ws) {
    if (need > (size_t)SPARROW_STATIC_WS_BYTES)
      return fail(SPARROW_ERR_UNSUPPORTED,
                  "this call needs %zu bytes of split partials, the static scratch holds %zu: use "
                  "sparrow_verify_attn with a workspace of the caller's",
                  need, (size_t)SPARROW_STATIC_WS_BYTES);
    if (int rc = static_scratch(&workspace)) return rc;
    workspace_bytes = SPARROW_STATIC_WS_BYTES;
  }
  if (!workspace || workspace_bytes < need)
    return fail(SPARROW_ERR_WORKSPACE, "workspace of %zu bytes needed, %zu given%s", need,
                workspace_bytes, workspace ? "" : " (NULL)");
  if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0)
    return fail(SPARROW_ERR_INVALID_ARG, "workspace must be 256-byte aligned");
  VerifyArgs a;
  a.q = q; a.k = k; a.v = v; a.parent = parent;
  a.parent_stride = parent ? desc->parent_stride : 0;
  a.B = B; a.n_q = n_q; a.Hq = desc->n_q_heads; a.Hkv = desc->n_kv_heads; a.d = desc->head_dim;
  a.chunk = chunk; a.n_slots = n_slots;
  a.scale_log2 = scale_log2_of(desc);
  a.stride_tok = desc->kv_stride_token; a.stride_head = desc->kv_stride_head;
  size_t bytes_o, bytes_ml;
  verify_ws_layout(desc, n_slots, n_q, mfma, &bytes_o, &bytes_ml);
  a.part_o = (float *)workspace;
  a.part_ml = (float *)((char *)workspace + bytes_o);
  a.out = out; a.lse = lse;
  hipStream_t st = (hipStream_t)hip_stream;
  if (passes & 1) {
    hipError_t e = mfma ? launch_verify_partial_mfma(a, tab, st)
                        : launch_verify_partial_generic(desc->dtype, a, tab, st);
    if (e != hipSuccess) return fail(SPARROW_ERR_DEVICE, "verify partial launch: %s", hipGetErrorString(e));
  }
  if (passes & 2) {
    hipError_t e = mfma ? launch_verify_combine_mfma(a, tab, st) : launch_verify_combine(desc->dtype, a, tab, st);
    if (e != hipSuccess) return fail(SPARROW_ERR_DEVICE, "verify combine launch: %s", hipGetErrorString(e));
  }
  return SPARROW_OK;
}

int sparrow_verify_attn_passes(const sparrow_attn_desc *desc, const void *q, const void *k,
                               const void *v, const int32_t *cu_seqlens, const int32_t *parent,
                               int32_t B, int32_t n_q, void *out, float *lse, void *workspace,
                               size_t workspace_bytes, void *hip_stream, int32_t passes) {
  return verify_body(desc, q, k, v, cu_seqlens, parent, B, n_q, out, lse, workspace, workspace_bytes,
                     hip_stream, passes, false);
}

int sparrow_verify_attn_static(const sparrow_attn_desc *desc, const void *q, const void *k,
                               const void *v, const int32_t *cu_seqlens, const int32_t *parent,
                               int32_t B, int32_t n_q, void *out, float *lse, void *hip_stream) {
  return verify_body(desc, q, k, v, cu_seqlens, parent, B, n_q, out, lse, nullptr, 0, hip_stream, 3,
                     true);
}

// ------------------------------------------------------------------ acceptance
static int accept_candidates(int32_t dtype, int M, int H, int V) {
  if (lm_head_mfma_supported(dtype, M, H, V)) return accept_num_candidates(dtype, M, H, V);
  return generic_num_candidates(V);
}

size_t sparrow_accept_workspace(int32_t dtype, int32_t B, int32_t n_q, int32_t hidden,
                                int32_t vocab) {
  if (B <= 0 || n_q < 0 || hidden <= 0 || vocab <= 0) return 0;
  const int M = B * (n_q + 1);
  const size_t n = (size_t)M * accept_candidates(dtype, M, hidden, vocab);
  return round_up(n * sizeof(float), 256) + round_up(n * sizeof(int32_t), 256);
}

// Shared body of the greedy and the stochastic acceptance.  sample == nullptr: greedy.
struct SampleParams {
  float temperature;
  const float *u_accept, *u_bonus;   // both given, or both NULL (generated from seed / offset)
  const float *draft_q;              // NULL: deterministic-children rule
  uint64_t seed, offset;
};

static size_t accept_sample_extra(int M, int vocab, size_t *logits_bytes, size_t *stats_bytes) {
  *logits_bytes = round_up((size_t)M * vocab * sizeof(float), 256);
  *stats_bytes = round_up((size_t)M * kStatChunks * 2 * sizeof(float), 256);
  return *logits_bytes + *stats_bytes + round_up((size_t)M * ((vocab + 255) / 256) * sizeof(float), 256);
}

size_t sparrow_accept_sample_workspace(int32_t dtype, int32_t B, int32_t n_q, int32_t hidden,
                                       int32_t vocab) {
  if (B <= 0 || n_q < 0 || hidden <= 0 || vocab <= 0) return 0;
  size_t lb, sb;
  return sparrow_accept_workspace(dtype, B, n_q, hidden, vocab) +
         accept_sample_extra(B * (n_q + 1), vocab, &lb, &sb);
}

static int accept_body(int32_t dtype, const void *hidden_rows, const void *lm_head,
                       const int32_t *draft_ids, const int32_t *parent, int32_t parent_stride,
                       int32_t B, int32_t n_q,
                       int32_t hidden, int32_t vocab, int32_t *target_ids, int32_t *accept_len,
                       int32_t *accept_path, int32_t *bonus_id, void *workspace,
                       size_t workspace_bytes, void *hip_stream, const SampleParams *sample) {
  g_err[0] = 0;
  if (dtype != SPARROW_F32 && dtype != SPARROW_BF16)
    return fail(SPARROW_ERR_UNSUPPORTED, "dtype %d is neither SPARROW_F32 nor SPARROW_BF16", dtype);
  if (B < 0 || n_q < 0) return fail(SPARROW_ERR_INVALID_ARG, "B = %d, n_q = %d: negative", B, n_q);
  if (B == 0) return SPARROW_OK;
  if (n_q > SPARROW_MAX_NQ) return fail(SPARROW_ERR_UNSUPPORTED, "n_q = %d exceeds %d", n_q, SPARROW_MAX_NQ);
  if ((int64_t)B * (n_q + 1) > kAcceptMaxRows)
    return fail(SPARROW_ERR_UNSUPPORTED, "B*(n_q+1) = %lld rows exceeds %d", (long long)B * (n_q + 1), kAcceptMaxRows);
  if (hidden <= 0 || vocab <= 0) return fail(SPARROW_ERR_INVALID_ARG, "hidden = %d, vocab = %d", hidden, vocab);
  if (parent && parent_stride != 0 && parent_stride < n_q)
    return fail(SPARROW_ERR_INVALID_ARG, "parent_stride = %d must be 0 (one shared tree) or at least n_q = %d",
                parent_stride, n_q);
  const int per = dtype == SPARROW_BF16 ? 8 : 4;
  if (hidden % per != 0)
    return fail(SPARROW_ERR_UNSUPPORTED, "hidden = %d must be a multiple of %d (16-byte rows)", hidden, per);
  if (!hidden_rows || !lm_head || (!sample && !target_ids) || !accept_len || !bonus_id ||
      (n_q > 0 && (!draft_ids || !accept_path)))
    return fail(SPARROW_ERR_INVALID_ARG, "NULL pointer among hidden_rows/lm_head/draft_ids/outputs");
  if (sample) {
    if (!(sample->temperature > 0.f) || std::isinf(sample->temperature))
      return fail(SPARROW_ERR_INVALID_ARG, "temperature must be finite and > 0");
    if (vocab > kSampleMaxVocab)
      return fail(SPARROW_ERR_UNSUPPORTED, "vocab = %d exceeds %d (stochastic acceptance)", vocab, kSampleMaxVocab);
    const bool generated = !sample->u_bonus && !sample->u_accept;
    if (!generated && (!sample->u_bonus || (n_q > 0 && !sample->u_accept)))
      return fail(SPARROW_ERR_INVALID_ARG, "u_accept and u_bonus must both be given or both be NULL");
    if (sample->draft_q && !aligned16(sample->draft_q))
      return fail(SPARROW_ERR_INVALID_ARG, "draft_probs must be 16-byte aligned");
  }
  if (!aligned16(hidden_rows) || !aligned16(lm_head))
    return fail(SPARROW_ERR_INVALID_ARG, "hidden_rows and lm_head must be 16-byte aligned");
  const int M = B * (n_q + 1);
  const bool mfma = lm_head_mfma_supported(dtype, M, hidden, vocab);
  const int n_cand = accept_candidates(dtype, M, hidden, vocab);
  const size_t base = sparrow_accept_workspace(dtype, B, n_q, hidden, vocab);
  size_t logits_bytes = 0, stats_bytes = 0;
  const size_t need = base + (sample ? accept_sample_extra(M, vocab, &logits_bytes, &stats_bytes) : 0);
  if (!workspace || workspace_bytes < need)
    return fail(SPARROW_ERR_WORKSPACE, "workspace of %zu bytes needed, %zu given%s", need,
                workspace_bytes, workspace ? "" : " (NULL)");
  if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0)
    return fail(SPARROW_ERR_INVALID_ARG, "workspace must be 256-byte aligned");
  AcceptArgs a;
  a.hidden = hidden_rows; a.lm_head = lm_head; a.draft_ids = draft_ids; a.parent = parent;
  a.parent_stride = parent ? parent_stride : 0;
  a.B = B; a.n_q = n_q; a.M = M; a.H = hidden; a.V = vocab; a.n_cand = n_cand;
  a.cand_val = (float *)workspace;
  a.cand_idx = (int32_t *)((char *)workspace + round_up((size_t)M * n_cand * sizeof(float), 256));
  a.target_ids = target_ids; a.accept_len = accept_len; a.accept_path = accept_path;
  a.bonus_id = bonus_id;
  a.logits = sample ? (float *)((char *)workspace + base) : nullptr;
  hipStream_t st = (hipStream_t)hip_stream;
  hipError_t e = mfma ? launch_lm_head_mfma(a, st) : launch_lm_head_generic(dtype, a, st);
  if (e != hipSuccess) return fail(SPARROW_ERR_DEVICE, "lm_head launch: %s", hipGetErrorString(e));
  if (!sample) {
    e = launch_accept_finalize(a, st);
    if (e != hipSuccess) return fail(SPARROW_ERR_DEVICE, "accept finalize launch: %s", hipGetErrorString(e));
    return SPARROW_OK;
  }
  SampleArgs s;
  s.logits = a.logits; s.draft_ids = draft_ids; s.parent = parent;
  s.parent_stride = a.parent_stride;
  s.u_accept = sample->u_accept; s.u_bonus = sample->u_bonus;
  s.draft_q = sample->draft_q; s.seed = sample->seed; s.offset = sample->offset;
  s.stats = (float *)((char *)workspace + base + logits_bytes);
  s.blk_sum = (float *)((char *)workspace + base + logits_bytes + stats_bytes);
  s.accept_len = accept_len; s.accept_path = accept_path; s.bonus_id = bonus_id;
  s.B = B; s.n_q = n_q; s.M = M; s.V = vocab;
  s.inv_temp_log2 = 1.4426950408889634f / sample->temperature;
  e = launch_logit_stats(s, st);
  if (e != hipSuccess) return fail(SPARROW_ERR_DEVICE, "logit statistics launch: %s", hipGetErrorString(e));
  e = launch_accept_sample(s, st);
  if (e != hipSuccess) return fail(SPARROW_ERR_DEVICE, "accept sample launch: %s", hipGetErrorString(e));
  return SPARROW_OK;
}

int sparrow_accept_trees(int32_t dtype, const void *hidden_rows, const void *lm_head,
                         const int32_t *draft_ids, const int32_t *parent, int32_t parent_stride,
                         int32_t B, int32_t n_q, int32_t hidden, int32_t vocab, int32_t *target_ids,
                         int32_t *accept_len, int32_t *accept_path, int32_t *bonus_id,
                         void *workspace, size_t workspace_bytes, void *hip_stream) {
  return accept_body(dtype, hidden_rows, lm_head, draft_ids, parent, parent_stride, B, n_q, hidden,
                     vocab, target_ids, accept_len, accept_path, bonus_id, workspace, workspace_bytes,
                     hip_stream, nullptr);
}

int sparrow_accept(int32_t dtype, const void *hidden_rows, const void *lm_head,
                   const int32_t *draft_ids, const int32_t *parent, int32_t B, int32_t n_q,
                   int32_t hidden, int32_t vocab, int32_t *target_ids, int32_t *accept_len,
                   int32_t *accept_path, int32_t *bonus_id, void *workspace,
                   size_t workspace_bytes, void *hip_stream) {
  return sparrow_accept_trees(dtype, hidden_rows, lm_head, draft_ids, parent, 0, B, n_q, hidden, vocab,
                              target_ids, accept_len, accept_path, bonus_id, workspace,
                              workspace_bytes, hip_stream);
}

int sparrow_accept_sample_trees(int32_t dtype, const void *hidden_rows, const void *lm_head,
                                const int32_t *draft_ids, const int32_t *parent,
                                int32_t parent_stride, int32_t B, int32_t n_q, int32_t hidden,
                                int32_t vocab, float temperature, const float *u_accept,
                                const float *u_bonus, int32_t *accept_len, int32_t *accept_path,
                                int32_t *bonus_id, void *workspace, size_t workspace_bytes,
                                void *hip_stream) {
  const SampleParams sp_ = {temperature, u_accept, u_bonus, nullptr, 0, 0};
  if (!u_bonus || (n_q > 0 && !u_accept)) {
    g_err[0] = 0;
    return fail(SPARROW_ERR_INVALID_ARG, "NULL pointer among u_accept/u_bonus");
  }
  return accept_body(dtype, hidden_rows, lm_head, draft_ids, parent, parent_stride, B, n_q, hidden,
                     vocab, nullptr, accept_len, accept_path, bonus_id, workspace, workspace_bytes,
                     hip_stream, &sp_);
}

int sparrow_accept_sample_q(int32_t dtype, const void *hidden_rows, const void *lm_head,
                            const int32_t *draft_ids, const int32_t *parent, int32_t parent_stride,
                            int32_t B, int32_t n_q, int32_t hidden, int32_t vocab, float temperature,
                            const float *draft_probs, const float *u_accept, const float *u_bonus,
                            uint64_t seed, uint64_t offset, int32_t *accept_len,
                            int32_t *accept_path, int32_t *bonus_id, void *workspace,
                            size_t workspace_bytes, void *hip_stream) {
  const SampleParams sp_ = {temperature, u_accept, u_bonus, draft_probs, seed, offset};
  return accept_body(dtype, hidden_rows, lm_head, draft_ids, parent, parent_stride, B, n_q, hidden,
                     vocab, nullptr, accept_len, accept_path, bonus_id, workspace, workspace_bytes,
                     hip_stream, &sp_);
}

int sparrow_accept_sample(int32_t dtype, const void *hidden_rows, const void *lm_head,
                          const int32_t *draft_ids, const int32_t *parent, int32_t B, int32_t n_q,
                          int32_t hidden, int32_t vocab, float temperature, const float *u_accept,
                          const float *u_bonus, int32_t *accept_len, int32_t *accept_path,
                          int32_t *bonus_id, void *workspace, size_t workspace_bytes,
                          void *hip_stream) {
  return sparrow_accept_sample_trees(dtype, hidden_rows, lm_head, draft_ids, parent, 0, B, n_q, hidden,
                                     vocab, temperature, u_accept, u_bonus, accept_len, accept_path,
                                     bonus_id, workspace, workspace_bytes, hip_stream);
}

// ------------------------------------------------------------------ dynamic draft tree
static size_t topk_cand_bytes(int M, int k) { return round_up((size_t)M * kStatChunks * k * sizeof(float), 256); }

size_t sparrow_draft_topk_workspace(int32_t dtype, int32_t M, int32_t hidden, int32_t vocab,
                                    int32_t k) {
  if (M <= 0 || hidden <= 0 || vocab <= 0 || k <= 0) return 0;
  size_t lb, sb;
  return sparrow_accept_workspace(dtype, 1, M - 1, hidden, vocab) + accept_sample_extra(M, vocab, &lb, &sb) +
         2 * topk_cand_bytes(M, k);
}

int sparrow_draft_topk(int32_t dtype, const void *hidden_rows, const void *lm_head, int32_t M,
                       int32_t hidden, int32_t vocab, int32_t k, int32_t *ids, float *logp,
                       void *workspace, size_t workspace_bytes, void *hip_stream) {
  g_err[0] = 0;
  if (dtype != SPARROW_F32 && dtype != SPARROW_BF16)
    return fail(SPARROW_ERR_UNSUPPORTED, "dtype %d is neither SPARROW_F32 nor SPARROW_BF16", dtype);
  if (M < 0) return fail(SPARROW_ERR_INVALID_ARG, "M = %d: negative", M);
  if (M == 0) return SPARROW_OK;
  if (M > kAcceptMaxRows) return fail(SPARROW_ERR_UNSUPPORTED, "M = %d rows exceeds %d", M, kAcceptMaxRows);
  if (hidden <= 0 || vocab <= 0) return fail(SPARROW_ERR_INVALID_ARG, "hidden = %d, vocab = %d", hidden, vocab);
  if (k < 1 || k > kTreeMaxWidth || k > vocab)
    return fail(SPARROW_ERR_UNSUPPORTED, "k = %d (supported: 1..%d, at most vocab)", k, kTreeMaxWidth);
  if (vocab > 262144) return fail(SPARROW_ERR_UNSUPPORTED, "vocab = %d exceeds 262144 (top-k)", vocab);
  const int per = dtype == SPARROW_BF16 ? 8 : 4;
  if (hidden % per != 0)
    return fail(SPARROW_ERR_UNSUPPORTED, "hidden = %d must be a multiple of %d (16-byte rows)", hidden, per);
  if (!hidden_rows || !lm_head || !ids || !logp)
    return fail(SPARROW_ERR_INVALID_ARG, "NULL pointer among hidden_rows/lm_head/ids/logp");
  if (!aligned16(hidden_rows) || !aligned16(lm_head))
    return fail(SPARROW_ERR_INVALID_ARG, "hidden_rows and lm_head must be 16-byte aligned");
  const size_t need = sparrow_draft_topk_workspace(dtype, M, hidden, vocab, k);
  if (!workspace || workspace_bytes < need)
    return fail(SPARROW_ERR_WORKSPACE, "workspace of %zu bytes needed, %zu given%s", need,
                workspace_bytes, workspace ? "" : " (NULL)");
  if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0)
    return fail(SPARROW_ERR_INVALID_ARG, "workspace must be 256-byte aligned");
  const bool mfma = lm_head_mfma_supported(dtype, M, hidden, vocab);
  const int n_cand = accept_candidates(dtype, M, hidden, vocab);
  const size_t base = sparrow_accept_workspace(dtype, 1, M - 1, hidden, vocab);
  size_t lb, sb;
  const size_t extra = accept_sample_extra(M, vocab, &lb, &sb);
  char *ws = (char *)workspace;
  AcceptArgs a;
  memset(&a, 0, sizeof(a));
  a.hidden = hidden_rows; a.lm_head = lm_head;
  a.B = 1; a.n_q = M - 1; a.M = M; a.H = hidden; a.V = vocab; a.n_cand = n_cand;
  a.cand_val = (float *)ws;
  a.cand_idx = (int32_t *)(ws + round_up((size_t)M * n_cand * sizeof(float), 256));
  a.logits = (float *)(ws + base);
  hipStream_t st = (hipStream_t)hip_stream;
  hipError_t e = mfma ? launch_lm_head_mfma(a, st) : launch_lm_head_generic(dtype, a, st);
  if (e != hipSuccess) return fail(SPARROW_ERR_DEVICE, "lm_head launch: %s", hipGetErrorString(e));
  TopkArgs t;
  t.logits = a.logits; t.stats = (float *)(ws + base + lb);      // written by the chunk kernel
  t.cand_val = (float *)(ws + base + extra);
  t.cand_idx = (int32_t *)(ws + base + extra + topk_cand_bytes(M, k));
  t.ids = ids; t.logp = logp; t.M = M; t.V = vocab; t.k = k;
  e = launch_topk(t, st);
  if (e != hipSuccess) return fail(SPARROW_ERR_DEVICE, "top-k launch: %s", hipGetErrorString(e));
  return SPARROW_OK;
}

int sparrow_tree_expand(int32_t n_front, int32_t width, const int32_t *front_in,
                        const int32_t *cand_ids, const float *cand_logp, int32_t *pool_tok,
                        int32_t *pool_par, float *pool_score, int32_t n_pool, int32_t *front_out,
                        void *hip_stream) {
  g_err[0] = 0;
  if (width < 1 || width > kTreeMaxWidth || n_front < 1 || n_front > kTreeMaxWidth)
    return fail(SPARROW_ERR_UNSUPPORTED, "width = %d, n_front = %d (supported: 1..%d each)", width, n_front, kTreeMaxWidth);
  if (n_pool < 0 || n_pool + n_front * width > kTreeMaxPool)
    return fail(SPARROW_ERR_UNSUPPORTED, "pool of %d + %d entries exceeds %d", n_pool, n_front * width, kTreeMaxPool);
  if (!cand_ids || !cand_logp || !pool_tok || !pool_par || !pool_score || !front_out)
    return fail(SPARROW_ERR_INVALID_ARG, "NULL pointer among the candidate / pool / frontier arrays");
  if (!front_in && (n_front != 1 || n_pool != 0))
    return fail(SPARROW_ERR_INVALID_ARG, "front_in may only be NULL at level 0 (n_front = 1, n_pool = 0)");
  ExpandArgs a;
  a.front_in = front_in; a.cand_ids = cand_ids; a.cand_logp = cand_logp;
  a.pool_tok = pool_tok; a.pool_par = pool_par; a.pool_score = pool_score; a.front_out = front_out;
  a.n_front = n_front; a.width = width; a.n_pool = n_pool;
  const hipError_t e = launch_tree_expand(a, (hipStream_t)hip_stream);
  if (e != hipSuccess) return fail(SPARROW_ERR_DEVICE, "tree expand launch: %s", hipGetErrorString(e));
  return SPARROW_OK;
}

int sparrow_tree_select(const int32_t *pool_tok, const int32_t *pool_par, const float *pool_score,
                        int32_t n_pool, int32_t total, int32_t *parent, int32_t *ids,
                        int32_t *pool_index, void *hip_stream) {
  g_err[0] = 0;
  if (n_pool < 0 || n_pool > kTreeMaxPool) return fail(SPARROW_ERR_UNSUPPORTED, "n_pool = %d (0..%d)", n_pool, kTreeMaxPool);
  if (total < 0 || total > SPARROW_MAX_NQ) return fail(SPARROW_ERR_UNSUPPORTED, "total = %d (0..%d)", total, SPARROW_MAX_NQ);
  if (n_pool == 0 || total == 0) return SPARROW_OK;
  if (!pool_tok || !pool_par || !pool_score || !parent || !ids || !pool_index)
    return fail(SPARROW_ERR_INVALID_ARG, "NULL pointer among the pool / output arrays");
  SelectArgs a;
  a.pool_tok = pool_tok; a.pool_par = pool_par; a.pool_score = pool_score;
  a.parent = parent; a.ids = ids; a.pool_index = pool_index; a.n_pool = n_pool; a.total = total;
  const hipError_t e = launch_tree_select(a, (hipStream_t)hip_stream);
  if (e != hipSuccess) return fail(SPARROW_ERR_DEVICE, "tree select launch: %s", hipGetErrorString(e));
  return SPARROW_OK;
}

}  // extern "C"
