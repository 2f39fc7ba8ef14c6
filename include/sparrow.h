/*
 * sparrow.h — C ABI of the MI355X (gfx950) hot path of one Sparrow
 * speculative-decoding step for video LLMs:
 *
 *   sparrow_draft_window_attn   draft model's text-anchored window attention
 *   sparrow_verify_attn         target model's verification attention
 *   sparrow_accept              lm_head GEMM -> per-row argmax -> greedy acceptance
 *   sparrow_accept_sample       the same at temperature > 0 (rejection rule + bonus draw)
 *   sparrow_draft_topk / sparrow_tree_expand / sparrow_tree_select   dynamic draft tree
 * and, one step upstream of the draft attention,
 *   sparrow_hsr_fc              draft input by hidden state reuse
 *   sparrow_draft_qkv_append    draft layer norm / QKV / rotary step + K/V append
 * and, one step downstream of the acceptance,
 *   sparrow_kv_commit           accepted K/V rows moved behind the context, next hidden row
 *
 * C99, no C++ or HIP types.  "dev" pointers are device (HBM) addresses, "host"
 * pointers are ordinary host memory.
 *
 * Common rules
 *  - Ownership: the caller owns every buffer, the workspace included.  The
 *    library never allocates or frees device memory and keeps no pointer
 *    after a call returns.
 *  - Asynchrony: a call validates its scalar and host arguments, enqueues its
 *    kernels on `hip_stream` (a hipStream_t passed as void*, NULL = the default
 *    stream) and returns without synchronising.  Host arrays are fully read
 *    before the call returns.  Device buffers must stay valid until the
 *    stream has passed the enqueued work.  Calls are graph-capturable; the
 *    first call of an entry point in a process may do one-time set-up of its
 *    kernels (raising their LDS limit), so make one call outside capture first.
 *  - Errors: every entry point returns a sparrow_status (0 = ok, negative =
 *    error) and sparrow_last_error() describes the reason.  On a validation
 *    error (INVALID_ARG, UNSUPPORTED, WORKSPACE) nothing has been enqueued;
 *    SPARROW_ERR_DEVICE means the HIP runtime refused a launch, and earlier
 *    kernels of the same call may already be enqueued (the outputs are then
 *    unspecified).  Contents of device arrays (text_idx ascending and
 *    in range, parent[i] in [-1, i)) are preconditions that cannot be checked
 *    without a device read; violating them gives undefined results but never
 *    an out-of-bounds access as long as indices stay inside the sequence.
 *  - Types: SPARROW_F32 tensors hold IEEE float, SPARROW_BF16 tensors hold
 *    bfloat16; all arithmetic accumulates in fp32.  Device pointers must be
 *    16-byte aligned, head_dim is innermost and contiguous.
 *  - Query head h reads KV head h / (n_q_heads / n_kv_heads).
 */
#ifndef SPARROW_H
#define SPARROW_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  SPARROW_OK = 0,
  SPARROW_ERR_INVALID_ARG = -1,  /* NULL pointer, bad size, misaligned pointer, bad host array */
  SPARROW_ERR_UNSUPPORTED = -2,  /* dtype / head_dim / size outside what the kernels cover */
  SPARROW_ERR_WORKSPACE = -3,    /* workspace NULL or smaller than the *_workspace() query */
  SPARROW_ERR_DEVICE = -4        /* the HIP runtime refused a launch */
} sparrow_status;

typedef enum { SPARROW_F32 = 0, SPARROW_BF16 = 1 } sparrow_dtype;

/* Limits (SPARROW_ERR_UNSUPPORTED beyond them). */
#define SPARROW_MAX_BATCH 64   /* sequences per call */
#define SPARROW_MAX_NQ 64      /* draft rows (chain length or tree nodes) per sequence */
#define SPARROW_MAX_ACCEPT_ROWS 512   /* logit rows B*(n_q+1) of one acceptance call */

/* Shared by both attention calls. */
typedef struct {
  int32_t dtype;        /* sparrow_dtype of q, k, v and out */
  int32_t n_q_heads;    /* Hq */
  int32_t n_kv_heads;   /* Hkv, divides Hq */
  int32_t head_dim;     /* d: 64 or 128 */
  float scale;          /* softmax scale; 0 selects 1/sqrt(head_dim), the per-head reading of
                           the "d" of Eq. 2 */
  int64_t kv_stride_token; /* elements between consecutive tokens of k (and of v) */
  int64_t kv_stride_head;  /* elements between consecutive KV heads of one token.  Two layouts:
                              token-major [T, Hkv, d] (stride_token >= n_kv_heads*stride_head) or
                              head-major [Hkv, T, d] (stride_head >= stride_token; that
                              stride_head spans all T tokens is the caller's precondition).
                              Head-major lets a workgroup stream one contiguous range per KV
                              head and measures ~4 % faster on the verification attention. */
  int32_t parent_stride;   /* sparrow_verify_attn only: 0 = `parent` holds one tree [n_q] shared by
                              all sequences of the call; >= n_q = every sequence has a tree of its
                              own (dynamic draft trees differ between requests), sequence b's
                              parents at parent[b*parent_stride + i].  Ignored if parent is NULL. */
} sparrow_attn_desc;

/*
 * Draft model's visually-aware text-anchored window attention (Section
 * "Visually-Aware Text-Anchored Window Attention via Hidden State Reuse",
 * Eq. 2): for every sequence b and query head h,
 *     out[b,h,:] = softmax(scale * q[b,h,:] . K_T^T) V_T
 * where T is the set of the min(window, n_text_b) most recent text positions
 * of sequence b.  Keys and values at visual positions are never addressed: the
 * kernel walks `text_idx`, the precomputed position-type index.
 *
 *  q          dev [B, Hq, d]      the one draft query of each sequence
 *  k, v       dev                 draft-layer K/V indexed by absolute position; token t of
 *                                 sequence b, head c starts at element
 *                                 (cu_seqlens[b] + t)*kv_stride_token + c*kv_stride_head
 *  cu_seqlens host int32 [B+1]    token offset of every sequence in k/v (ascending)
 *  text_idx   dev  int32          ascending sequence-local text positions, sequences packed
 *  cu_text    host int32 [B+1]    offsets into text_idx; every sequence needs >= 1 text position
 *                                 (the query's own position is the last one)
 *  window     > 0                 clamped to the sequence's number of text positions
 *  out        dev [B, Hq, d]      same dtype as q
 *  lse        dev float [B, Hq]   natural-log sum-exp of the scaled scores, or NULL
 *  workspace  unused by this call (size query returns 0); may be NULL
 */
size_t sparrow_draft_window_attn_workspace(const sparrow_attn_desc *desc, int32_t B,
                                           int32_t window);
int sparrow_draft_window_attn(const sparrow_attn_desc *desc, const void *q, const void *k,
                              const void *v, const int32_t *cu_seqlens, const int32_t *text_idx,
                              const int32_t *cu_text, int32_t B, int32_t window, void *out,
                              float *lse, void *workspace, size_t workspace_bytes,
                              void *hip_stream);

/*
 * Target model's verification attention (the "parallel verification by the
 * target model" of the draft-then-verify loop, Introduction; dynamic draft
 * trees, Experiment section): n_q draft rows per sequence are scored in one
 * pass against the sequence's whole KV cache.  Row i of sequence b attends to
 * all L_b context tokens and, among the n_q draft tokens, to itself and its
 * ancestors in the draft tree.
 *
 *  q          dev [B*n_q, Hq, d]
 *  k, v       dev               per sequence: L_b context rows followed by its n_q draft rows
 *  cu_seqlens host int32 [B+1]  sequence b owns rows cu_seqlens[b] .. cu_seqlens[b+1]-1
 *                               (= L_b + n_q rows, L_b >= 0)
 *  parent     dev int32 [n_q]   tree shared by all sequences: parent[i] in [-1, i), -1 = child of
 *                               the last accepted token; NULL = chain (parent[i] = i-1).  With
 *                               desc->parent_stride >= n_q: one tree per sequence, [B, parent_stride]
 *  out        dev [B*n_q, Hq, d]
 *  lse        dev float [B*n_q, Hq] or NULL
 *  workspace  dev, at least sparrow_verify_attn_workspace() bytes, 256-byte aligned; holds the
 *             per-split partial results in a format internal to the library
 *  total_tokens = cu_seqlens[B] - cu_seqlens[0], the rows of the call's sequences
 *  B = 0 or n_q = 0: SPARROW_OK and nothing is enqueued.
 */
size_t sparrow_verify_attn_workspace(const sparrow_attn_desc *desc, int32_t B, int32_t n_q,
                                     int64_t total_tokens);
int sparrow_verify_attn(const sparrow_attn_desc *desc, const void *q, const void *k,
                        const void *v, const int32_t *cu_seqlens, const int32_t *parent,
                        int32_t B, int32_t n_q, void *out, float *lse, void *workspace,
                        size_t workspace_bytes, void *hip_stream);

/*
 * Profiling hook: sparrow_verify_attn with only some of its passes enqueued.  `passes` is a bit
 * set: 1 = the split-context partial pass (reads q/k/v, writes the workspace), 2 = the combine
 * pass (reads the workspace, writes out/lse); 3 is sparrow_verify_attn itself.  Arguments,
 * validation and errors are those of sparrow_verify_attn; `out` is only written by pass 2 and
 * is only meaningful if the workspace holds the partials of a matching pass 1.
 */
int sparrow_verify_attn_passes(const sparrow_attn_desc *desc, const void *q, const void *k,
                               const void *v, const int32_t *cu_seqlens, const int32_t *parent,
                               int32_t B, int32_t n_q, void *out, float *lse, void *workspace,
                               size_t workspace_bytes, void *hip_stream, int32_t passes);

/*
 * sparrow_verify_attn for callers that cannot allocate device memory or hand over a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, validation, kernels and results as sparrow_verify_attn, minus the workspace: the
 * split partials go to a scratch array of SPARROW_STATIC_WS_BYTES that is part of the library's
 * device code (one copy per GPU, held until the process ends).  The call allocates and frees
 * nothing.  The device that owns hip_stream and the buffers must be the current device.
 *  - A call whose partials need more than SPARROW_STATIC_WS_BYTES returns
 *    SPARROW_ERR_UNSUPPORTED and enqueues nothing (the message states the size; use
 *    sparrow_verify_attn with a caller workspace).  Every configuration of the benchmark fits:
 *    one 26k-token layer with a chain of 8 takes 4.3 MB, with a 60-node tree 7.7 MB, the ragged
 *    batch of 8 takes 4.9 MB.
 *  - All calls on one GPU share that GPU's array: calls that may overlap in time (different
 *    streams, different host threads with different streams) race on it; calls on one stream
 *    are ordered and safe.  Nothing in the array has to start at zero (the combine pass only
 *    reads what the partial pass of the same call wrote), so no clearing is enqueued.
 *  - The first call on a GPU looks the array's device address up (and may load the library's
 *    code object onto that GPU): make it outside graph capture.
 */
#define SPARROW_STATIC_WS_BYTES (16u * 1024u * 1024u)
int sparrow_verify_attn_static(const sparrow_attn_desc *desc, const void *q, const void *k,
                               const void *v, const int32_t *cu_seqlens, const int32_t *parent,
                               int32_t B, int32_t n_q, void *out, float *lse, void *hip_stream);

/*
 * Greedy (temperature 0, lossless) acceptance: logits = hidden_rows . lm_head^T,
 * target token of every row = lowest index attaining the row maximum, then the
 * longest accepted path: starting at the last accepted token (row 0), move to
 * the lowest-numbered child whose drafted token equals the target token of the
 * current row, until no child matches.  Tokens generated by the step =
 * accept_len + 1 (the bonus token), the paper's average accepted length.
 *
 *  hidden_rows dev [B*(n_q+1), hidden]  row 0 of a sequence = last accepted token, row 1+i =
 *                                       draft node i; final norm already applied
 *  lm_head     dev [vocab, hidden]      row-major, no bias
 *  draft_ids   dev int32 [B*n_q]
 *  parent      dev int32 [n_q] or NULL (chain)
 *  target_ids  dev int32 out [B*(n_q+1)]
 *  accept_len  dev int32 out [B]        in [0, tree depth]
 *  accept_path dev int32 out [B*n_q]    accepted node indices root-first, -1 padded
 *  bonus_id    dev int32 out [B]        target token at the last accepted row
 *  workspace   dev, at least sparrow_accept_workspace() bytes (per-tile argmax candidates)
 *  Limits: B*(n_q+1) <= SPARROW_MAX_ACCEPT_ROWS logit rows (the weights are streamed once per 64
 *  rows).  n_q = 0 is allowed (plain greedy decode of row 0).
 * sparrow_accept_trees: the same with one draft tree per sequence (a batch of requests that each
 *  grew a dynamic tree): parent dev int32 [B, parent_stride], parent_stride >= n_q (0 = the shared
 *  [n_q] form of sparrow_accept).
 */
size_t sparrow_accept_workspace(int32_t dtype, int32_t B, int32_t n_q, int32_t hidden,
                                int32_t vocab);
int sparrow_accept(int32_t dtype, const void *hidden_rows, const void *lm_head,
                   const int32_t *draft_ids, const int32_t *parent, int32_t B, int32_t n_q,
                   int32_t hidden, int32_t vocab, int32_t *target_ids, int32_t *accept_len,
                   int32_t *accept_path, int32_t *bonus_id, void *workspace,
                   size_t workspace_bytes, void *hip_stream);
int sparrow_accept_trees(int32_t dtype, const void *hidden_rows, const void *lm_head,
                         const int32_t *draft_ids, const int32_t *parent, int32_t parent_stride,
                         int32_t B, int32_t n_q, int32_t hidden, int32_t vocab, int32_t *target_ids,
                         int32_t *accept_len, int32_t *accept_path, int32_t *bonus_id,
                         void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Stochastic acceptance at temperature > 0, lossless (the paper's "Temp = 1"
 * regime; it relies on the distribution guarantee of speculative sampling,
 * Related Work, and does not restate the rule).  Rule implemented: recursive
 * rejection over the children of the current tree node, for draft trees whose
 * nodes are chosen deterministically (dynamic top-k trees, Experiment
 * section), i.e. a draft that proposes each child with certainty.  With
 * p = softmax(logits / temperature) of the current node's row and S = 1:
 * children are tried in increasing node index; child j with token x is
 * accepted if u_accept[b][j] * S <= p[x]; otherwise x is struck out (S -= p[x],
 * p[x] = 0; a later child with a struck-out token is skipped).  The accepted
 * child becomes the current node.  When no child is accepted, or at a leaf,
 * the bonus token is drawn from what is left of p by inverse CDF in
 * vocabulary order: bonus = min { t : sum_{v<=t} p[v] >= u_bonus[b] * S }.
 * The first token emitted by a step is then distributed exactly as p.
 *
 *  Arguments as sparrow_accept (logits = hidden_rows . lm_head^T), plus
 *  temperature > 0
 *  u_accept    dev float [B, n_q]   uniforms in [0, 1) supplied by the caller, one per node
 *  u_bonus     dev float [B]
 *  accept_len, accept_path, bonus_id   as sparrow_accept (no target_ids: there is no single
 *                                       target token per row)
 *  workspace   dev, at least sparrow_accept_sample_workspace() bytes, 256-byte aligned (argmax
 *              candidates, the B*(n_q+1) x vocab fp32 logits, per-row softmax statistics)
 *  All arithmetic of the rule is fp32 (exp2 of pre-scaled logits); a decision closer to its
 *  threshold than ~1e-5 of the row's mass may differ from exact arithmetic.
 */
size_t sparrow_accept_sample_workspace(int32_t dtype, int32_t B, int32_t n_q, int32_t hidden,
                                       int32_t vocab);
int sparrow_accept_sample(int32_t dtype, const void *hidden_rows, const void *lm_head,
                          const int32_t *draft_ids, const int32_t *parent, int32_t B, int32_t n_q,
                          int32_t hidden, int32_t vocab, float temperature, const float *u_accept,
                          const float *u_bonus, int32_t *accept_len, int32_t *accept_path,
                          int32_t *bonus_id, void *workspace, size_t workspace_bytes,
                          void *hip_stream);
/* The same with one draft tree per sequence: parent dev int32 [B, parent_stride] (see
 * sparrow_accept_trees). */
int sparrow_accept_sample_trees(int32_t dtype, const void *hidden_rows, const void *lm_head,
                                const int32_t *draft_ids, const int32_t *parent,
                                int32_t parent_stride, int32_t B, int32_t n_q, int32_t hidden,
                                int32_t vocab, float temperature, const float *u_accept,
                                const float *u_bonus, int32_t *accept_len, int32_t *accept_path,
                                int32_t *bonus_id, void *workspace, size_t workspace_bytes,
                                void *hip_stream);

/*
 * Stochastic acceptance against a SAMPLED draft, and with uniforms generated by the library:
 * the speculative-sampling rule behind the paper's losslessness at temperature > 0 (Related
 * Work: speculative sampling's distribution guarantee; "Temp = 1" blocks of the result tables)
 * for a draft that draws its proposals from a distribution q instead of proposing them with
 * certainty.  draft_probs holds, for every logit row r, the distribution the tokens of row r's
 * children were drawn from (independently, if there are several).  With p = softmax(logits /
 * temperature) of the current row, residual R = p and S = 1: child j with token x is accepted if
 * R[x] > 0 and u_accept[b][j] * q[x] * S <= R[x], i.e. with probability min(1, (R[x]/S) / q[x]);
 * on a rejection R[v] <- max(R[v] - S q[v], 0) for all v and S <- sum R (the normalised
 * max(p - q, 0)); the accepted child becomes the current node; when no child is accepted, or at
 * a leaf, bonus = min { t : sum_{v<=t} R[v] >= u_bonus[b] * S }.  The first emitted token is
 * then distributed exactly as p.
 *
 *  draft_probs dev float [B*(n_q+1), vocab], 16-byte aligned, rows of leaves are not read;
 *              NULL = the deterministic-children rule of sparrow_accept_sample
 *  u_accept, u_bonus   both dev as in sparrow_accept_sample, or both NULL: the uniforms are then
 *              generated by Philox4x32-10 (Salmon et al., SC'11) under the key (seed low word,
 *              seed high word): node j of sequence b takes the first output word of the counter
 *              (offset low, offset high, b, j), the bonus draw that of (offset low, offset high,
 *              b, 0xFFFFFFFF); uniform = (word >> 8) * 2^-24.  A caller advances `offset` by one
 *              per step, so no step reuses a number.
 *  parent, parent_stride   as sparrow_accept_trees;  workspace: sparrow_accept_sample_workspace()
 *  A rejection costs one pass of one workgroup over the row's logits and draft probabilities.
 */
int sparrow_accept_sample_q(int32_t dtype, const void *hidden_rows, const void *lm_head,
                            const int32_t *draft_ids, const int32_t *parent, int32_t parent_stride,
                            int32_t B, int32_t n_q, int32_t hidden, int32_t vocab, float temperature,
                            const float *draft_probs, const float *u_accept, const float *u_bonus,
                            uint64_t seed, uint64_t offset, int32_t *accept_len,
                            int32_t *accept_path, int32_t *bonus_id, void *workspace,
                            size_t workspace_bytes, void *hip_stream);

/*
 * Dynamic draft tree (Experiment section: dynamic tree structure with the
 * configuration "total tokens - depth - width", e.g. 30-4-8; the procedure is
 * not printed, the best-first expansion of the tree-speculation work the paper
 * builds on is implemented).  A node's score is the sum of the draft's
 * log-probabilities along its path.  Level 0: the `width` most likely tokens
 * after the root.  Level d: every frontier node proposes its `width` most
 * likely next tokens; all candidates join the pool, the `width` best of them
 * form the next frontier.  At the end the `total` best pool nodes are kept
 * (closed under ancestors, because log-probabilities are <= 0) and renumbered
 * in pool order, which gives parent[i] < i as sparrow_verify_attn expects.
 * "Better" is everywhere: higher value, then lower index / token id.
 * The draft's forward pass between two levels is the caller's.
 *
 * sparrow_draft_topk: logits = hidden_rows . lm_head^T; per row the k largest
 *   logits in decreasing order with their natural-log softmax values.
 *   hidden_rows dev [M, hidden], lm_head dev [vocab, hidden]; ids dev int32 out [M, k];
 *   logp dev float out [M, k]; workspace dev >= sparrow_draft_topk_workspace() bytes, 256-byte
 *   aligned.  Limits: M <= SPARROW_MAX_ACCEPT_ROWS, 1 <= k <= 16, k <= vocab <= 262,144.
 * sparrow_tree_expand: one level.  front_in dev int32 [n_front] pool indices of the frontier (NULL
 *   at level 0: the root, n_front = 1); cand_ids dev int32 / cand_logp dev float [n_front, width]
 *   (rows of sparrow_draft_topk for the frontier nodes); the candidates are appended to the pool
 *   arrays (pool_tok, pool_par dev int32, pool_score dev float, each with room for n_pool +
 *   n_front*width entries) at n_pool in (frontier, candidate) order; front_out dev int32 [width]
 *   receives the pool indices of the next frontier, best first (width <= n_front*width).
 *   Limits: width, n_front <= 16; pool size <= 2048.
 * sparrow_tree_select: keeps the min(total, n_pool) best nodes: parent, ids, pool_index dev int32
 *   out, one entry per kept node in pool order.  Limits: total <= 64, n_pool <= 2048.
 */
size_t sparrow_draft_topk_workspace(int32_t dtype, int32_t M, int32_t hidden, int32_t vocab,
                                    int32_t k);
int sparrow_draft_topk(int32_t dtype, const void *hidden_rows, const void *lm_head, int32_t M,
                       int32_t hidden, int32_t vocab, int32_t k, int32_t *ids, float *logp,
                       void *workspace, size_t workspace_bytes, void *hip_stream);
int sparrow_tree_expand(int32_t n_front, int32_t width, const int32_t *front_in,
                        const int32_t *cand_ids, const float *cand_logp, int32_t *pool_tok,
                        int32_t *pool_par, float *pool_score, int32_t n_pool, int32_t *front_out,
                        void *hip_stream);
int sparrow_tree_select(const int32_t *pool_tok, const int32_t *pool_par, const float *pool_score,
                        int32_t n_pool, int32_t total, int32_t *parent, int32_t *ids,
                        int32_t *pool_index, void *hip_stream);

/*
 * Input of the draft model by hidden state reuse (Section "Visually-Aware
 * Text-Anchored Window Attention via Hidden State Reuse", Eq. 1): for each of
 * the M new tokens
 *     z[m,:] = W_fc . concat(embed[token_ids[m],:], h_prev[m,:]) + b_fc
 * i.e. the projection, back to the model width, of the token's embedding
 * joined with the target model's hidden state of the previous step (which
 * carries the visual context, so the draft never reads a visual token).
 *
 *  dtype      sparrow_dtype of embed, h_prev, w_fc, b_fc and z
 *  embed      dev [vocab, hidden]
 *  token_ids  dev int32 [M], values in [0, vocab) (out-of-range ids are clamped into the table)
 *  h_prev     dev [M, hidden]
 *  w_fc       dev [hidden, 2*hidden] row-major: columns 0..hidden-1 meet the embedding,
 *             columns hidden..2*hidden-1 the hidden state
 *  b_fc       dev [hidden] or NULL
 *  z          dev out [M, hidden]
 *  Limits: M <= 64, hidden a multiple of 8.  M = 0: SPARROW_OK, nothing enqueued.
 */
int sparrow_hsr_fc(int32_t dtype, const void *embed, const int32_t *token_ids, const void *h_prev,
                   const void *w_fc, const void *b_fc, int32_t M, int32_t hidden, int32_t vocab,
                   void *z, void *hip_stream);

/*
 * Input side of the draft's decoder layer for the M new tokens, producing
 * what sparrow_draft_window_attn reads.  The paper gives no formula for the
 * draft layer itself; it has the target's layer architecture, here the Qwen2
 * family's: RMSNorm, a QKV projection with bias, rotate-half rotary embedding.
 *     u = z / sqrt(mean(z^2) + eps) * norm_weight
 *     y = W_qkv u + b_qkv          rows of W_qkv: Hq query heads, Hkv key heads, Hkv value heads
 *     q, k rotated per head:  out[i] = x[i] cos[i] - x[i+d/2] sin[i],
 *                             out[i+d/2] = x[i+d/2] cos[i] + x[i] sin[i]        (i < d/2)
 * q goes to q_out; k and v of token m are written to row kv_rows[m] of the
 * draft K/V cache (the append at the token's position).
 *
 *  desc        dtype of z, norm_weight, w_qkv, b_qkv, q_out and the cache; heads, head_dim and
 *              the cache strides (scale is ignored)
 *  z           dev [M, hidden]
 *  norm_weight dev [hidden]
 *  w_qkv       dev [(Hq + 2*Hkv)*d, hidden] row-major;  b_qkv dev [(Hq + 2*Hkv)*d] or NULL
 *  rope_cos, rope_sin  dev float [M, d/2]: the rotary table rows of the tokens' positions
 *                      (the caller owns the table; the library does not evaluate angles)
 *  kv_rows     host int32 [M]: cache row of token m (cu_seqlens[b] + position), all distinct and
 *              >= 0 (checked); that they lie inside the caches is the caller's precondition
 *  q_out       dev out [M, Hq, d]
 *  k_cache, v_cache  dev; row r, head c starts at element r*kv_stride_token + c*kv_stride_head
 *  Limits: M <= 64, hidden a multiple of 8.  M = 0: SPARROW_OK, nothing enqueued.
 */
int sparrow_draft_qkv_append(const sparrow_attn_desc *desc, const void *z, const void *norm_weight,
                             float eps, const void *w_qkv, const void *b_qkv,
                             const float *rope_cos, const float *rope_sin,
                             const int32_t *kv_rows, int32_t M, int32_t hidden, void *q_out,
                             void *k_cache, void *v_cache, void *hip_stream);

/*
 * Post-accept commit, the step after sparrow_accept (the paper leaves its
 * mechanics open; it follows from verifying a draft tree against one KV cache
 * and from reusing the target's hidden state, Eq. 1): in every layer, the K/V
 * rows of the accepted draft nodes are moved up behind the context in path
 * order, so that the sequence's cache is contiguous again,
 *     row L_b + j  <-  row L_b + accept_path[b][j]     for j < accept_len[b],
 * and the hidden row of the last accepted node (row 0 of the sequence if none
 * was accepted) is copied out as the draft's next h.
 *
 *  desc        dtype, n_kv_heads, head_dim and the strides of every layer's K and V
 *  k_layers, v_layers  host arrays [n_layers] of device pointers, the layout of sparrow_verify_attn
 *  cu_seqlens  host int32 [B+1]: sequence b owns L_b context rows followed by n_q draft rows
 *  accept_path dev int32 [B, n_q], accept_len dev int32 [B]: as written by sparrow_accept
 *              (entries are clamped into [0, n_q) before use)
 *  hidden_rows dev [B*(n_q+1), hidden] or NULL; next_hidden dev out [B, hidden] (required if
 *              hidden_rows is given); hidden*element size a multiple of 16 bytes
 *  Limits: n_layers <= 64, B <= 64, n_q <= 64.  B = 0 or n_layers = 0 with no hidden_rows: no-op.
 *  The new sequence lengths (L_b + accept_len[b]) are the caller's bookkeeping.
 */
int sparrow_kv_commit(const sparrow_attn_desc *desc, void *const *k_layers, void *const *v_layers,
                      int32_t n_layers, const int32_t *cu_seqlens, int32_t B, int32_t n_q,
                      const int32_t *accept_path, const int32_t *accept_len,
                      const void *hidden_rows, int32_t hidden, void *next_hidden,
                      void *hip_stream);

/*
 * Measurement aid (no part of the method): enqueues a kernel that reads `bytes` bytes at `dev_ptr`
 * once, with the same 16-byte non-temporal loads the attention kernels use, and does nothing
 * else; bench.py times it on a layer's K and V to show what moving those bytes costs on the
 * device at hand.  dev_ptr 16-byte aligned, bytes a multiple of 16; sink dev, 4 bytes, may be
 * written.  sparrow_stream_read_shape chooses the launch: `workgroups` of 256 lanes (1..65536),
 * `loads_in_flight` per lane (2, 4, 8 or 16), and `regions` = 0 (the grid sweeps the range front
 * to back) or 1 (every workgroup reads one contiguous region of its own); sparrow_stream_read is
 * the shape (1024, 8, 0).
 */
int sparrow_stream_read(const void *dev_ptr, size_t bytes, void *sink, void *hip_stream);
int sparrow_stream_read_shape(const void *dev_ptr, size_t bytes, void *sink, int32_t workgroups,
                              int32_t loads_in_flight, int32_t regions, void *hip_stream);

/*
 * Debug aids: synchronous checks of the device-resident preconditions that the entry points
 * above cannot check without a device read.  The arrays may live in device memory (they are
 * copied to the host on hip_stream, which is synchronised) or in ordinary host memory (read in
 * place; this also works on a machine without a GPU).  SPARROW_OK, or SPARROW_ERR_INVALID_ARG with
 * sparrow_last_error() naming the first offending entry.  Not for the hot path.
 *
 * sparrow_debug_validate_parent: every tree satisfies parent[i] in [-1, i) (nodes numbered so
 *   that a parent precedes its children; the ancestor walks of sparrow_verify_attn and the
 *   acceptance walks then terminate).  parent [n_q] with parent_stride 0 (B is ignored), or
 *   [B, parent_stride] with parent_stride >= n_q.
 * sparrow_debug_validate_text_idx: for every sequence b, text_idx[cu_text[b] .. cu_text[b+1]) is
 *   strictly ascending and inside [0, cu_seqlens[b+1] - cu_seqlens[b]), and holds at least one
 *   entry.  cu_seqlens, cu_text: host int32 [B+1].
 */
int sparrow_debug_validate_parent(const int32_t *parent, int32_t parent_stride, int32_t B,
                                  int32_t n_q, void *hip_stream);
int sparrow_debug_validate_text_idx(const int32_t *text_idx, const int32_t *cu_seqlens,
                                    const int32_t *cu_text, int32_t B, void *hip_stream);

/* Thread-local description of the last error on this thread; "" if none. */
const char *sparrow_last_error(void);

/* Library version, "major.minor". */
const char *sparrow_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SPARROW_H */
