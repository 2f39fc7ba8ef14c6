/*
 * CPU oracle for the Sparrow speculative-decoding hot path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, fp64 statement of
 * what the path computes, written from the paper's definitions.  It shares no
 * code with the HIP library and is never used by it; only the tests, the
 * smoke check and the benchmark's cpu_baseline leg call it.
 *
 * All results here have a plain mathematical definition that the GPU kernels
 * merely reach by another order of operations (online softmax, split context,
 * matrix-core tiles), so every function below is that definition written out:
 * two-pass softmax, no tiling, no splitting, no reordering.  The only
 * concession to run time is an OpenMP "parallel for" over independent output
 * rows.
 *
 * Pins (tests/test_oracle_*.py): torch's CPU fp64 scaled_dot_product_attention
 * with an explicit dense mask, scipy's softmax/logsumexp, numpy matmul+argmax,
 * closed forms (constant V, zero K, one dominant key), invariants (all-text
 * window == causal decode, n_q = 1 == decode, chain-shaped tree == chain,
 * per-path decomposition of a tree, row permutation, GQA == replicated MHA),
 * and brute-force enumeration of small acceptance problems; for the draft's
 * input side (tests/test_oracle_hsr.py) numpy matmul on the concatenated
 * input, the Qwen2 RMSNorm / rotary-embedding modules of the transformers
 * package run in float64, and the rotation invariants of the rotary embedding.
 * Nothing numeric is printed in the paper for these steps, so no golden value
 * from the paper exists; end-to-end accepted-length tables are out of reach
 * (trained weights and videos are not available).
 *
 * Layout conventions (all row-major, doubles):
 *   q   [rows, Hq, d]
 *   K,V token t, kv head c, element x at  t*stride_tok + c*stride_head + x
 *   out [rows, Hq, d], lse [rows, Hq]
 * Query head h reads kv head h / (Hq/Hkv)  (contiguous groups).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* Softmax attention of one query vector over an explicit list of key rows:
 *   s_j = scale * <q, K[tok_j]>,  p = softmax(s),  o = sum_j p_j V[tok_j]
 * (Eq. 2 with the key set given by `tok`).  Also returns log(sum exp s). */
static void attend_list(const double *q, const double *K, const double *V,
                        const int64_t *tok, int n, int d, double scale,
                        int64_t stride_tok, double *o, double *lse, double *s)
{
    double m = -INFINITY;
    for (int j = 0; j < n; ++j) {
        const double *kr = K + tok[j] * stride_tok;
        double acc = 0.0;
        for (int x = 0; x < d; ++x) acc += q[x] * kr[x];
        s[j] = scale * acc;
        if (s[j] > m) m = s[j];
    }
    double l = 0.0;
    for (int j = 0; j < n; ++j) { s[j] = exp(s[j] - m); l += s[j]; }
    for (int x = 0; x < d; ++x) o[x] = 0.0;
    for (int j = 0; j < n; ++j) {
        const double *vr = V + tok[j] * stride_tok;
        double p = s[j] / l;
        for (int x = 0; x < d; ++x) o[x] += p * vr[x];
    }
    if (lse) *lse = m + log(l);
}

/* Draft model's text-anchored window attention (VATA, Eq. 2; "discards the
 * visual KV cache", attention closed within the text domain T).  The window
 * reading: the `window` most recent text positions; window >= |T| gives Eq. 2
 * over all of T.  The query's own position is the last text position. */
int oracle_draft_window_attn(const double *q, const double *K, const double *V,
                             const int32_t *cu_seqlens, const int32_t *text_idx,
                             const int32_t *cu_text, int B, int Hq, int Hkv, int d,
                             double scale, int window,
                             int64_t stride_tok, int64_t stride_head,
                             double *out, double *lse)
{
    if (Hq % Hkv != 0 || window <= 0) return -1;
    const int g = Hq / Hkv;
    for (int b = 0; b < B; ++b)
        if (cu_text[b + 1] - cu_text[b] <= 0) return -1; /* softmax over nothing */
    #pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        for (int h = 0; h < Hq; ++h) {
            const int n_text = cu_text[b + 1] - cu_text[b];
            const int n = n_text < window ? n_text : window;
            const int32_t *idx = text_idx + cu_text[b] + (n_text - n);
            int64_t *tok = (int64_t *)malloc(sizeof(int64_t) * (size_t)n);
            double *s = (double *)malloc(sizeof(double) * (size_t)n);
            for (int j = 0; j < n; ++j) tok[j] = (int64_t)cu_seqlens[b] + idx[j];
            const int c = h / g;
            attend_list(q + ((int64_t)b * Hq + h) * d, K + c * stride_head, V + c * stride_head,
                        tok, n, d, scale, stride_tok,
                        out + ((int64_t)b * Hq + h) * d,
                        lse ? lse + (int64_t)b * Hq + h : NULL, s);
            free(tok); free(s);
        }
    }
    return 0;
}

/* Target's verification attention: n_q draft rows per sequence, each seeing
 * the whole context of its sequence plus, among the draft rows, itself and
 * its ancestors in the draft tree (parent[i] in [-1, i); NULL = chain, i.e.
 * row i sees draft rows 0..i).  Sequence b owns rows cu_seqlens[b] ..
 * cu_seqlens[b+1]-1 of K/V: L_b context rows followed by its n_q draft rows. */
int oracle_verify_attn(const double *q, const double *K, const double *V,
                       const int32_t *cu_seqlens, const int32_t *parent,
                       int B, int n_q, int Hq, int Hkv, int d, double scale,
                       int64_t stride_tok, int64_t stride_head,
                       double *out, double *lse)
{
    if (Hq % Hkv != 0) return -1;
    const int g = Hq / Hkv;
    for (int i = 0; parent && i < n_q; ++i)
        if (parent[i] < -1 || parent[i] >= i) return -1;
    for (int b = 0; b < B; ++b)
        if (cu_seqlens[b + 1] - cu_seqlens[b] < n_q) return -1;
    #pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        for (int i = 0; i < n_q; ++i) {
            const int L = cu_seqlens[b + 1] - cu_seqlens[b] - n_q;
            int64_t *tok = (int64_t *)malloc(sizeof(int64_t) * (size_t)(L + n_q));
            double *s = (double *)malloc(sizeof(double) * (size_t)(L + n_q));
            int n = 0;
            for (int t = 0; t < L; ++t) tok[n++] = (int64_t)cu_seqlens[b] + t;
            if (parent) {
                /* ancestors-or-self, then put them in ascending order */
                int first = n;
                for (int a = i; a >= 0; a = parent[a]) tok[n++] = (int64_t)cu_seqlens[b] + L + a;
                for (int lo = first, hi = n - 1; lo < hi; ++lo, --hi) {
                    int64_t tmp = tok[lo]; tok[lo] = tok[hi]; tok[hi] = tmp;
                }
            } else {
                for (int a = 0; a <= i; ++a) tok[n++] = (int64_t)cu_seqlens[b] + L + a;
            }
            for (int h = 0; h < Hq; ++h) {
                const int c = h / g;
                const int64_t row = (int64_t)b * n_q + i;
                attend_list(q + (row * Hq + h) * d, K + c * stride_head, V + c * stride_head,
                            tok, n, d, scale, stride_tok,
                            out + (row * Hq + h) * d,
                            lse ? lse + row * Hq + h : NULL, s);
            }
            free(tok); free(s);
        }
    }
    return 0;
}

/* lm_head: logits[r, v] = sum_x hidden[r, x] * W[v, x]   (no bias). */
void oracle_logits(const double *hidden, const double *W, int rows, int H, int64_t vocab,
                   double *logits)
{
    #pragma omp parallel for schedule(static)
    for (int64_t v = 0; v < vocab; ++v) {
        const double *w = W + v * H;
        for (int r = 0; r < rows; ++r) {
            const double *hr = hidden + (int64_t)r * H;
            double acc = 0.0;
            for (int x = 0; x < H; ++x) acc += hr[x] * w[x];
            logits[(int64_t)r * vocab + v] = acc;
        }
    }
}

/* Greedy (temperature 0) target token per row: the smallest index attaining
 * the row maximum.  margin[r] = best - second best (0 on an exact tie). */
void oracle_argmax(const double *logits, int rows, int64_t vocab, int32_t *ids, double *margin)
{
    for (int r = 0; r < rows; ++r) {
        const double *lr = logits + (int64_t)r * vocab;
        int64_t best = 0;
        for (int64_t v = 1; v < vocab; ++v) if (lr[v] > lr[best]) best = v;
        double second = -INFINITY;
        for (int64_t v = 0; v < vocab; ++v) if (v != best && lr[v] > second) second = lr[v];
        ids[r] = (int32_t)best;
        if (margin) margin[r] = vocab > 1 ? lr[best] - second : INFINITY;
    }
}

/* Greedy acceptance (lossless at temperature 0): starting from the last
 * accepted token (row 0 of each sequence's n_q+1 rows), repeatedly move to the
 * child whose drafted token equals the target's greedy token at the current
 * row; the lowest-numbered such child wins.  Row 1+i belongs to draft node i.
 * Outputs: accept_len [B], accept_path [B, n_q] (node indices root-first, -1
 * padded), bonus_id [B] = target token at the last accepted row. */
int oracle_accept(const int32_t *target_ids, const int32_t *draft_ids, const int32_t *parent,
                  int B, int n_q, int32_t *accept_len, int32_t *accept_path, int32_t *bonus_id)
{
    for (int i = 0; parent && i < n_q; ++i)
        if (parent[i] < -1 || parent[i] >= i) return -1;
    for (int b = 0; b < B; ++b) {
        const int32_t *t = target_ids + (int64_t)b * (n_q + 1);
        const int32_t *dr = draft_ids + (int64_t)b * n_q;
        int32_t *path = accept_path + (int64_t)b * n_q;
        for (int i = 0; i < n_q; ++i) path[i] = -1;
        int cur = -1, len = 0;
        for (;;) {
            int next = -1;
            for (int j = 0; j < n_q && next < 0; ++j) {
                const int pj = parent ? parent[j] : j - 1;
                if (pj == cur && dr[j] == t[cur + 1]) next = j;
            }
            if (next < 0) break;
            path[len++] = next;
            cur = next;
        }
        accept_len[b] = len;
        bonus_id[b] = t[cur + 1];
    }
    return 0;
}

/* ------------------------------------------------------------------------
 * Draft input side (the step before the draft's window attention).
 * ------------------------------------------------------------------------ */

/* Hidden state reuse (Section "Visually-Aware Text-Anchored Window Attention
 * via Hidden State Reuse", Eq. 1): z_t = FC(e_t (+) h_{t-1}), the projection
 * of the concatenation of the current token's embedding and the target
 * model's hidden state of the previous step back to the model width.
 *   e [M, H] (embedding rows already gathered), h [M, H],
 *   W [H, 2H] row-major (output feature n reads W[n, 0:H] . e + W[n, H:2H] . h),
 *   bias [H] or NULL, z [M, H]. */
void oracle_hsr_fc(const double *e, const double *h, const double *W, const double *bias,
                   int M, int H, double *z)
{
    #pragma omp parallel for schedule(static)
    for (int n = 0; n < H; ++n) {
        const double *w = W + (int64_t)n * 2 * H;
        for (int m = 0; m < M; ++m) {
            double acc = bias ? bias[n] : 0.0;
            for (int x = 0; x < H; ++x) acc += w[x] * e[(int64_t)m * H + x];
            for (int x = 0; x < H; ++x) acc += w[H + x] * h[(int64_t)m * H + x];
            z[(int64_t)m * H + n] = acc;
        }
    }
}

/* Input side of the draft's decoder layer, with the target's layer
 * architecture (the paper builds the draft from the target's layer type and
 * gives no formula of its own; this is the RMSNorm / biased QKV projection /
 * rotate-half rotary embedding of the Qwen2 family):
 *   u = z / sqrt(mean(z^2) + eps) * gamma
 *   y = W u + bias,            W [(Hq + 2 Hkv) d, H], rows ordered q heads, k heads, v heads
 *   rotary embedding on every q and k head with the row's (cos, sin) [d/2]:
 *     out[i]       = x[i] cos[i] - x[i + d/2] sin[i]
 *     out[i + d/2] = x[i + d/2] cos[i] + x[i] sin[i]          (i < d/2)
 * Outputs q [M, Hq, d], k [M, Hkv, d] (rotated), v [M, Hkv, d]. */
void oracle_draft_qkv(const double *z, const double *gamma, double eps, const double *W,
                      const double *bias, const double *rope_cos, const double *rope_sin,
                      int M, int H, int Hq, int Hkv, int d, double *q, double *k, double *v)
{
    const int N = (Hq + 2 * Hkv) * d;
    const int half = d / 2;
    double *u = (double *)malloc(sizeof(double) * (size_t)M * H);
    double *y = (double *)malloc(sizeof(double) * (size_t)M * N);
    for (int m = 0; m < M; ++m) {
        double ss = 0.0;
        for (int x = 0; x < H; ++x) ss += z[(int64_t)m * H + x] * z[(int64_t)m * H + x];
        const double r = 1.0 / sqrt(ss / H + eps);
        for (int x = 0; x < H; ++x) u[(int64_t)m * H + x] = z[(int64_t)m * H + x] * r * gamma[x];
    }
    #pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        const double *w = W + (int64_t)n * H;
        for (int m = 0; m < M; ++m) {
            double acc = bias ? bias[n] : 0.0;
            for (int x = 0; x < H; ++x) acc += w[x] * u[(int64_t)m * H + x];
            y[(int64_t)m * N + n] = acc;
        }
    }
    for (int m = 0; m < M; ++m) {
        const double *cs = rope_cos + (int64_t)m * half, *sn = rope_sin + (int64_t)m * half;
        for (int hd = 0; hd < Hq + 2 * Hkv; ++hd) {
            const double *x = y + (int64_t)m * N + (int64_t)hd * d;
            double *o;
            int rotate = 1;
            if (hd < Hq) o = q + ((int64_t)m * Hq + hd) * d;
            else if (hd < Hq + Hkv) o = k + ((int64_t)m * Hkv + (hd - Hq)) * d;
            else { o = v + ((int64_t)m * Hkv + (hd - Hq - Hkv)) * d; rotate = 0; }
            for (int i = 0; i < half; ++i) {
                if (rotate) {
                    o[i] = x[i] * cs[i] - x[i + half] * sn[i];
                    o[i + half] = x[i + half] * cs[i] + x[i] * sn[i];
                } else {
                    o[i] = x[i];
                    o[i + half] = x[i + half];
                }
            }
        }
    }
    free(u);
    free(y);
}

/* Rotary tables of the rotate-half convention: angle(pos, i) = pos * theta^(-2 i / d), i < d/2. */
void oracle_rope_table(const int32_t *pos, int M, int d, double theta, double *rope_cos,
                       double *rope_sin)
{
    const int half = d / 2;
    for (int m = 0; m < M; ++m)
        for (int i = 0; i < half; ++i) {
            const double ang = (double)pos[m] * pow(theta, -2.0 * i / d);
            rope_cos[(int64_t)m * half + i] = cos(ang);
            rope_sin[(int64_t)m * half + i] = sin(ang);
        }
}

/* ------------------------------------------------------------------------
 * Post-accept commit (the step after greedy acceptance; the paper leaves the
 * mechanics open, it follows from verifying a tree and reusing hidden states):
 * the K/V rows of the accepted draft nodes become the next context rows, in
 * path order, and the hidden state of the last accepted row is handed to the
 * draft model for the next step (the h of Eq. 1).
 *   cache  [T, row_elems] one layer's K or V as doubles; sequence b owns rows
 *          cu[b] .. cu[b+1]-1 = L_b context rows then n_q draft rows
 *   after the call row cu[b] + L_b + j holds what row cu[b] + L_b + path[b][j]
 *   held before it, for j < accept_len[b]; every other row is unchanged.
 * ------------------------------------------------------------------------ */
void oracle_kv_commit(double *cache, int64_t row_elems, const int32_t *cu, int B, int n_q,
                      const int32_t *accept_path, const int32_t *accept_len)
{
    double *tmp = (double *)malloc(sizeof(double) * (size_t)(n_q > 0 ? n_q : 1) * row_elems);
    for (int b = 0; b < B; ++b) {
        const int64_t first = (int64_t)cu[b + 1] - n_q;          /* first draft row */
        const int len = accept_len[b];
        for (int j = 0; j < len; ++j)                            /* read everything first */
            memcpy(tmp + (int64_t)j * row_elems,
                   cache + (first + accept_path[(int64_t)b * n_q + j]) * row_elems,
                   sizeof(double) * row_elems);
        for (int j = 0; j < len; ++j)
            memcpy(cache + (first + j) * row_elems, tmp + (int64_t)j * row_elems,
                   sizeof(double) * row_elems);
    }
    free(tmp);
}

/* Hidden row handed to the draft for the next step: the row of the last accepted node, or row 0
 * of the sequence (the last accepted token of the previous step) if nothing was accepted.
 *   hidden [B*(n_q+1), H], out [B, H] */
void oracle_next_hidden(const double *hidden, int B, int n_q, int H, const int32_t *accept_path,
                        const int32_t *accept_len, double *out)
{
    for (int b = 0; b < B; ++b) {
        const int len = accept_len[b];
        const int row = len > 0 ? 1 + accept_path[(int64_t)b * n_q + len - 1] : 0;
        memcpy(out + (int64_t)b * H, hidden + ((int64_t)b * (n_q + 1) + row) * H, sizeof(double) * H);
    }
}

/* ------------------------------------------------------------------------
 * Stochastic acceptance (temperature > 0), lossless: the paper reports a
 * Temp = 1 regime for its dynamic draft trees and relies on the distribution
 * guarantee of speculative sampling (Related Work, first paragraph) without
 * restating the rule.  Reading taken: the recursive rejection rule of the
 * tree-speculation line of work it builds on, for trees whose nodes are chosen
 * deterministically (top-k), i.e. a draft that proposes each child with
 * certainty:
 *   at the current node, p = softmax(logits / T) of the node's row;
 *   its children are tried in increasing node index; child j with token x
 *   is accepted if  u_accept[j] * S <= p[x],  where S is the probability mass
 *   not yet rejected (1 at first); otherwise x is struck out (S -= p[x],
 *   p[x] = 0) and the next child is tried (a child whose token is already
 *   struck out is skipped);
 *   an accepted child becomes the current node; if no child is accepted (or
 *   the node is a leaf) the step ends with a bonus token drawn from what is
 *   left of p by inverse CDF in vocabulary order:
 *   bonus = min { t : sum_{v <= t} p[v] >= u_bonus * S }.
 * The first token emitted this way is distributed exactly as p.
 *
 * logits [B*(n_q+1), V] (row 0 of a sequence = last accepted token, row 1+i =
 * node i); u_accept [B, n_q], u_bonus [B] uniforms in [0, 1) supplied by the
 * caller.  Outputs as in oracle_accept.  margin (optional, [B]) = the smallest
 * distance of any decision of the walk from its threshold, relative to the
 * threshold's scale: min over tests of |u S - p[x]| / S and, for the bonus, of
 * the distance of u S to the two CDF values around it divided by S.
 * ------------------------------------------------------------------------ */
int oracle_accept_sample(const double *logits, const int32_t *draft_ids, const int32_t *parent,
                         int B, int n_q, int64_t V, double temperature, const double *u_accept,
                         const double *u_bonus, int32_t *accept_len, int32_t *accept_path,
                         int32_t *bonus_id, double *margin)
{
    if (!(temperature > 0.0)) return -2;
    for (int i = 0; parent && i < n_q; ++i)
        if (parent[i] < -1 || parent[i] >= i) return -1;
    double *p = (double *)malloc(sizeof(double) * (size_t)V);
    for (int b = 0; b < B; ++b) {
        const int32_t *dr = draft_ids + (int64_t)b * n_q;
        int32_t *path = accept_path + (int64_t)b * n_q;
        for (int i = 0; i < n_q; ++i) path[i] = -1;
        int cur = -1, len = 0;
        double worst = INFINITY;
        for (;;) {
            const double *lr = logits + ((int64_t)b * (n_q + 1) + cur + 1) * V;
            double mx = -INFINITY, Z = 0.0;
            for (int64_t v = 0; v < V; ++v) if (lr[v] / temperature > mx) mx = lr[v] / temperature;
            for (int64_t v = 0; v < V; ++v) { p[v] = exp(lr[v] / temperature - mx); Z += p[v]; }
            for (int64_t v = 0; v < V; ++v) p[v] /= Z;
            double S = 1.0;
            int next = -1;
            for (int j = 0; j < n_q && next < 0; ++j) {
                const int pj = parent ? parent[j] : j - 1;
                if (pj != cur) continue;
                const int32_t x = dr[j];
                if (x < 0 || x >= V || p[x] == 0.0) continue;      /* struck out already */
                const double lhs = u_accept[(int64_t)b * n_q + j] * S;
                const double gap = fabs(lhs - p[x]) / S;
                if (gap < worst) worst = gap;
                if (lhs <= p[x]) next = j;
                else { S -= p[x]; p[x] = 0.0; }
            }
            if (next >= 0) { path[len++] = next; cur = next; continue; }
            /* bonus token from the remaining mass */
            const double target = u_bonus[b] * S;
            double cdf = 0.0;
            int64_t pick = -1, last_pos = -1;
            for (int64_t v = 0; v < V; ++v) {
                if (p[v] <= 0.0) continue;
                last_pos = v;
                const double before = cdf;
                cdf += p[v];
                if (cdf >= target) {
                    pick = v;
                    double g = (cdf - target) / S;
                    if (before > 0.0 && (target - before) / S < g) g = (target - before) / S;
                    if (g < worst) worst = g;
                    break;
                }
            }
            if (pick < 0) pick = last_pos;          /* rounding left the sum a hair below target */
            bonus_id[b] = (int32_t)pick;
            break;
        }
        accept_len[b] = len;
        if (margin) margin[b] = worst;
    }
    free(p);
    return 0;
}

/* ------------------------------------------------------------------------
 * Stochastic acceptance against a SAMPLED draft (temperature > 0): the
 * speculative-sampling rule whose distribution guarantee the paper relies on
 * (Related Work, first paragraph), for a draft that draws its proposals from
 * a distribution q instead of proposing them with certainty, extended to
 * several sibling proposals drawn independently from the same q (multi-round
 * rejection of the tree-speculation line of work):
 *   at the current node, p = softmax(logits / T) of the node's row and q =
 *   the draft's distribution over the children's tokens (row of draft_q);
 *   the residual is R = p with mass S = 1;
 *   children are tried in increasing node index; child j with token x is
 *   accepted with probability min(1, (R[x] / S) / q[x]), i.e. if
 *       R[x] > 0  and  u_accept[j] * q[x] * S <= R[x];
 *   on a rejection the residual becomes R[v] <- max(R[v] - S q[v], 0) for
 *   every v, S <- sum_v R[v]   (the normalised max(p - q, 0) of the rule);
 *   an accepted child becomes the current node (fresh p, q, R);
 *   when no child is accepted, or at a leaf, the bonus token is drawn from
 *   the residual by inverse CDF in vocabulary order:
 *       bonus = min { t : sum_{v <= t} R[v] >= u_bonus * S }.
 * With children drawn i.i.d. from q the first emitted token is distributed
 * exactly as p (pinned by Monte Carlo and closed forms in the tests).
 *
 * draft_q [B*(n_q+1), V]: row r = distribution the children of row r were
 * drawn from (row 0 of a sequence = last accepted token, row 1+i = node i);
 * rows of leaves are not read.  Other arguments and outputs as
 * oracle_accept_sample.  margin: the bonus draw as there (distance of u S to
 * the CDF values around it, over S); an acceptance test compares two numbers
 * that can both be tiny against S (a tail token has q[x] and p[x] ~ 1e-5), so
 * its distance |u q[x] S - R[x]| is taken relative to the magnitudes that
 * went into it: u q[x] S + p[x] + q[x] * (sum of the S of the rejections so
 * far at this node) -- the scale on which rounding moves either side.
 * ------------------------------------------------------------------------ */
int oracle_accept_sample_q(const double *logits, const int32_t *draft_ids, const int32_t *parent,
                           int B, int n_q, int64_t V, double temperature, const double *draft_q,
                           const double *u_accept, const double *u_bonus, int32_t *accept_len,
                           int32_t *accept_path, int32_t *bonus_id, double *margin)
{
    if (!(temperature > 0.0)) return -2;
    for (int i = 0; parent && i < n_q; ++i)
        if (parent[i] < -1 || parent[i] >= i) return -1;
    double *R = (double *)malloc(sizeof(double) * (size_t)V);
    for (int b = 0; b < B; ++b) {
        const int32_t *dr = draft_ids + (int64_t)b * n_q;
        int32_t *path = accept_path + (int64_t)b * n_q;
        for (int i = 0; i < n_q; ++i) path[i] = -1;
        int cur = -1, len = 0;
        double worst = INFINITY;
        for (;;) {
            const int64_t row = (int64_t)b * (n_q + 1) + cur + 1;
            const double *lr = logits + row * V;
            const double *q = draft_q + row * V;
            double mx = -INFINITY, Z = 0.0;
            for (int64_t v = 0; v < V; ++v) if (lr[v] / temperature > mx) mx = lr[v] / temperature;
            for (int64_t v = 0; v < V; ++v) { R[v] = exp(lr[v] / temperature - mx); Z += R[v]; }
            for (int64_t v = 0; v < V; ++v) R[v] /= Z;
            double S = 1.0, S_spent = 0.0;              /* S_spent: sum of S over the rejections */
            int next = -1;
            for (int j = 0; j < n_q && next < 0; ++j) {
                const int pj = parent ? parent[j] : j - 1;
                if (pj != cur) continue;
                const int32_t x = dr[j];
                if (x < 0 || x >= V) continue;
                const double lhs = u_accept[(int64_t)b * n_q + j] * q[x] * S;
                const double px = exp(lr[x] / temperature - mx) / Z;
                const double scale = lhs + px + q[x] * S_spent;
                const double gap = scale > 0.0 ? fabs(lhs - R[x]) / scale : 0.0;
                if (gap < worst) worst = gap;
                if (R[x] > 0.0 && lhs <= R[x]) { next = j; break; }
                S_spent += S;
                double S_new = 0.0;                     /* rejected: R <- max(R - S q, 0) */
                for (int64_t v = 0; v < V; ++v) {
                    const double r = R[v] - S * q[v];
                    R[v] = r > 0.0 ? r : 0.0;
                    S_new += R[v];
                }
                S = S_new;
            }
            if (next >= 0) { path[len++] = next; cur = next; continue; }
            const double target = u_bonus[b] * S;
            double cdf = 0.0;
            int64_t pick = -1, last_pos = -1;
            for (int64_t v = 0; v < V; ++v) {
                if (R[v] <= 0.0) continue;
                last_pos = v;
                const double before = cdf;
                cdf += R[v];
                if (cdf >= target) {
                    pick = v;
                    double g = (cdf - target) / S;
                    if (before > 0.0 && (target - before) / S < g) g = (target - before) / S;
                    if (g < worst) worst = g;
                    break;
                }
            }
            if (pick < 0) pick = last_pos;          /* rounding left the sum a hair below target */
            bonus_id[b] = (int32_t)(pick < 0 ? 0 : pick);
            break;
        }
        accept_len[b] = len;
        if (margin) margin[b] = worst;
    }
    free(R);
    return 0;
}

/* ------------------------------------------------------------------------
 * Counter-based random numbers for the acceptance tests: Philox4x32 with 10
 * rounds (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as
 * 1, 2, 3", SC'11).  One round maps the counter (c0, c1, c2, c3) with round
 * key (k0, k1) to (hi(M1 c2) ^ c1 ^ k0, lo(M1 c2), hi(M0 c0) ^ c3 ^ k1,
 * lo(M0 c0)) with the multipliers M0 = 0xD2511F53, M1 = 0xCD9E8D57; the key
 * grows by the Weyl constants (0x9E3779B9, 0xBB67AE85) after every round.
 * Uniforms: the top 24 bits of a 32-bit output, times 2^-24, in [0, 1).
 *   u_accept[b][j] = first output word of counter (offset lo, offset hi, b, j),
 *   u_bonus[b]     = first output word of counter (offset lo, offset hi, b, 0xFFFFFFFF),
 * both under the key (seed lo, seed hi).
 * ------------------------------------------------------------------------ */
void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n1 = (uint32_t)p1;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        const uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

void oracle_philox_uniforms(uint64_t seed, uint64_t offset, int B, int n_q, double *u_accept,
                            double *u_bonus)
{
    const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    for (int b = 0; b < B; ++b) {
        for (int j = 0; j <= n_q; ++j) {
            const uint32_t ctr[4] = {(uint32_t)offset, (uint32_t)(offset >> 32), (uint32_t)b,
                                     j < n_q ? (uint32_t)j : 0xFFFFFFFFu};
            uint32_t out[4];
            oracle_philox4x32_10(ctr, key, out);
            const double u = (double)(out[0] >> 8) * (1.0 / 16777216.0);
            if (j < n_q) u_accept[(int64_t)b * n_q + j] = u; else u_bonus[b] = u;
        }
    }
}

/* ------------------------------------------------------------------------
 * Dynamic draft tree (Experiment section: "dynamic tree structure",
 * configuration total tokens - depth - width, e.g. 30-4-8).  The paper names
 * the configuration and not the procedure; reading taken: the best-first
 * expansion of the tree-speculation work it builds on.
 *   score of a node = sum of the draft's log-probabilities along its path;
 *   level 0: the `width` most likely tokens after the root;
 *   level d: every frontier node proposes its `width` most likely next tokens;
 *            all width*width candidates join the pool, the `width` best of
 *            them (by score) form the next frontier;
 *   at the end the `total` best nodes of the whole pool are kept (a node's
 *   score never exceeds its parent's, so the kept set is closed under
 *   ancestors), renumbered in pool order (parents before children).
 * Ties are broken towards the lower pool index / lower token id everywhere.
 * ------------------------------------------------------------------------ */

/* The k largest logits of every row, in decreasing order (equal values: lower token id first),
 * with their natural-log softmax values.  margin[r] (optional) = the smallest gap between two
 * consecutive logits among the k+1 largest of the row (what separates the selected tokens from
 * each other and from the first one left out). */
void oracle_topk_logprob(const double *logits, int M, int64_t V, int k, int32_t *ids,
                         double *logp, double *margin)
{
    #pragma omp parallel for schedule(static)
    for (int r = 0; r < M; ++r) {
        const double *lr = logits + (int64_t)r * V;
        double mx = -INFINITY, Z = 0.0;
        for (int64_t v = 0; v < V; ++v) if (lr[v] > mx) mx = lr[v];
        for (int64_t v = 0; v < V; ++v) Z += exp(lr[v] - mx);
        const double lse = mx + log(Z);
        double prev = INFINITY, worst = INFINITY;
        int64_t prev_id = -1;
        for (int j = 0; j <= k; ++j) {           /* selection by repeated scan: k is small */
            int64_t best = -1;
            for (int64_t v = 0; v < V; ++v) {
                const int after_prev = lr[v] < prev || (lr[v] == prev && v > prev_id);
                if (!after_prev) continue;
                if (best < 0 || lr[v] > lr[best]) best = v;
            }
            if (best < 0) break;
            if (j > 0 && prev - lr[best] < worst) worst = prev - lr[best];
            if (j < k) { ids[(int64_t)r * k + j] = (int32_t)best; logp[(int64_t)r * k + j] = lr[best] - lse; }
            prev = lr[best];
            prev_id = best;
        }
        if (margin) margin[r] = worst;
    }
}

/* One level of the expansion.  n_front frontier nodes (pool indices front_in, or NULL at level 0
 * where the single "frontier node" is the root, index -1, score 0) each propose `width`
 * candidates (cand_ids, cand_logp [n_front, width]).  The candidates are appended to the pool at
 * n_pool.. in (frontier order, candidate order); front_out [width] receives the pool indices of
 * the `width` best of them, best first.  Returns the new pool size.  margin (optional): smallest
 * score gap between consecutive candidates among the width+1 best. */
int oracle_tree_expand(int n_front, int width, const int32_t *front_in, const int32_t *cand_ids,
                       const double *cand_logp, int32_t *pool_tok, int32_t *pool_par,
                       double *pool_score, int n_pool, int32_t *front_out, double *margin)
{
    const int n_new = n_front * width;
    for (int f = 0; f < n_front; ++f)
        for (int j = 0; j < width; ++j) {
            const int p = front_in ? front_in[f] : -1;
            const int i = n_pool + f * width + j;
            pool_tok[i] = cand_ids[f * width + j];
            pool_par[i] = p;
            pool_score[i] = (p >= 0 ? pool_score[p] : 0.0) + cand_logp[f * width + j];
        }
    double prev = INFINITY, worst = INFINITY;
    int prev_i = -1;
    for (int j = 0; j <= width && j < n_new + 1; ++j) {
        int best = -1;
        for (int i = n_pool; i < n_pool + n_new; ++i) {
            const int after_prev = pool_score[i] < prev || (pool_score[i] == prev && i > prev_i);
            if (!after_prev) continue;
            if (best < 0 || pool_score[i] > pool_score[best]) best = i;
        }
        if (best < 0) break;
        if (j > 0 && prev - pool_score[best] < worst) worst = prev - pool_score[best];
        if (j < width) front_out[j] = best;
        prev = pool_score[best];
        prev_i = best;
    }
    if (margin) *margin = worst;
    return n_pool + n_new;
}

/* Final selection: the `total` best pool nodes (score, then lower pool index), renumbered in
 * pool order.  Outputs parent [total] (-1 = child of the root), ids [total], pool_index [total].
 * Returns the number of nodes kept (min(total, n_pool)); -1 if the kept set is not closed under
 * ancestors (cannot happen for log-probabilities <= 0). */
int oracle_tree_select(const int32_t *pool_tok, const int32_t *pool_par, const double *pool_score,
                       int n_pool, int total, int32_t *parent, int32_t *ids, int32_t *pool_index,
                       double *margin)
{
    const int keep = total < n_pool ? total : n_pool;
    char *sel = (char *)calloc((size_t)(n_pool > 0 ? n_pool : 1), 1);
    double prev = INFINITY, worst = INFINITY;
    int prev_i = -1;
    for (int j = 0; j <= keep; ++j) {
        int best = -1;
        for (int i = 0; i < n_pool; ++i) {
            const int after_prev = pool_score[i] < prev || (pool_score[i] == prev && i > prev_i);
            if (!after_prev) continue;
            if (best < 0 || pool_score[i] > pool_score[best]) best = i;
        }
        if (best < 0) break;
        if (j > 0 && prev - pool_score[best] < worst) worst = prev - pool_score[best];
        if (j < keep) sel[best] = 1;
        prev = pool_score[best];
        prev_i = best;
    }
    int n = 0, rc = keep;
    int32_t *new_id = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n_pool > 0 ? n_pool : 1));
    for (int i = 0; i < n_pool; ++i) {
        new_id[i] = -1;
        if (!sel[i]) continue;
        const int p = pool_par[i];
        if (p >= 0 && !sel[p]) rc = -1;
        new_id[i] = n;
        parent[n] = p >= 0 ? new_id[p] : -1;
        ids[n] = pool_tok[i];
        pool_index[n] = i;
        ++n;
    }
    if (margin) *margin = worst;
    free(sel);
    free(new_id);
    return rc;
}
