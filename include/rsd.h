/*
 * rsd.h -- C ABI of the draft-tree hot path of Recursive Speculative Decoding
 * (RSD, arXiv 2402.14160) for AMD MI355X (gfx950).
 *
 * Conventions common to every call
 * --------------------------------
 *  - Every array pointer is a DEVICE pointer owned by the caller.  The library
 *    never allocates, frees or keeps any of them.  Scratch memory comes from the
 *    caller through (workspace, workspace_bytes); the matching
 *    rsd_*_workspace_bytes() call gives the size needed (it may be 0, then
 *    workspace may be NULL).  Workspace contents need not be initialised; the
 *    pointer must be 16-byte aligned (RSD_ERR_WORKSPACE otherwise).
 *  - `stream` is a hipStream_t passed as void*.  Calls only enqueue work on it
 *    and never synchronise; outputs are valid once the stream has drained.
 *  - Return value: RSD_OK or a negative rsd_status.  On an error nothing is
 *    launched.  Data-dependent anomalies (non-finite logits, an empty residual)
 *    are reported through device-side flag arrays, not through the return code.
 *  - Randomness is a pure function of (seed, step, stream tag, sequence id,
 *    node row, vocabulary index): Philox4x32-10 with key = (seed lo, seed hi) and
 *    counter = (vocab_index >> 2, node_row, seq, tag | step << 4); entry x uses
 *    output word x & 3.  Tags: 0 drafting Gumbel noise, 1 accept/reject uniform
 *    (vocab_index 0, node_row = the verified node), 2 last-token Gumbel noise
 *    (node_row = the node whose distribution is sampled).  Only the low 28 bits of
 *    `step` enter the counter: streams repeat after 2^28 steps of one seed.  A 32-bit word w maps
 *    to u = (2*(w >> 9) + 1) * 2^-24 and to the Gumbel variate -log(-log u).
 *  - Tree layout: nodes of one sequence are stored in level order; node 0 is the
 *    root (the last already-known token), parent[0] = -1 and 0 <= parent[i] < i
 *    for i > 0.  Children of one parent appear in the order they were drafted
 *    (decreasing perturbed score); they need not be contiguous.  Logit row i of a
 *    sequence holds the model's next-token logits after the token sequence that
 *    ends in node i.
 *  - All floating-point arrays are fp32 unless stated otherwise; index arrays
 *    are int32.  Row-major, innermost dimension contiguous.
 */
#ifndef RSD_H
#define RSD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum rsd_status {
    RSD_OK = 0,
    RSD_ERR_NULL = -1,        /* a required pointer is NULL                              */
    RSD_ERR_SHAPE = -2,       /* a size is out of range or a pointer/stride is misaligned */
    RSD_ERR_TREE = -3,        /* host-checked tree violates the layout contract          */
    RSD_ERR_WORKSPACE = -4,   /* workspace missing, too small or not 16-byte aligned      */
    RSD_ERR_LAUNCH = -5,      /* the HIP runtime refused a launch                        */
    RSD_ERR_UNSUPPORTED = -6, /* valid request outside what the kernels implement        */
    RSD_ERR_TOO_LARGE = -7    /* request needs more scratch than a fixed-size buffer holds  */
} rsd_status;

/* Compile-time limits. */
#define RSD_K_MAX 16        /* samples per row (Gumbel-Top-k), beam width, siblings per parent */
#define RSD_NODES_MAX 256   /* tree nodes per sequence, root included                         */
#define RSD_VOCAB_MAX 65536 /* vocabulary entries per row for the sampling calls              */

#define RSD_DTYPE_BF16 0
#define RSD_DTYPE_F32 1

#define RSD_MODE_PATH 0       /* verify only the sibling groups on the accepted path     */
#define RSD_MODE_ALL_GROUPS 1 /* verify every sibling group in parallel, then walk        */

#define RSD_BASELINE_KSEQ 0        /* K-SEQ draft selection of SpecTr                          */
#define RSD_BASELINE_MULTIROUND 1  /* multi-round rejection sampling of SpecInfer              */

/* bits of the per-sequence flag word written by rsd_recursive_reject */
#define RSD_FLAG_DEGENERATE_RESIDUAL 1u /* a residual had no positive mass; q^(k) was kept */
#define RSD_FLAG_NONFINITE 2u           /* a non-finite normaliser was met                  */

/* Library version (major*10000 + minor*100 + patch). */
int32_t rsd_version(void);

/* Static, human-readable text for a status code. Never NULL. */
const char *rsd_status_string(int32_t status);

/* Host-side check of one sequence's parent array against the tree layout
 * contract.  parent_host is a HOST pointer to n_nodes ints.
 * Returns RSD_OK, RSD_ERR_NULL, RSD_ERR_SHAPE (n_nodes < 1 or > RSD_NODES_MAX)
 * or RSD_ERR_TREE. */
int32_t rsd_validate_tree(const int32_t *parent_host, int32_t n_nodes);

/* ---------------------------------------------------------------------------
 * Vocabulary log-softmax normaliser (Sec. 3.2.1, Eq. (5): phi = log p(.|tau);
 * the target-side counterpart of Sec. 3.2.2).
 *   lse[r] = log sum_x exp(logits[r, x] * inv_temperature),  r < R.
 * logits: [R, V] fp32 with row stride ld (elements); logits must be 16-byte
 * aligned and ld a multiple of 4.  1 <= V; R may be 0 (no-op).
 * Needs no workspace.
 * ------------------------------------------------------------------------- */
int32_t rsd_log_softmax_lse(const float *logits, int64_t ld, int32_t R, int32_t V,
                            float inv_temperature, float *lse, void *stream);

/* ---------------------------------------------------------------------------
 * Gumbel-Top-k sampling without replacement (Sec. 3.2.1 RSD-C, Eqs. (5)-(7);
 * Alg. 4 SampleWithGumbelTopK).  Per row r:
 *   phi = log-softmax(logits[r] * inv_temperature); phi~ = phi + Gumbel noise;
 *   outputs the k_r = min(k_per_row[r], k_max) entries with the largest phi~ in
 *   decreasing order (ties: lower token first).  Entries with -inf logits are
 *   never returned, so count[r] may be below k_r.
 * Inputs
 *   logits      [R, V], row stride ld; 16-byte aligned, ld % 4 == 0
 *   k_per_row   [R] or NULL (= k_max everywhere); values < 0 are treated as 0
 *   seq_id      [R] or NULL (= 0): Philox sequence coordinate of the row
 *   node_id     [R] or NULL (= r): Philox node-row coordinate of the row
 * Outputs (each [R, k_max] unless noted; unused slots: token -1, values -inf)
 *   tokens, perturbed (phi~), logprob (phi), lse [R], count [R]
 *   perturbed, logprob, lse, count may each be NULL when not wanted.
 * Limits: 1 <= k_max <= RSD_K_MAX, 1 <= V <= RSD_VOCAB_MAX, k_max <= V.
 * Needs no workspace (rsd_gumbel_topk_workspace_bytes returns 0).
 * ------------------------------------------------------------------------- */
size_t rsd_gumbel_topk_workspace_bytes(int32_t R, int32_t V, int32_t k_max);
int32_t rsd_gumbel_topk(const float *logits, int64_t ld, int32_t R, int32_t V, int32_t k_max,
                        const int32_t *k_per_row, float inv_temperature,
                        const int32_t *seq_id, const int32_t *node_id,
                        uint64_t seed, uint32_t step,
                        int32_t *tokens, float *perturbed, float *logprob, float *lse,
                        int32_t *count, void *workspace, size_t workspace_bytes, void *stream);

/* ---------------------------------------------------------------------------
 * One Stochastic Beam Search expansion (Sec. 3.2.1 RSD-S, Eqs. (10)-(12);
 * Alg. 9 SampleWithStochasticBeam).  Per sequence b with n_in[b] live beam rows:
 *   Phi = log-softmax(logits[b,w]) + sum_logprob[b,w];  Phi~ = Phi + Gumbel;
 *   psi = T(trunc_gumbel[b,w], Phi~) with the row maximum of Phi~ (Eq. (11));
 *   the W (parent row, token) pairs with the largest psi over all live rows are
 *   returned in decreasing psi (ties: lower row, then lower token) with their
 *   Phi (new sum log-prob) and psi (new truncated Gumbel).
 * Inputs
 *   logits        [B, W_in, V] contiguous, 16-byte aligned, V % 4 == 0 or W_in*B == 1
 *                 (every row must start 16-byte aligned)
 *   sum_logprob, trunc_gumbel  [B, W_in]  (root beam: one live row holding 0, 0)
 *   n_in          [B] live rows per sequence, 0 <= n_in[b] <= W_in
 *   seq_id        [B] or NULL (= b);  node_id [B, W_in] or NULL (= w)
 * Outputs ([B, W]; unused slots token/parent -1, scores -inf)
 *   tokens, parent (index of the parent row within the W_in rows),
 *   sum_logprob_out, trunc_gumbel_out, n_out [B]; lse [B, W_in] or NULL.
 * Limits: 1 <= W <= RSD_K_MAX, 1 <= W_in <= RSD_K_MAX, V <= RSD_VOCAB_MAX, W <= V.
 * ------------------------------------------------------------------------- */
size_t rsd_sbs_step_workspace_bytes(int32_t B, int32_t W_in, int32_t V, int32_t W);
int32_t rsd_sbs_step(const float *logits, const float *sum_logprob, const float *trunc_gumbel,
                     const int32_t *n_in, const int32_t *seq_id, const int32_t *node_id,
                     int32_t B, int32_t W_in, int32_t V, int32_t W, float inv_temperature,
                     uint64_t seed, uint32_t step,
                     int32_t *tokens, int32_t *parent, float *sum_logprob_out,
                     float *trunc_gumbel_out, int32_t *n_out, float *lse,
                     void *workspace, size_t workspace_bytes, void *stream);

/* ---------------------------------------------------------------------------
 * rsd_sbs_step for callers that cannot allocate device memory or bring a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments (without the workspace pair), same kernels and
 * bit-identical outputs as rsd_sbs_step; the per-row candidate lists live in a
 * device array of RSD_SBS_STATIC_SCRATCH_BYTES bytes inside the library (one copy
 * per GPU, held until the process ends).  The call allocates and frees nothing.
 * Limit: rsd_sbs_step_workspace_bytes(B, W_in, V, W) <= RSD_SBS_STATIC_SCRATCH_BYTES,
 *   else RSD_ERR_TOO_LARGE and nothing is launched (e.g. B * W_in up to 1024 rows
 *   at W = 16 fit).
 * All calls on one GPU share that GPU's array: two calls whose kernels may overlap
 * (different streams, no ordering between them) race; calls on one stream do not.
 * The array keeps the previous call's contents; nothing in it needs clearing, every
 * slot a call reads was written by that call.  The first call on a device looks the
 * array's address up (no allocation); make that call outside stream capture.
 * ------------------------------------------------------------------------- */
#define RSD_SBS_STATIC_SCRATCH_BYTES 524288
int32_t rsd_sbs_step_static(const float *logits, const float *sum_logprob,
                            const float *trunc_gumbel, const int32_t *n_in, const int32_t *seq_id,
                            const int32_t *node_id, int32_t B, int32_t W_in, int32_t V, int32_t W,
                            float inv_temperature, uint64_t seed, uint32_t step,
                            int32_t *tokens, int32_t *parent, float *sum_logprob_out,
                            float *trunc_gumbel_out, int32_t *n_out, float *lse, void *stream);

/* ---------------------------------------------------------------------------
 * Tree-masked attention of the draft-tree tokens (Sec. 3.2.2, tree evaluation
 * with the target model; Alg. 2 step 2; mask of Alg. 5 BuildAttentionMask).
 * Query row i of sequence b attends the first prefix_len[b] cached keys and the
 * tree nodes j that are i itself or an ancestor of i (the root is an ancestor of
 * every node):  out[i] = sum_j softmax_j(scale * q_i . k_j) v_j.
 * Query head h reads KV head h / (H_q / H_kv).
 * Inputs (dtype = RSD_DTYPE_BF16: 2-byte bfloat16; RSD_DTYPE_F32: fp32)
 *   q                  [B, H_q, N_max, D] contiguous
 *   k_prefix, v_prefix element strides (prefix_stride_b, prefix_stride_h, prefix_stride_p),
 *                      D contiguous; may be NULL when every prefix_len is 0
 *   k_tree, v_tree     [B, H_kv, N_max, D] contiguous
 *   prefix_len [B], n_nodes [B] (0 <= n_nodes[b] <= N_max), parent [B, N_max]
 *   P_max              upper bound of prefix_len (used to size the launch)
 *   num_splits         key-range splits per (sequence, head); 0 = choose automatically,
 *                      values above 32 are taken as 32
 * Outputs
 *   out     [B, H_q, N_max, D] fp32; rows i >= n_nodes[b] are not written
 *   lse_out [B, H_q, N_max] natural-log softmax normaliser, or NULL.  On the bf16 path it
 *           is the log of the sum of the bf16-rounded weights that multiply V (the sum
 *           `out` is normalised by), within 2^-8 relative of the exact sum.
 * Limits: bf16: D in {64, 128}; f32: D <= 256; N_max <= RSD_NODES_MAX;
 *   H_q % H_kv == 0; scale positive and finite (else RSD_ERR_SHAPE); all tensors 16-byte
 *   aligned, prefix strides multiples of 8 (bf16) or 4 (f32).  Invalid parent values are
 *   clamped on the device (no fault).
 * Workspace: rsd_tree_attention_workspace_bytes(...) with the same num_splits.
 * ------------------------------------------------------------------------- */
size_t rsd_tree_attention_workspace_bytes(int32_t dtype, int32_t B, int32_t H_q, int32_t H_kv,
                                          int32_t N_max, int32_t D, int32_t P_max,
                                          int32_t num_splits);
int32_t rsd_tree_attention(const void *q, const void *k_prefix, const void *v_prefix,
                           const void *k_tree, const void *v_tree, int32_t dtype,
                           int32_t B, int32_t H_q, int32_t H_kv, int32_t N_max, int32_t D,
                           int32_t P_max, int64_t prefix_stride_b, int64_t prefix_stride_h,
                           int64_t prefix_stride_p,
                           const int32_t *prefix_len, const int32_t *n_nodes,
                           const int32_t *parent, float scale, int32_t num_splits,
                           float *out, float *lse_out,
                           void *workspace, size_t workspace_bytes, void *stream);

/* ---------------------------------------------------------------------------
 * The same attention for L layers in one call (Alg. 2 / Alg. 7, step 2: the target
 * model evaluates the draft tree in every layer; the tree, its mask and the prefix
 * lengths are the same in all of them).  Layer l reads q + l * q_stride_l,
 * k_prefix / v_prefix + l * prefix_stride_l, k_tree / v_tree + l * tree_stride_l and
 * writes out + l * out_stride_l (lse_out + l * lse_stride_l); strides are in
 * elements of the respective tensor, multiples of 8 (bf16) or 4 (fp32) for the
 * inputs and of 4 for `out`.  Inside a layer every tensor is laid out as for
 * rsd_tree_attention, and every output row equals what that call gives for the
 * layer alone.  The ancestor sets and the launch plan are shared: the work of all
 * L * B (layer, sequence) pairs goes into one set of launches, so that a small
 * batch fills the chip over its layers instead of splitting the prefix.
 * Limits: those of rsd_tree_attention, 1 <= L, L * B <= 65535.
 * Workspace: rsd_tree_attention_layers_workspace_bytes(...) with the same num_splits.
 * ------------------------------------------------------------------------- */
size_t rsd_tree_attention_layers_workspace_bytes(int32_t dtype, int32_t L, int32_t B, int32_t H_q,
                                                 int32_t H_kv, int32_t N_max, int32_t D,
                                                 int32_t P_max, int32_t num_splits);
int32_t rsd_tree_attention_layers(const void *q, const void *k_prefix, const void *v_prefix,
                                  const void *k_tree, const void *v_tree, int32_t dtype,
                                  int32_t L, int64_t q_stride_l, int64_t prefix_stride_l,
                                  int64_t tree_stride_l, int64_t out_stride_l, int64_t lse_stride_l,
                                  int32_t B, int32_t H_q, int32_t H_kv, int32_t N_max, int32_t D,
                                  int32_t P_max, int64_t prefix_stride_b, int64_t prefix_stride_h,
                                  int64_t prefix_stride_p,
                                  const int32_t *prefix_len, const int32_t *n_nodes,
                                  const int32_t *parent, float scale, int32_t num_splits,
                                  float *out, float *lse_out,
                                  void *workspace, size_t workspace_bytes, void *stream);

/* ---------------------------------------------------------------------------
 * Recursive rejection sampling over the draft tree (Sec. 3.1, Eqs. (1)-(4),
 * Alg. 1; Sec. 3.2.2 verification; Alg. 6 RecursiveRejectionSampling).
 * Starting at the root, the children of the current node form one sibling
 * group x_1..x_K (stored order) with p = softmax(draft_logits[b, node]),
 * q = softmax(target_logits[b, node]):
 *   Theta_k = min(1, q^(k)(x_k) / p^(k)(x_k)),  accept child k iff u < Theta_k,
 *   q^(k+1) = Norm[(q^(k) - p^(k))^+],  p^(k+1) = p^(k) with x_k zeroed, renormalised.
 * The first accepted child becomes the current node.  When all children are
 * rejected the last token is the Gumbel-max sample of q^(K+1); a node without
 * children samples the last token from q itself.
 * Inputs
 *   draft_logits, target_logits [B, N_max, V] contiguous, 16-byte aligned, V % 4 == 0, V <= 131072
 *   tokens [B, N_max] (tokens[b,0] unused), parent [B, N_max], n_nodes [B] (>= 1)
 *   seq_id [B] or NULL (= b)
 *   mode   RSD_MODE_PATH or RSD_MODE_ALL_GROUPS (identical decisions; the second
 *          computes every group's thresholds as if its earlier siblings were rejected)
 * Outputs
 *   accepted_nodes  [B, depth_max] node ids along the accepted path (-1 padded)
 *   accepted_tokens [B, depth_max] or NULL
 *   n_accepted [B], last_token [B]
 *   final_node [B] or NULL   node at which the last token was drawn
 *   theta      [B, N_max] or NULL  thresholds of verified nodes (NaN elsewhere)
 *   uniforms   [B, N_max] or NULL  the uniform of every node
 *   flags      [B] or NULL         RSD_FLAG_* bits
 * Limits: N_max <= RSD_NODES_MAX; at most RSD_K_MAX children per node
 *   (further children are ignored and RSD_FLAG_NONFINITE is not set for that);
 *   1 <= depth_max.  A path longer than depth_max is truncated in the outputs only.
 * Workspace: rsd_recursive_reject_workspace_bytes(B, N_max, V).
 * ------------------------------------------------------------------------- */
size_t rsd_recursive_reject_workspace_bytes(int32_t B, int32_t N_max, int32_t V);
int32_t rsd_recursive_reject(const float *draft_logits, const float *target_logits,
                             int32_t B, int32_t N_max, int32_t V, float inv_temperature,
                             const int32_t *tokens, const int32_t *parent,
                             const int32_t *n_nodes, const int32_t *seq_id, int32_t mode,
                             uint64_t seed, uint32_t step,
                             int32_t *accepted_nodes, int32_t *accepted_tokens,
                             int32_t depth_max, int32_t *n_accepted, int32_t *last_token,
                             int32_t *final_node, float *theta, float *uniforms,
                             uint32_t *flags, void *workspace, size_t workspace_bytes,
                             void *stream);

/* ---------------------------------------------------------------------------
 * FilterKVCache (Alg. 2 / Alg. 7, step 4): after the verification, append to the
 * cache the key/value rows of the decoded tokens that the tree evaluation just
 * produced: the root (tree node 0, the last known token) and then the accepted
 * nodes in path order.  For sequence b and every KV head h:
 *   cache[b, h, prefix_len[b] + j, :] = tree[b, h, node_j, :],  node_0 = 0,
 *   node_j = accepted_nodes[b, j - 1]  (1 <= j <= n_accepted[b]),
 *   prefix_len_out[b] = min(prefix_len[b] + 1 + n_accepted[b], capacity).
 * Call once for the target cache and once for the draft cache.
 * Inputs / in-out (all device pointers; the cache is modified in place)
 *   k_cache, v_cache  element strides (cache_stride_b, cache_stride_h, cache_stride_p),
 *                     D contiguous, `capacity` rows per (sequence, head)
 *   k_tree, v_tree    [B, H_kv, N_max, D] contiguous; must not overlap the cache
 *   prefix_len [B], accepted_nodes [B, depth_max] (-1 padded), n_accepted [B]
 *   (the outputs of rsd_recursive_reject fit as they are)
 * Outputs
 *   prefix_len_out [B]  must not alias prefix_len
 *   flags [B] or NULL   bit 0: rows beyond `capacity` were dropped
 * Limits: dtype bf16 or f32; D * element size a multiple of 16; 16-byte aligned
 *   pointers and strides; N_max, depth_max <= RSD_NODES_MAX.  Node ids outside
 *   [0, N_max) are clamped on the device (no fault).  No workspace.
 * ------------------------------------------------------------------------- */
int32_t rsd_filter_kv_cache(void *k_cache, void *v_cache, const void *k_tree, const void *v_tree,
                            int32_t dtype, int32_t B, int32_t H_kv, int32_t N_max, int32_t D,
                            int32_t capacity, int64_t cache_stride_b, int64_t cache_stride_h,
                            int64_t cache_stride_p, const int32_t *prefix_len,
                            const int32_t *accepted_nodes, int32_t depth_max,
                            const int32_t *n_accepted, int32_t *prefix_len_out, uint32_t *flags,
                            void *stream);

/* ---------------------------------------------------------------------------
 * Top-k / nucleus (top-p) filtering of logit rows (Sec. 4, experiment setup:
 * nucleus sampling with p = 0.95; the samplers of Alg. 4 and Alg. 9 drop
 * candidates whose log-probability is -inf after such filtering).  Per row, with
 * P = softmax(logits * inv_temperature) over the finite entries:
 *   top_k > 0 : keep the top_k most probable entries;
 *   top_p < 1 : keep the smallest set of most probable entries whose mass reaches
 *               top_p (of the distribution renormalised over the top-k set when
 *               both are given);
 *   entries as probable as the least probable kept entry are kept too.
 * Kept entries are copied unchanged (not scaled), all others become -inf, so the
 * result feeds rsd_gumbel_topk / rsd_sbs_step / rsd_recursive_reject directly.
 * Inputs   logits [R, V] fp32 device, row stride ld (multiple of 4, >= V), 16-byte aligned
 * Outputs  out    [R, V] fp32 device, row stride out_ld (same rules); may be `logits` itself
 *          kept   [R] number of kept entries, or NULL
 * Limits: 1 <= V <= RSD_VOCAB_MAX; inv_temperature > 0; top_k >= 0 (0 = off);
 *   top_p > 0 (>= 1 = off).  -inf / NaN entries are never kept.  No workspace.
 * Precision: probabilities are ranked as 2^y with y = (logit - row max) *
 *   inv_temperature * log2(e) held in fp32, so two entries whose probabilities
 *   differ by less than about |y| * 2^-22 * ln 2 (relative) may count as equally
 *   probable, and sums of probabilities are fp32 (about 1e-6 of mass).  With top_p
 *   given, entries below 2^-126 of the row maximum carry no mass and are dropped;
 *   top_k alone ranks them too, down to 2^-2142 of the maximum, below which an
 *   entry is never kept.
 * ------------------------------------------------------------------------- */
int32_t rsd_filter_logits(const float *logits, int64_t ld, int32_t R, int32_t V,
                          float inv_temperature, int32_t top_k, float top_p, float *out,
                          int64_t out_ld, int32_t *kept, void *stream);

/* ---------------------------------------------------------------------------
 * Baseline verifiers of one level of K draft tokens drawn i.i.d. (with
 * replacement) from the draft distribution (Sec. 2, tree-based speculative
 * decoding; compared with recursive rejection sampling in the toy example of
 * Sec. 3.1).  Per row r with p = softmax(draft_logits[r]), q = softmax(target_logits[r])
 * and drafts x_1..x_K = drafts[r, :]:
 *   RSD_BASELINE_KSEQ        accept x_k with probability min(1, q(x_k) / (gamma p(x_k)));
 *                            all rejected: draw from
 *                            Norm[(q - min(p, q/gamma) (1 - (1-beta)^K) / beta)^+],
 *                            beta = sum_x min(p(x), q(x)/gamma);
 *   RSD_BASELINE_MULTIROUND  accept x_k with probability min(1, q^(k)(x_k) / p(x_k)),
 *                            q^(1) = q, q^(k+1) = Norm[(q^(k) - p)^+];
 *                            all rejected: draw from q^(K+1).
 * The first accepted draft is the output; the final draw is a Gumbel-max sample.
 * Randomness: uniform of draft k = accept stream (tag 1) at (seq_id[r], node_id[r],
 * vocabulary index k); final noise = last-token stream (tag 2) at (seq_id[r], node_id[r]).
 * Inputs
 *   draft_logits, target_logits [R, V] fp32, row stride ld (elements, >= V), 16-byte aligned bases
 *   drafts [R, K] tokens (clamped into the vocabulary), 1 <= K <= RSD_K_MAX
 *   gamma  K-SEQ only, 1 <= gamma <= K (gamma = K is always admissible)
 *   seq_id [R] or NULL (= 0), node_id [R] or NULL (= r)
 * Outputs
 *   accepted [R]  index of the accepted draft, or -1
 *   token    [R]  the accepted draft token, or the token drawn from the residual
 *   theta    [R, K] or NULL  every draft's threshold, as if all earlier ones were rejected
 *   flags    [R] or NULL     RSD_FLAG_NONFINITE; RSD_FLAG_DEGENERATE_RESIDUAL when the draw used a
 *                            residual that had no mass (the previous distribution was kept) or, for
 *                            K-SEQ, a gamma too small for the residual to be non-negative
 * No workspace.  The rows are streamed once per pass (multi-round: K + 2 passes).
 * ------------------------------------------------------------------------- */
int32_t rsd_baseline_verify(const float *draft_logits, const float *target_logits, int64_t ld,
                            int32_t R, int32_t V, const int32_t *drafts, int32_t K, int32_t method,
                            float gamma, float inv_temperature, const int32_t *seq_id,
                            const int32_t *node_id, uint64_t seed, uint32_t step,
                            int32_t *accepted, int32_t *token, float *theta, uint32_t *flags,
                            void *stream);

#ifdef __cplusplus
}
#endif
#endif /* RSD_H */
