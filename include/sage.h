/*
 * sage.h -- C ABI of the MI355X (gfx950) hot path of SAGE, entropy-guided adaptive
 * speculative decoding: the per-step draft-tree machinery around the target model's
 * parallel verification.
 *
 * Four operations, one call each, in the order a decoding step uses them
 * (Alg. 1: Phase 3 prepares the tree that Phase 1/2 of the next iteration use):
 *
 *   sage_entropy_topk    Sec. 3.1, Eq. (7)-(9)   confidence from the draft distribution
 *                        (also the target's greedy token per tree node, k = 1)
 *   sage_build_tree      Sec. 3.2, Eq. (10)-(12) adaptive depth/width, recursive expansion
 *   sage_tree_attention  Sec. 2.2 tree mask, Alg. 1 Phase 2: the attention operator of the
 *                        target's single verification pass over all tree nodes
 *   sage_verify_accept   Sec. 2.2 / Sec. 3.3 Phase 2: longest accepted root-to-leaf prefix
 *
 * Conventions common to all calls
 *   - Every data pointer is caller-owned DEVICE memory unless marked (host).  The library
 *     keeps no state, allocates nothing, never synchronises and never frees.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the default
 *     stream).  Outputs are valid once the stream reaches that point.
 *   - Sizes that change from step to step (n_nodes, kv_len, n_valid) are read on the
 *     device, so the four calls chain without a host round trip.
 *   - Per-sequence tree arrays have a fixed stride of SAGE_MAX_NODES entries; entries at or
 *     beyond n_nodes[b] are neither read nor written.  Node 0 is the root (the last
 *     committed token); nodes are in creation order (depth-first, pre-order), so
 *     parent[v] < v.  A tree always has its root: every call that takes n_nodes treats a
 *     value below 1 as 1 and a value above SAGE_MAX_NODES as SAGE_MAX_NODES.  (Row groups of
 *     sage_entropy_topk are a different thing: n_valid[g] = 0 processes no row of group g.)
 *   - Return value: SAGE_OK, or an error code; on error nothing has been enqueued.
 *   - Logits must be finite or -inf (NaN / +inf give unspecified values, never a fault).
 */
#ifndef SAGE_H
#define SAGE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SAGE_MAX_NODES 64   /* tree nodes per sequence incl. the root: one 64-bit mask word, one wavefront */
#define SAGE_MAX_TOPK 64    /* largest k of sage_entropy_topk */
#define SAGE_MAX_DEPTH 31   /* largest d_max of sage_build_tree */

enum sage_status {
    SAGE_OK = 0,
    SAGE_INVALID_ARG = 1,          /* null pointer, size or parameter out of range, bad stride/alignment */
    SAGE_UNSUPPORTED = 2,          /* valid request outside the instantiated kernels (e.g. bf16 head_dim != 128) */
    SAGE_WORKSPACE_TOO_SMALL = 3,
    SAGE_LAUNCH_FAILED = 4         /* hipGetLastError() after a launch */
};

enum sage_dtype { SAGE_F32 = 0, SAGE_BF16 = 1 };

/* Tree hyper-parameters of Alg. 1 (D_min, D_max, W_min, W_max, k, N_max).  The paper's
 * experiments use 3, 8, 2, 10, 10, 64.  Constraints: 1 <= d_min <= d_max <= SAGE_MAX_DEPTH,
 * 1 <= w_min <= w_max <= k <= SAGE_MAX_TOPK, 1 <= n_max <= SAGE_MAX_NODES (root included). */
typedef struct sage_tree_params {
    int d_min, d_max, w_min, w_max, k, n_max;
} sage_tree_params;

/* ------------------------------------------------------------------------------------------
 * sage_entropy_topk -- Sec. 3.1.  For each row x[0..vocab) of logits:
 *   P = softmax(x) (Eq. 1);  entropy = -sum P ln P (nats, full vocabulary, 0 ln 0 = 0);
 *   Top_k = first k indices under the total order (logit descending, index ascending);
 *   topk_prob = P on Top_k;  topk_renorm = topk_prob / sum(topk_prob)           (Eq. 7);
 *   topk_entropy = -sum topk_renorm ln topk_renorm                              (Eq. 8);
 *   alpha = clamp(1 - topk_entropy / ln k, 0, 1), alpha = 1 when k = 1          (Eq. 9).
 * With k = 1, topk_idx is the greedy (argmax, ties to the lowest index) token of each row,
 * which is how the target's choice at every tree node is obtained.
 *
 * logits       [rows, vocab], dtype f32 or bf16, row r starts at element r * row_stride;
 *              rows must be 16-byte aligned (row_stride * elem size multiple of 16).
 * n_valid      nullable.  Rows form groups of rows_per_group; only the first
 *              n_valid[g] rows of group g are processed (e.g. rows_per_group = 64 and
 *              n_valid = n_nodes for per-node target logits); other rows' outputs are untouched.
 * entropy, topk_entropy, alpha   [rows] f32;  topk_idx [rows,k] i32;
 * topk_prob, topk_renorm         [rows,k] f32.  Any output pointer except topk_idx may be NULL.
 * workspace    sage_entropy_topk_workspace_bytes(rows, vocab, k) bytes, 16-byte aligned.
 * Errors: INVALID_ARG for null logits/topk_idx/workspace, rows < 0, vocab < 1, k outside
 * [1, min(vocab, SAGE_MAX_TOPK)], misaligned rows; WORKSPACE_TOO_SMALL.
 */
size_t sage_entropy_topk_workspace_bytes(int rows, int vocab, int k);
int sage_entropy_topk(const void* logits, int dtype, int rows, int vocab, long row_stride, int k,
                      const int* n_valid, int rows_per_group,
                      float* entropy, int* topk_idx, float* topk_prob, float* topk_renorm,
                      float* topk_entropy, float* alpha,
                      void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * sage_build_tree -- Sec. 3.2.  Per sequence b, from topk_renorm[b, 0..k) (descending) and
 * alpha[b], in IEEE fp32 without fused multiply-add:
 *   D = floor(d_min + alpha (d_max - d_min) + 0.5)                              (Eq. 10)
 *   W = min(k, floor(w_min + (1 - alpha)(w_max - w_min) + 0.5))                 (Eq. 11)
 *   expand(u) at level l = depth(u) + 1 <= D:  W_1 = W;  for l > 1
 *       W_l = min(k, max(1, floor((W / l) (0.5 + cum(u)))))                     (Eq. 12)
 *     for r = 0 .. W_l - 1:  c = cum(u) * topk_renorm[r];  if c > 0.1 l / D the candidate
 *     becomes node v = n++ (parent u, depth l, rank r, cum c) and is expanded at once;
 *     nothing is added once n == n_max.
 * The same renormalised top-k vector is used at every node (the tree is planned for the
 * next step from the current step's distribution).
 *
 * topk_renorm [B,k] f32, alpha [B] f32, params (host) copied at call time.
 * d_max_seq [B] i32 (device), nullable: when given, sequence b uses d_max_seq[b], clamped to
 * [d_min, SAGE_MAX_DEPTH], in place of params->d_max (the maximum depth that
 * sage_update_history maintains, Sec. 3.3).
 * topk_idx [B,k] i32, nullable: the vocabulary ids of the k candidates (as written by
 * sage_entropy_topk); with it, node_token[b][v] = topk_idx[b][rank(v)] is the draft token of
 * node v (the candidate a node stands for), root -1.
 * n_nodes [B] i32; parent, depth, rank [B,64] i32 (root: -1, 0, -1); anc_mask [B,64] u64,
 * bit j of anc_mask[b][v] set iff j is v or an ancestor of v; cum_prob [B,64] f32, nullable;
 * node_token [B,64] i32, nullable (requires topk_idx).
 * Errors: INVALID_ARG for null pointers, B < 0, k != params->k, parameter constraints,
 * node_token without topk_idx.
 */
int sage_build_tree(const float* topk_renorm, const float* alpha, const int* topk_idx, int B, int k,
                    const sage_tree_params* params, const int* d_max_seq,
                    int* n_nodes, int* parent, int* depth, int* rank, uint64_t* anc_mask, float* cum_prob,
                    int* node_token, void* stream);

/* ------------------------------------------------------------------------------------------
 * sage_tree_attention -- the attention operator of the verify pass (Alg. 1 Phase 2) under
 * the tree mask of Sec. 2.2.  For sequence b, node i < n_nodes[b], query head h
 * (kv head g = h / (Hq / Hkv)):
 *   keys/values = all cache positions j < kv_len[b]  U  tree nodes t with bit t set in
 *   anc_mask[b][i];   O[b,i,h,:] = softmax_j(scale * Q[b,i,h,:] . K_j) V_j.
 *
 * Q, O    [B,64,Hq,d];  Kt, Vt [B,64,Hkv,d] (keys/values of the tree nodes themselves);
 * Kc, Vc  cache: element (b, j, g, c) at (kv_start[b] + j) * kv_token_stride
 *         + g * kv_head_stride + c  (strides in elements; rows 16-byte aligned);
 * kv_start [B] i64, kv_len [B] i32 (device); max_kv_len (host) >= every kv_len[b], used
 * only to size the launch; dtype applies to Q, K, V and O alike.
 * bf16: MFMA path, requires d == 128, Hq / Hkv <= 16, kv_token_stride <= 2^24 elements;
 * fp32: d <= 256, multiple of 4.
 * Accumulation is fp32; bf16 outputs are rounded to nearest even.
 * first_node [B] i32 (device), nullable = all zero: only the rows of nodes first_node[b] <= i <
 * n_nodes[b] are computed and written; earlier nodes still serve as keys and values through
 * the masks.  This is the draft side of Alg. 1 Phase 1, where the tree grows by one level per
 * forward pass and call l needs the rows of level l only (nodes in level order).  Values
 * outside [0, n_nodes[b]) are clamped into that range.
 * workspace: sage_tree_attention_workspace_bytes(...) bytes, 256-byte aligned.
 * Errors: INVALID_ARG (null pointers, B < 0, Hq % Hkv != 0, strides, max_kv_len < 0),
 * UNSUPPORTED (shape outside the above), WORKSPACE_TOO_SMALL.
 */
size_t sage_tree_attention_workspace_bytes(int dtype, int B, int Hq, int Hkv, int d, int max_kv_len);
int sage_tree_attention(const void* Q, const void* Kc, const void* Vc, const void* Kt, const void* Vt, void* O,
                        int dtype, int B, int Hq, int Hkv, int d,
                        const int64_t* kv_start, const int* kv_len, int max_kv_len,
                        long kv_token_stride, long kv_head_stride,
                        const uint64_t* anc_mask, const int* n_nodes, const int* first_node, float scale,
                        void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * sage_verify_accept -- acceptance under greedy decoding (Sec. 2.2, Sec. 3.3 Phase 2,
 * Def. 4.1).  Node i > 0 matches iff token[i] == target_argmax[parent[i]]; it is accepted iff
 * it and all its ancestors match.  best_node = deepest accepted node (ties: lowest index),
 * accept_len = tau = its depth.  path_nodes = root .. best_node; out_tokens = the tau draft
 * tokens on that path followed by target_argmax[best_node] (tau + 1 tokens advance).
 *
 * token, target_argmax, parent, depth [B,64] i32; anc_mask [B,64] u64 (as emitted by
 * sage_build_tree; it must be the ancestor-or-self relation of parent[]); n_nodes [B].
 * accept_len, best_node [B] i32; path_nodes, out_tokens [B,path_cap] i32, padded with -1.
 * path_cap (host) must exceed the deepest node's depth (d_max + 1 suffices); deeper paths
 * are truncated to path_cap entries, never written out of bounds.
 * Errors: INVALID_ARG for null pointers, B < 0, path_cap < 1.
 */
int sage_verify_accept(const int* token, const int* target_argmax, const int* parent, const int* depth,
                       const uint64_t* anc_mask, const int* n_nodes, int B, int path_cap,
                       int* accept_len, int* best_node, int* path_nodes, int* out_tokens, void* stream);

/* ------------------------------------------------------------------------------------------
 * sage_commit_path -- the accepted tokens join the context (Alg. 1 Phase 3, Sec. 2.2): one
 * layer's share.  For sequence b with tau = accept_len[b] and path = path_nodes[b][0..tau]
 * (root first, as sage_verify_accept emits it), the K and V rows of the tau + 1 path nodes
 * (the root, whose K/V is not in the cache yet, and the tau accepted draft tokens) are
 * copied, bytes unchanged, to cache positions kv_len[b] + j, j = 0..tau.  The bonus token
 * has no K/V yet; it is the next step's root.  kv_len is read, not changed: every layer
 * commits against the same old length; call sage_advance_kv_len once afterwards.
 *
 * Kt, Vt [B,64,Hkv,d] (device); Kc, Vc cache addressed as in sage_tree_attention (rows
 * 16-byte aligned, d * element size a multiple of 16); kv_capacity (host): positions per
 * sequence that the cache holds, positions at or beyond it are not written;
 * path_nodes [B,path_cap] i32, accept_len [B] i32 (device).  Entries of path_nodes outside
 * [0,64) are skipped.  Errors: INVALID_ARG (null pointers, sizes, strides, alignment),
 * UNSUPPORTED (B > 65535, path_cap > 64).
 *
 * sage_advance_kv_len -- kv_len[b] = min(kv_len[b] + accept_len[b] + 1, kv_capacity), in place.
 */
int sage_commit_path(const void* Kt, const void* Vt, void* Kc, void* Vc, int dtype, int B, int Hkv, int d,
                     const int64_t* kv_start, const int* kv_len, int kv_capacity,
                     long kv_token_stride, long kv_head_stride,
                     const int* path_nodes, const int* accept_len, int path_cap, void* stream);
int sage_advance_kv_len(int* kv_len, const int* accept_len, int B, int kv_capacity, void* stream);

/* ------------------------------------------------------------------------------------------
 * sage_update_history -- adaptive history tracking (Sec. 3.3; Sec. 5 "Implementation details":
 * window 10, thresholds 2 and 3).  Per sequence b the step's acceptance length accept_len[b]
 * enters a sliding window of the last `window` values; the moving average runs over the
 * values present (fewer than `window` during the first steps).  Average < lo: d_max[b]
 * drops by one, not below d_floor; average > hi: it rises by one, not above d_cap; otherwise
 * unchanged (both comparisons strict, evaluated as sum vs threshold * count in fp32).
 * Feed d_max to sage_build_tree as d_max_seq.
 *
 * State, all device, updated in place: hist [B,window] i32 (ring, slot = count mod window),
 * count [B] i32 (steps so far; start at 0), d_max [B] i32.  avg_out [B] f32, nullable.
 * Errors: INVALID_ARG (null pointers, B < 0, window outside [1,64], d_floor < 1,
 * d_floor > d_cap, d_cap > SAGE_MAX_DEPTH, lo > hi).
 */
int sage_update_history(const int* accept_len, int B, int window, float lo, float hi, int d_floor, int d_cap,
                        int* hist, int* count, int* d_max, float* avg_out, void* stream);

/* ------------------------------------------------------------------------------------------
 * sage_close_step -- what closes a step of Alg. 1 (Phase 3 update of the context, Sec. 3.3
 * adaptive history tracking) in one launch: sage_commit_path for one layer, then
 * sage_advance_kv_len, then sage_update_history, with the same arguments, semantics and
 * results (one workgroup per sequence does all three in that order; the path rows are copied
 * against the old kv_len[b], which is then advanced in place).  For models with several
 * layers, commit the other layers with sage_commit_path first.
 * d_max_in / d_max_out [B] i32 (device): the depth limit is read from d_max_in and the updated
 * one written to d_max_out.  They may be the same array; two arrays let a tree-planning call
 * that runs concurrently on another stream keep reading the limit of the previous step.
 * Errors: as for the three calls it replaces.
 */
int sage_close_step(const void* Kt, const void* Vt, void* Kc, void* Vc, int dtype, int B, int Hkv, int d,
                    const int64_t* kv_start, int* kv_len, int kv_capacity,
                    long kv_token_stride, long kv_head_stride,
                    const int* path_nodes, const int* accept_len, int path_cap,
                    int window, float lo, float hi, int d_floor, int d_cap,
                    int* hist, int* count, const int* d_max_in, int* d_max_out, float* avg_out, void* stream);

/* ------------------------------------------------------------------------------------------
 * sage_lm_head_topk -- sage_entropy_topk on logits that are never stored: row r of the
 * logits is hidden[r, :] . weight[v, :] over v < vocab (the target's output projection,
 * whose softmax is the distribution of Eq. 1 and whose argmax is the greedy token of
 * Def. 4.1).  Products are accumulated in fp32 and not rounded to a storage type; outputs,
 * row groups and n_valid exactly as in sage_entropy_topk.
 *
 * hidden [rows, dim], weight [vocab, dim], row-major with row strides in elements, rows
 * 16-byte aligned.  This build: bf16, dim a multiple of 128, row strides <= 2^24 elements,
 * vocab <= 655360; k = 1 for any number of rows (the target's node rows), 1 < k <= 16 for up
 * to 64 rows (a draft model's rows, Sec. 3.1); others: UNSUPPORTED.  The weight matrix is
 * fetched from HBM once per call; rows that n_valid marks dead cost nothing (live rows are
 * packed into blocks of 128 before the pass).
 * workspace: sage_lm_head_topk_workspace_bytes(rows, vocab, k) bytes, 16-byte aligned.
 * Errors: INVALID_ARG (null pointers, sizes, strides, alignment, k outside [1, min(vocab,
 * SAGE_MAX_TOPK)]), UNSUPPORTED, WORKSPACE_TOO_SMALL.
 */
size_t sage_lm_head_topk_workspace_bytes(int rows, int vocab, int k);
int sage_lm_head_topk(const void* hidden, const void* weight, int dtype, int rows, int dim, int vocab,
                      long hidden_stride, long weight_stride, int k, const int* n_valid, int rows_per_group,
                      float* entropy, int* topk_idx, float* topk_prob, float* topk_renorm,
                      float* topk_entropy, float* alpha,
                      void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * The step with two launches fewer.  A step (Alg. 1) is a chain of small dependent launches;
 * each costs a few microseconds however little it computes.  sage_entropy_topk is two
 * launches (per-slice pass, per-row pass); these calls split it so that the per-row pass runs
 * inside the launch that consumes its result.  Results are bit-identical to the separate calls.
 *
 * sage_entropy_topk_slices: the per-slice pass of sage_entropy_topk only (Sec. 3.1 inputs:
 * same logits / dtype / rows / vocab / row_stride / k / n_valid / rows_per_group arguments,
 * same checks); leaves statistics and candidates in `workspace` (device,
 * sage_entropy_topk_workspace_bytes(rows, vocab, k) bytes, layout private to the library),
 * which must stay untouched until the consuming call below has run on the same stream.
 *
 * sage_build_tree_from_slices: finishes Eq. 7-9 for B draft rows (one per sequence: slices
 * filled with rows = B and this vocab and k) and builds each sequence's tree (Sec. 3.2) in
 * the same launch.  Outputs: those of sage_entropy_topk ([B] / [B,k]; topk_idx required, the
 * others nullable) and those of sage_build_tree (node_token nullable; cum_prob nullable).
 *
 * sage_verify_accept_from_slices: finishes the k = 1 reduction of the B * 64 target rows
 * (slices filled with rows = B * 64, k = 1, n_valid = n_nodes, rows_per_group = 64) and
 * applies the acceptance rule (Sec. 2.2, Sec. 3.3 Phase 2).  Outputs: target_argmax [B,64]
 * (required), entropy [B,64] (nullable; full-vocabulary entropy of each live target row) and
 * those of sage_verify_accept.  Rows of nodes >= n_nodes[b] are neither read nor written.
 * Errors as for the calls they replace; `slices` 16-byte aligned.
 *
 * sage_entropy_topk_slices_pair: two per-slice passes that do not depend on each other in ONE
 * launch: job A = sage_entropy_topk_slices(logits_a, rows_a, k = 1, n_valid_a, rows_per_group_a)
 * (the target rows of the trees being verified, Sec. 2.2) and job B = sage_entropy_topk_slices(
 * logits_b, rows_b, k_b > 1, every row valid) (draft rows, Sec. 3.1; in a decoding loop those of
 * the NEXT step, whose planning depends on nothing this step's verification produces).  Both
 * workspaces end up exactly as after the two separate calls; same dtype and vocab for both.
 * Errors: INVALID_ARG if n_valid_a is null or k_b < 2, otherwise those of the separate calls.
 */
int sage_entropy_topk_slices(const void* logits, int dtype, int rows, int vocab, long row_stride, int k,
                             const int* n_valid, int rows_per_group, void* workspace, size_t workspace_bytes,
                             void* stream);
int sage_entropy_topk_slices_pair(const void* logits_a, int rows_a, long row_stride_a, const int* n_valid_a,
                                  int rows_per_group_a, void* workspace_a, size_t workspace_a_bytes,
                                  const void* logits_b, int rows_b, long row_stride_b, int k_b, void* workspace_b,
                                  size_t workspace_b_bytes, int dtype, int vocab, void* stream);
int sage_build_tree_from_slices(void* slices, int vocab, int B, int k, const sage_tree_params* params,
                                const int* d_max_seq, float* entropy, int* topk_idx, float* topk_prob,
                                float* topk_renorm, float* topk_entropy, float* alpha, int* n_nodes, int* parent,
                                int* depth, int* rank, uint64_t* anc_mask, float* cum_prob, int* node_token,
                                void* stream);
int sage_verify_accept_from_slices(void* slices, int vocab, const int* token, const int* parent, const int* depth,
                                   const uint64_t* anc_mask, const int* n_nodes, int B, int path_cap,
                                   float* entropy, int* target_argmax, int* accept_len, int* best_node,
                                   int* path_nodes, int* out_tokens, void* stream);

/* ------------------------------------------------------------------------------------------
 * sage_verify_accept_close_from_slices -- sage_verify_accept_from_slices followed by
 * sage_close_step (one layer) in one launch: the workgroup that has found a sequence's
 * accepted path (Sec. 2.2) appends that path's K/V rows to the cache, advances the length and
 * updates the acceptance history (Alg. 1 Phase 3, Sec. 3.3) while the path is still on chip.
 * Arguments, semantics, results and errors: those of the two calls, in their order.
 */
int sage_verify_accept_close_from_slices(
    void* slices, int vocab, const int* token, const int* parent, const int* depth, const uint64_t* anc_mask,
    const int* n_nodes, int B, int path_cap, float* entropy, int* target_argmax, int* accept_len, int* best_node,
    int* path_nodes, int* out_tokens,
    const void* Kt, const void* Vt, void* Kc, void* Vc, int dtype, int Hkv, int d, const int64_t* kv_start, int* kv_len,
    int kv_capacity, long kv_token_stride, long kv_head_stride, int window, float lo, float hi, int d_floor, int d_cap,
    int* hist, int* count, const int* d_max_in, int* d_max_out, float* avg_out, void* stream);

/* ------------------------------------------------------------------------------------------
 * sage_tree_attention_with_plan -- sage_tree_attention and sage_build_tree_from_slices in one
 * launch.  With the lookahead of Sec. 3.2 the tree planned at a step (Sec. 3.1-3.2, from the
 * step's draft distribution) is the one verified at the NEXT step, so the planning of a step
 * and its verification attention (Alg. 1 Phase 2) touch disjoint data; here the planning
 * workgroups (one per sequence) ride in the attention launch beside the workgroups that
 * stream the cache, which removes planning's launch from the step's chain of dependent
 * launches.  Results of both halves are bit-identical to the two separate calls.
 *
 * Arguments: those of sage_tree_attention without first_node (a verify pass computes every
 * node's rows), through workspace_bytes, then those of
 * sage_build_tree_from_slices without its B (one draft row per sequence of the attention
 * batch: `slices` filled by sage_entropy_topk_slices with rows = B); the planned tree goes to
 * next_n_nodes / next_parent / next_depth / next_rank / next_anc_mask (/ next_cum_prob,
 * next_node_token, nullable), which must not be the arrays the attention reads (n_nodes,
 * anc_mask).  bf16 with at most 256 slices per draft row and at most 2400 candidates per row
 * in `slices` (vocab 152064 with k = 16: 149 slices, 2384 candidates): one launch (plus the
 * split merge of the attention); otherwise (fp32, longer lists) the two calls are enqueued
 * one after the other with the same results.
 * Errors: those of the two calls, checked before anything is enqueued; INVALID_ARG when the
 * planned tree's arrays alias the verified tree's.
 */
int sage_tree_attention_with_plan(
    const void* Q, const void* Kc, const void* Vc, const void* Kt, const void* Vt, void* O, int dtype, int B, int Hq, int Hkv,
    int d, const int64_t* kv_start, const int* kv_len, int max_kv_len, long kv_token_stride, long kv_head_stride,
    const uint64_t* anc_mask, const int* n_nodes, float scale, void* workspace, size_t workspace_bytes,
    void* slices, int vocab, int k, const sage_tree_params* params, const int* d_max_seq, float* entropy, int* topk_idx,
    float* topk_prob, float* topk_renorm, float* topk_entropy, float* alpha, int* next_n_nodes, int* next_parent,
    int* next_depth, int* next_rank, uint64_t* next_anc_mask, float* next_cum_prob, int* next_node_token, void* stream);

/* ------------------------------------------------------------------------------------------
 * sage_tree_attention_static -- sage_tree_attention for callers that cannot allocate: code
 * under HIP graph capture, serving loops and harnesses that must not call hipMalloc (or any
 * allocating routine) and so cannot provide a workspace sized per call.  Arguments, results
 * (bit-identical) and errors are those of sage_tree_attention without its workspace pair and
 * without first_node (every node's rows are computed): the
 * split partials live in a device array inside the library,
 * sage_tree_attention_static_scratch_bytes() = 40 MiB per GPU the library runs on, held until
 * the process ends.  The call allocates and frees nothing.
 * Limit: a call whose sage_tree_attention_workspace_bytes(...) exceeds that size returns
 * SAGE_WORKSPACE_TOO_SMALL and enqueues nothing (72B shape: one sequence of any length fits;
 * a batch of 16 fits; a batch of 24 does not).  fp32 calls use no scratch at all.
 * All calls on one GPU share the one array: two calls may not overlap in time on a GPU
 * (different streams without ordering, or two host threads), or their partials race.  Calls
 * ordered on one stream are safe; nothing needs clearing between calls.
 * Further error: LAUNCH_FAILED when the array's device address cannot be obtained.
 */
size_t sage_tree_attention_static_scratch_bytes(void);
int sage_tree_attention_static(const void* Q, const void* Kc, const void* Vc, const void* Kt, const void* Vt, void* O,
                               int dtype, int B, int Hq, int Hkv, int d,
                               const int64_t* kv_start, const int* kv_len, int max_kv_len,
                               long kv_token_stride, long kv_head_stride,
                               const uint64_t* anc_mask, const int* n_nodes, float scale, void* stream);

/* Library build identification (host): returns a static string naming the target architecture. */
const char* sage_build_info(void);

#ifdef __cplusplus
}
#endif
#endif /* SAGE_H */
