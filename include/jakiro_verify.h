/*
 * libjakiro_verify -- tree verification for Jakiro-style speculative decoding
 * on AMD MI355X (gfx950).  C ABI: plain pointers and sizes only.
 *
 * The two central calls follow the verification and refinement steps of speculative
 * decoding as the paper states them (Section 2.1, steps 2 and 3), applied to
 * the draft token TREE that Jakiro's two experts build (Section 3.1.2: at
 * every depth each activated expert proposes its own top-k candidates, the
 * higher-scoring expert's on the left; candidates are verified together
 * through a tree attention mask):
 *
 *   jk_tree_verify_attention  the attention of the target model's single
 *       verification pass: every tree node attends to the committed KV prefix,
 *       to itself and to its tree ancestors, and to nothing else, so that each
 *       node's result equals what ordinary decoding of its root-to-node path
 *       would give.
 *   jk_accept_path            the acceptance walk: greedy ("strict top-1
 *       verification", Section 3.2) or speculative sampling (accept with
 *       probability min(1, p/q); on rejection continue with
 *       norm(max(0, p - q)), Section 2.1), returning the accepted
 *       root-to-leaf path and the extra ("bonus") token.
 *
 * Around them: jk_commit_path* (the accepted path's K/V rows join the cache),
 * the paged-cache variants, and the draft side of a round (Section 3.1.2, 3.2):
 * jk_linear, jk_moe_experts, jk_draft_heads, jk_tree_grow / _tail / _finalize and
 * jk_gather_draft_probs produce the tree_tokens, parent[] and draft_probs that
 * the two central calls take.
 *
 * Conventions
 *   - "device" pointers are HIP device memory of the current device; "host"
 *     pointers are ordinary host memory.  The caller owns every buffer.  The
 *     library allocates no device memory and keeps no state between calls;
 *     scratch comes from the caller's workspace (sizes from the *_workspace
 *     functions; 256-byte aligned).  A workspace handed to jk_accept_path or
 *     jk_tree_verify_attention(_paged) must have been zero-filled once
 *     (jk_workspace_init, or any other means; of an attention workspace only the
 *     first JK_WORKSPACE_HEADER_BYTES matter) before its first use; after that it can be reused for
 *     any number of calls of any shape it is large enough for.  Those bytes hold
 *     the sticky device error word (jk_last_device_error) and the words through
 *     which workgroups of one call meet; the calls leave them consistent.
 *   - Calls enqueue work on `hip_stream` (a hipStream_t, NULL = default
 *     stream) and return without synchronising.  Outputs are valid once the
 *     stream has reached that point.  Calls that share a workspace must be
 *     ordered on one stream.
 *   - Errors are return codes only.  On any code other than JK_OK nothing was
 *     launched and no output was written.
 *   - Trees: parent[i] is the tree parent of node i, -1 for a child of the
 *     committed prefix (several such nodes are allowed), and -1 <= parent[i] < i
 *     (any topological numbering, e.g. BFS).  Children of one parent are
 *     ordered left to right by increasing index.  The array lives on the
 *     device, so the library cannot check it on the host: a node whose entry
 *     violates the rule is treated as having parent -1, and the kernel that
 *     repaired it sets JK_DEVERR_BAD_TREE in the workspace's error word
 *     (Section 3.1.2: candidates form a tree; a repaired tree is not the one
 *     the caller drafted).  jk_validate_tree checks a host copy.
 */
#ifndef JAKIRO_VERIFY_H
#define JAKIRO_VERIFY_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  JK_OK = 0,
  JK_ERR_INVALID_ARG = 1, /* null pointer, non-positive size, bad stride, bad scale/temperature */
  JK_ERR_BAD_TREE = 2,    /* jk_validate_tree only */
  JK_ERR_UNSUPPORTED = 3, /* shape outside the supported set (see each call) */
  JK_ERR_WORKSPACE = 4,   /* workspace missing, misaligned or too small */
  JK_ERR_HIP = 5,         /* a HIP runtime call failed (launch configuration, bad stream) */
  JK_ERR_SCRATCH_LIMIT = 6 /* jk_accept_path_greedy_static only: the input needs more than JK_STATIC_SCRATCH_BYTES */
} jk_status;

typedef enum { JK_BF16 = 0, JK_F32 = 1 } jk_dtype;
typedef enum { JK_GREEDY = 0, JK_SAMPLE = 1 } jk_mode;

#define JK_MAX_TREE 128 /* largest supported number of tree nodes */
#define JK_WORKSPACE_HEADER_BYTES 32768 /* start of an attention workspace that must be zero before its first use */
#define JK_STATIC_SCRATCH_BYTES (1 << 20) /* the library's built-in scratch buffer (jk_accept_path_greedy_static) */

/* Shape and layout of one attention call.  Strides are in ELEMENTS; the
 * innermost (head_dim) index is contiguous; for JK_BF16 every base pointer
 * and every stride must be a multiple of 8 elements (16 bytes), for JK_F32 a
 * multiple of 4 elements.
 *   q, out           [batch, n_tree, n_q_heads, head_dim]   (q_stride_* and o_stride_*)
 *   k_cache, v_cache [batch, capacity >= max_prefix_len, n_kv_heads, head_dim]
 *   k_tree, v_tree   [batch, n_tree, n_kv_heads, head_dim]
 * Query head h uses KV head h / (n_q_heads / n_kv_heads) (consecutive heads share). */
typedef struct {
  int32_t batch, n_tree, n_q_heads, n_kv_heads, head_dim;
  int64_t q_stride_b, q_stride_t, q_stride_h;
  int64_t kc_stride_b, kc_stride_l, kc_stride_h;
  int64_t kt_stride_b, kt_stride_t, kt_stride_h;
  int64_t o_stride_b, o_stride_t, o_stride_h;
  float scale;    /* softmax scale; 0 selects 1/sqrt(head_dim); must not be negative */
  int32_t dtype;  /* jk_dtype of q, k, v and out */
} jk_attn_desc;

/* Bytes of workspace jk_tree_verify_attention needs for this shape and this
 * upper bound on the prefix length.  Returns 0 for an invalid descriptor. */
size_t jk_tree_verify_attention_workspace(const jk_attn_desc* desc, int32_t max_prefix_len);

/* Tree-masked verification attention (Section 2.1 step 2; Section 3.1.2 tree mask).
 *
 * For every sequence b, node i and query head h:
 *     keys   = cache positions 0 .. prefix_len[b]-1  and  tree nodes {i, parent[i], parent[parent[i]], ...}
 *     out[b,i,h,:] = softmax_j(scale * <q[b,i,h,:], k_j>) . v_j
 *
 *   q, k_cache, v_cache, k_tree, v_tree   device, read only, layouts above
 *   parent       device int32 [batch, n_tree]
 *   prefix_len   device int32 [batch]; values are clamped to [0, max_prefix_len]
 *   max_prefix_len  host scalar: upper bound on prefix_len[], at most the cache
 *                capacity; it sizes the launch and the workspace.  (The lengths
 *                themselves stay on the device so that a decoding loop never
 *                needs a host round trip between its steps.)
 *   out          device, written; same dtype as q
 *   workspace    device, >= jk_tree_verify_attention_workspace(desc, max_prefix_len) bytes
 *
 * Supported: JK_BF16 with head_dim 64 or 128 (MFMA path), JK_F32 with
 * head_dim <= 256 and a multiple of 4 and max_prefix_len + n_tree <= 65536
 * (plain-ALU path); 1 <= n_tree <= JK_MAX_TREE;
 * n_q_heads a multiple of n_kv_heads; JK_BF16: kc_stride_l and kt_stride_t at
 * most 2^24 elements (JK_ERR_UNSUPPORTED beyond).  Value rows of tree nodes that a query
 * cannot see must be finite (they are multiplied by an exact zero); their key
 * rows, and anything in the cache beyond prefix_len, are never used.
 * Accumulation is fp32; JK_BF16 rounds the softmax weights to bf16 before the
 * value product and, when the key range is split over several workgroups, the
 * partial outputs to bf16 before they are merged (running maxima and sums stay
 * fp32). */
jk_status jk_tree_verify_attention(const jk_attn_desc* desc, const void* q, const void* k_cache,
                                   const void* v_cache, const void* k_tree, const void* v_tree,
                                   const int32_t* parent, const int32_t* prefix_len,
                                   int32_t max_prefix_len, void* out, void* workspace,
                                   size_t workspace_bytes, void* hip_stream);

/* Paged KV cache: one pool of fixed-size pages per tensor, [n_pages, page_size,
 * n_kv_heads, head_dim] with desc->kc_stride_l / kc_stride_h as the token and head
 * strides inside a page (kc_stride_b is ignored) and page_stride elements between
 * pages; token t of sequence b lives in page block_table[b * max_blocks + t /
 * page_size] at slot t % page_size.  Entries for tokens below prefix_len[b] must
 * be valid page ids; the other entries of a row (all max_blocks of them must be
 * readable) may hold anything: they may be read, and pages they name fetched
 * ahead of the length, but nothing of that reaches a result (ids outside
 * [0, n_pages) are clamped into the pool rather than followed, and reported in
 * the device error word only where a result depends on them).  The paper does not discuss cache layout:
 * this is a library convention for serving stacks. */
typedef struct {
  const int32_t* block_table; /* device int32 [batch, max_blocks] */
  int32_t max_blocks;         /* max_blocks * page_size >= max_prefix_len */
  int32_t page_size;          /* tokens per page, a multiple of 32 */
  int32_t n_pages;            /* pages in the pool */
  int64_t page_stride;        /* elements, a multiple of 8 */
} jk_paged_kv;

/* jk_tree_verify_attention over a paged cache (JK_BF16 only).  k_pool / v_pool
 * take the place of k_cache / v_cache; everything else, including the workspace
 * size (jk_tree_verify_attention_workspace), is as for the contiguous call. */
jk_status jk_tree_verify_attention_paged(const jk_attn_desc* desc, const jk_paged_kv* pages, const void* q,
                                         const void* k_pool, const void* v_pool, const void* k_tree,
                                         const void* v_tree, const int32_t* parent, const int32_t* prefix_len,
                                         int32_t max_prefix_len, void* out, void* workspace,
                                         size_t workspace_bytes, void* hip_stream);

/* Bytes of workspace jk_accept_path needs.  Returns 0 for invalid sizes.  About 2.1 MB of it are
 * the same for every shape and mode: the words through which the workgroups of a sampling
 * call meet, kept apart from everything a call of another shape or mode writes, so that calls
 * of both modes and any shapes may take turns on one workspace (sized for the largest). */
size_t jk_accept_path_workspace(int32_t batch, int32_t n_tree, int32_t vocab, int32_t mode);

/* Acceptance walk over the verified tree (Section 2.1 steps 2-3; Section 3.2
 * for greedy).  Logits row 0 is the target's distribution after the committed
 * prefix, row k+1 the one after tree node k; node k is judged with its
 * parent's row.  Starting at the prefix (c = -1):
 *   JK_GREEDY  t* = argmax of row c+1 (lowest id on ties); move to the first
 *              (left-most) child of c whose token is t*; stop when there is
 *              none; the bonus token is that last t*.
 *   JK_SAMPLE  p = softmax(row c+1 / temperature); children of c are tried
 *              left to right: child k with token x is accepted iff
 *              uniforms[k] * draft_probs[k][x] < p[x]; after a rejection p
 *              becomes max(0, p - draft_probs[k]) renormalised (kept if that
 *              sums to zero).  Stop when no child is accepted; the bonus token
 *              is the smallest v whose cumulative p exceeds uniforms[n_tree]
 *              times the total.
 *
 *   tree_tokens   device int32 [batch, n_tree]
 *   parent        device int32 [batch, n_tree]
 *   target_logits device fp32  [batch, n_tree+1, vocab], finite or -inf
 *   temperature   > 0; ignored by JK_GREEDY
 *   draft_probs   device fp32  [batch, n_tree, vocab]; required by JK_SAMPLE, else may be NULL
 *   uniforms      device fp32  [batch, n_tree+1] in [0,1); required by JK_SAMPLE
 *   out_path        device int32 [batch, max_depth]: accepted node ids, root-most first, -1 padded
 *   out_accept_len  device int32 [batch]: number of accepted nodes, at most max_depth
 *   out_bonus_token device int32 [batch]: the token that follows the last accepted node
 *   workspace     device, >= jk_accept_path_workspace(...) bytes
 *
 * max_depth stops the descent: after max_depth accepted nodes the children of the
 * last one are not examined and the bonus token comes from that node's own row
 * (argmax, or a draw from its softmax), i.e. the result is that of the same tree
 * cut below depth max_depth, and path[:accept_len] + bonus is always a sequence
 * the target model itself would have produced.
 *
 * Supported: 1 <= n_tree <= JK_MAX_TREE, vocab >= 1, max_depth >= 1.  Token ids
 * outside [0, vocab) are clamped into the range.  JK_SAMPLE runs several
 * workgroups per tree that wait for each other; the wait is bounded (a few
 * milliseconds), and if it ever expires (the device is too busy to keep them
 * resident together) out_accept_len and out_bonus_token are set to -1 for that
 * tree and JK_DEVERR_WALK_WAIT is set in the workspace's error word.  Nothing
 * else is lost: the workspace stays valid for further calls, jk_commit_path
 * treats a length of -1 as "commit nothing", and the caller may simply repeat
 * the call for that step (same inputs, same uniforms: the walk is a pure
 * function of them) or emit no draft token for it.
 * All sampling arithmetic (softmax, residuals, cumulative sums) is fp64, so a
 * decision can differ from exact arithmetic only when its two sides agree to
 * about 1e-13 relative. */
jk_status jk_accept_path(int32_t batch, int32_t n_tree, int32_t vocab, int32_t max_depth,
                         const int32_t* tree_tokens, const int32_t* parent,
                         const float* target_logits, int32_t mode, float temperature,
                         const float* draft_probs, const float* uniforms, int32_t* out_path,
                         int32_t* out_accept_len, int32_t* out_bonus_token, void* workspace,
                         size_t workspace_bytes, void* hip_stream);

/* jk_accept_path in JK_GREEDY mode for callers that cannot allocate device memory or hand
 * over a workspace: code running under HIP-graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  Same arguments, results and kernels as jk_accept_path(...,
 * JK_GREEDY, ...) minus the workspace: the per-chunk (max, argmax) partials live in a buffer
 * of JK_STATIC_SCRATCH_BYTES that is part of the library's device image (one copy per GPU the
 * library runs on, held until the process ends).  The call allocates and frees nothing.
 *
 * Limit: batch * (n_tree + 1) * ceil(vocab / 4096) * 8 bytes (each of the two partial arrays
 * rounded up to 256 bytes) must fit JK_STATIC_SCRATCH_BYTES; larger inputs return
 * JK_ERR_SCRATCH_LIMIT and launch nothing (61 rows x 128 256 entries need 16 KB, 65 535 rows
 * x 4096 entries 512 KB).  All calls on one GPU share that GPU's buffer: calls that overlap
 * in time on one GPU (different streams, different host threads) race and must be ordered
 * by the caller.  Nothing in the buffer needs to start at zero: every partial a call reads,
 * the same call has written.  Other return codes as for jk_accept_path. */
jk_status jk_accept_path_greedy_static(int32_t batch, int32_t n_tree, int32_t vocab, int32_t max_depth,
                                       const int32_t* tree_tokens, const int32_t* parent,
                                       const float* target_logits, int32_t* out_path,
                                       int32_t* out_accept_len, int32_t* out_bonus_token, void* hip_stream);

/* jk_accept_path with the draft distributions addressed through a row table instead of a
 * dense [batch][n_tree][vocab] array: node k of sequence b is tested against
 * draft_rows_all[draft_row[b][k]][:] (fp32 [n_draft_rows][vocab]; a row number outside the
 * table is clamped).  This is what jk_tree_finalize's q_row output and the draft_probs
 * buffers of the round's jk_draft_heads calls are, so the draft side's output can be
 * verified without copying 4 * vocab bytes per node (jk_gather_draft_probs).  Everything
 * else as for jk_accept_path; draft_row is device int32 [batch][n_tree] (JK_SAMPLE only). */
jk_status jk_accept_path_rows(int32_t batch, int32_t n_tree, int32_t vocab, int32_t max_depth,
                              const int32_t* tree_tokens, const int32_t* parent, const float* target_logits,
                              int32_t mode, float temperature, const float* draft_rows_all, int64_t n_draft_rows,
                              const int32_t* draft_row, const float* uniforms, int32_t* out_path,
                              int32_t* out_accept_len, int32_t* out_bonus_token, void* workspace,
                              size_t workspace_bytes, void* hip_stream);

/* Commit of the accepted path to one layer's KV cache (Section 2.1 step 3:
 * accepted tokens are appended to the sequence, the rest of the draft is
 * dropped).  For every sequence b and i < n_b the K and V rows (all KV heads) of
 * tree node path[b][i] are copied to cache position prefix_len[b] + i; with
 * `advance` != 0 prefix_len[b] then grows by n_b (the caches of all layers share
 * one length: set it on the last layer's call only).  n_b is accept_len[b] cut
 * to [0, max_depth], ended in front of the first path entry outside [0, n_tree)
 * and limited to the room left (cache_capacity - prefix_len[b]): a walk that
 * gave up (accept_len -1) commits nothing.  The token the target adds after
 * the last accepted node has no key/value yet and is not part of this call.
 *
 *   desc         as for jk_tree_verify_attention; only batch, n_tree, n_kv_heads,
 *                head_dim, dtype and the kc_ / kt_ strides are used
 *   k_tree, v_tree    device, read      [batch, n_tree, n_kv_heads, head_dim]
 *   k_cache, v_cache  device, written   [batch, cache_capacity, n_kv_heads, head_dim]
 *   path         device int32 [batch, max_depth] as written by jk_accept_path
 *   accept_len   device int32 [batch]
 *   prefix_len   device int32 [batch], read; written iff advance != 0
 *
 * Pointers and strides obey the alignment rules of the attention call (whole
 * 16-byte chunks).  Nothing is allocated; no workspace is needed. */
jk_status jk_commit_path(const jk_attn_desc* desc, const void* k_tree, const void* v_tree, void* k_cache,
                         void* v_cache, const int32_t* path, const int32_t* accept_len, int32_t max_depth,
                         int32_t cache_capacity, int32_t* prefix_len, int32_t advance, void* hip_stream);

/* The same commit for all layers of a model in one launch (a layer's copy is a
 * few tens of KB: a launch per layer costs more than the copies).  k_tree,
 * v_tree, k_cache and v_cache are DEVICE arrays of n_layers device pointers, one
 * tensor per layer, all of the shape, strides and dtype that `desc` gives and
 * 16-byte aligned (they live on the device, so the library cannot check them).
 * path, accept_len and prefix_len are shared by the layers; `advance` applies
 * once.  1 <= n_layers <= 65535. */
jk_status jk_commit_path_layers(const jk_attn_desc* desc, int32_t n_layers, const void* const* k_tree,
                                const void* const* v_tree, void* const* k_cache, void* const* v_cache,
                                const int32_t* path, const int32_t* accept_len, int32_t max_depth,
                                int32_t cache_capacity, int32_t* prefix_len, int32_t advance, void* hip_stream);

/* jk_commit_path_layers into paged caches: k_pool / v_pool are device arrays of
 * n_layers pool pointers, all described by `pages` (one block table for all
 * layers); the capacity is max_blocks * page_size.  The pages the new rows land
 * in must already be in the table. */
jk_status jk_commit_path_layers_paged(const jk_attn_desc* desc, const jk_paged_kv* pages, int32_t n_layers,
                                      const void* const* k_tree, const void* const* v_tree,
                                      void* const* k_pool, void* const* v_pool, const int32_t* path,
                                      const int32_t* accept_len, int32_t max_depth, int32_t* prefix_len,
                                      int32_t advance, void* hip_stream);

/* ---- the step in front of verification: the draft model's two output heads ----
 *
 * Jakiro's draft layer routes a hidden state to its two best experts and gives
 * both experts' features to the output embedding it shares with the target
 * model (Section 3.1.2 Eq. 4, Section 3.2 Eq. 6-8).  With f1, f2 the features of
 * the expert with the larger / smaller router score and s1 >= s2 those scores:
 *
 *   JK_HEADS_DECOUPLED    x_left = s1 f1,           x_right = s2 f2           (Eq. 4)
 *   JK_HEADS_CONTRASTIVE  x_moe  = s1 f1 + s2 f2,   x_const = beta f1 - alpha f2   (Eq. 6, 7)
 *   logits[r][h] = w_head . x_h            (both heads, one pass over w_head)
 *   draft_probs[r][h] = softmax(logits[r][h] / temperature)      (the q of the acceptance test)
 *   topk_tokens[r][h] = the top_k largest logits' token ids, best first, equal
 *                       logits by increasing id; topk_probs their draft_probs
 *
 * (Eq. 4 as printed puts the mixed feature into both heads; the per-expert
 * features of Eq. 6 are what is computed here, so that left + right = moe.)
 * The heads' inputs are rounded to bf16 once, products accumulate in fp32.
 *
 *   rows         hidden states in this call (tree nodes being expanded, all
 *                sequences together), 1..128
 *   d_model      feature width, a multiple of 128, at most 16384
 *   vocab        rows of w_head, top_k..2^24
 *   top_k        1..16
 *   f_top        device bf16 [rows][2][d_model], 16-byte aligned
 *   s_top        device fp32 [rows][2]
 *   w_head       device bf16 [vocab][d_model], 16-byte aligned
 *   logits       device fp32 [rows][2][vocab], written
 *   draft_probs  device fp32 [rows][2][vocab], written; may be NULL
 *   topk_tokens  device int32 [rows][2][top_k], written
 *   topk_probs   device fp32 [rows][2][top_k], written
 *   workspace    device, jk_draft_heads_workspace(rows, d_model, vocab) bytes, 256-byte aligned
 * A logits row containing NaN gives unspecified candidates for that row; a row
 * with fewer than top_k logits above -inf reports token 0 with probability 0 in
 * the remaining places.
 * JK_ERR_UNSUPPORTED for rows, d_model or top_k outside the ranges above. */
typedef enum { JK_HEADS_DECOUPLED = 0, JK_HEADS_CONTRASTIVE = 1 } jk_heads_mode;

typedef struct {
  int32_t rows, d_model, vocab, top_k;
  int32_t mode;      /* jk_heads_mode */
  float temperature; /* > 0 */
  float alpha, beta; /* Eq. 7; ignored for JK_HEADS_DECOUPLED */
} jk_draft_heads_desc;

size_t jk_draft_heads_workspace(int32_t rows, int32_t d_model, int32_t vocab);

jk_status jk_draft_heads(const jk_draft_heads_desc* desc, const void* f_top, const float* s_top,
                         const void* w_head, float* logits, float* draft_probs, int32_t* topk_tokens,
                         float* topk_probs, void* workspace, size_t workspace_bytes, void* hip_stream);

/* The draft layer's router and expert MLPs that produce jk_draft_heads' inputs
 * (Section 3.1.2, Eq. 2, 3 and 5 with K = 2 activated experts), for `rows`
 * hidden states u (Eq. 1's output: the draft layer's attention plus residual is
 * an input here):
 *
 *   s_j = softmax_j(u . e_j)                  router over the n_experts centroids (Eq. 2, fp32)
 *   top1, top2 = the two largest s_j, larger first, ties to the lower expert (Eq. 5)
 *   f_top[r][k] = Expert_topk(u_r) + u_r      Expert_j(x) = w_down_j (silu(w_gate_j x) * (w_up_j x))
 *   f_mix[r]    = s_top1 Expert_top1(u_r) + s_top2 Expert_top2(u_r) + u_r            (Eq. 3)
 *
 * (The paper calls the experts lightweight MLPs and leaves out normalisation
 * layers; the gated form is this library's reading.)  The projections run
 * through the same MFMA kernel as jk_draft_heads with bf16 operands and fp32
 * accumulation; the hidden activation silu(gate)*up and the outputs are rounded
 * to bf16 once each.  Every expert that at least one row selected is evaluated
 * for all rows (its weights are streamed once either way; gathering rows would
 * cost more than the MFMAs it saves); experts that no row selected are skipped.
 *
 *   rows        1..128;  d_model, d_ff multiples of 128 up to 65536;  n_experts 2..64
 *   u           device bf16 [rows][d_model], 16-byte aligned
 *   centroids   device bf16 [n_experts][d_model]
 *   w_gate, w_up  device bf16 [n_experts][d_ff][d_model];  w_down [n_experts][d_model][d_ff]
 *   f_top       device bf16 [rows][2][d_model], written
 *   s_top       device fp32 [rows][2], written;  expert_idx device int32 [rows][2], written
 *   f_mix       device bf16 [rows][d_model], written; may be NULL
 *   workspace   jk_moe_experts_workspace(desc) bytes, 256-byte aligned */
typedef struct {
  int32_t rows, d_model, d_ff, n_experts;
} jk_moe_desc;

size_t jk_moe_experts_workspace(const jk_moe_desc* desc);

jk_status jk_moe_experts(const jk_moe_desc* desc, const void* u, const void* centroids, const void* w_gate,
                         const void* w_up, const void* w_down, void* f_top, float* s_top, int32_t* expert_idx,
                         void* f_mix, void* workspace, size_t workspace_bytes, void* hip_stream);

/* ---- growing the draft tree from the heads' candidate lists ----
 *
 * Section 3.1.2: at every depth both activated experts propose their own top-k
 * candidates for each expanded node, the expert with the larger router score on
 * the left, following the top-k construction of a dynamically built tree.  The
 * paper fixes no further detail; this library grows the tree like this, per
 * sequence (all decisions on fp32 scores, ties to the lower node index):
 *
 *   jk_tree_grow      one depth.  For every frontier node f (in node order), expert
 *       e = left, right, rank j: a new node with token cand_tokens[f][e][j], parent f,
 *       score = score(f) * cand_probs[f][e][j] (the root scores 1), numbered in that
 *       order behind the existing nodes: children of a node are ordered left to right
 *       by index, the left expert's list first.  Nodes beyond max_nodes are dropped.
 *       The `width` best new nodes, in increasing index, are the next frontier (if there
 *       are fewer new nodes the remaining places repeat the first one).
 *   jk_tree_finalize  keeps the n_keep best nodes (a node never scores above its parent,
 *       so ancestors come along), renumbers them in increasing old index and translates
 *       the parents: tree_tokens / parent as jk_tree_verify_attention and jk_accept_path
 *       take them.  n_valid[b] = min(nodes grown, n_keep); places beyond it hold token -1.
 *   jk_gather_draft_probs  draft_probs[b][i][:] = q_all[q_row[b][i]][:], the dense array
 *       jk_accept_path takes (q_all: all draft distributions of the round, one row per
 *       (hidden state, head), e.g. the draft_probs outputs of the round's jk_draft_heads
 *       calls in one buffer; a row number outside [0, n_q_rows) is clamped).
 *
 * The state arrays are device memory owned by the caller: tokens, parent, q_row
 * int32 [batch][max_nodes], score fp32 [batch][max_nodes], n_nodes int32 [batch]
 * (zero before the first depth of a round).  q_row of a node is
 * q_row_base + 2 * (b * n_front + f) + e: the row of the distribution its token
 * was a candidate of, when the rows of the call's hidden states start at q_row_base.
 *   n_front      frontier nodes per sequence in this call (1 for the root: frontier_in NULL)
 *   top_k, width n_front * 2 * top_k <= 256, 1 <= width <= 256
 *   frontier_in  device int32 [batch][n_front] (the previous call's frontier_out) or NULL
 *   cand_tokens, cand_probs  device [batch * n_front][2][top_k] (jk_draft_heads' topk outputs
 *                for the hidden states of the frontier nodes, sequence-major)
 *   frontier_out device int32 [batch][width], written
 *   max_nodes    1..1024;  1 <= n_keep <= max_nodes;  old_index may be NULL */
typedef struct {
  int32_t* tokens;
  int32_t* parent;
  float* score;
  int32_t* q_row;
  int32_t* n_nodes;
  int32_t max_nodes;
} jk_tree_state;

jk_status jk_tree_grow(const jk_tree_state* state, int32_t batch, int32_t n_front, int32_t top_k, int32_t width,
                       int32_t q_row_base, const int32_t* frontier_in, const int32_t* cand_tokens,
                       const float* cand_probs, int32_t* frontier_out, void* hip_stream);

/* The last draft pass when jk_draft_heads ran in JK_HEADS_CONTRASTIVE mode (Section 3.2, Eq. 6-8:
 * the contrastive head predicts one position further than the mixture head from the same
 * features, which saves one pass of the draft model).  Reading: every frontier node gets the
 * first k1 candidates of its mixture list (head 0) as children; then each of the `width` best
 * children (ties to the lower index), in index order, gets the first k2 candidates of its
 * parent's contrastive list (head 1) as children.  All children are numbered before all
 * grandchildren; q_row is q_row_base + 2 (b n_front + f) for children and one more for
 * grandchildren.  cand_tokens / cand_probs as for jk_tree_grow with lists of top_k entries;
 * k1, k2 <= top_k, n_front * k1 <= 256, width * k2 <= 256. */
jk_status jk_tree_grow_tail(const jk_tree_state* state, int32_t batch, int32_t n_front, int32_t top_k, int32_t k1,
                            int32_t k2, int32_t width, int32_t q_row_base, const int32_t* frontier_in,
                            const int32_t* cand_tokens, const float* cand_probs, void* hip_stream);

/* One depth of a PREDEFINED tree shape (Section 3.1.2: the two candidate lists can also fill
 * a static tree): new node j (j < n_new, appended in this order) hangs under frontier node
 * frontier_in[b][shape_slot[j]] and takes candidate shape_rank[j] of that node's list of
 * expert shape_expert[j] (0 = left, 1 = right); score and q_row as in jk_tree_grow.  The
 * shape arrays are device int32 [n_new], the same for every sequence (entries outside their
 * ranges are clamped).  frontier_out[b][i] (may be NULL with n_next = 0) is the index of new
 * node next_index[i]: the parents of the next depth; new_ids (device int32 [batch][n_new], may
 * be NULL) receives the indices of all new nodes (-1 for nodes dropped at max_nodes).
 * n_new <= 4096. */
jk_status jk_tree_fill_static(const jk_tree_state* state, int32_t batch, int32_t n_front, int32_t top_k,
                              int32_t q_row_base, const int32_t* frontier_in, const int32_t* cand_tokens,
                              const float* cand_probs, const int32_t* shape_slot, const int32_t* shape_expert,
                              const int32_t* shape_rank, int32_t n_new, const int32_t* next_index, int32_t n_next,
                              int32_t* frontier_out, int32_t* new_ids, void* hip_stream);

jk_status jk_tree_finalize(const jk_tree_state* state, int32_t batch, int32_t n_keep, int32_t* tree_tokens,
                           int32_t* parent, int32_t* q_row, int32_t* old_index, int32_t* n_valid, void* hip_stream);

jk_status jk_gather_draft_probs(int32_t batch, int32_t n_tree, int32_t vocab, const float* q_all, int64_t n_q_rows,
                                const int32_t* q_row, float* draft_probs, void* hip_stream);

/* The draft layer's remaining dense pieces (Section 3.1.1: a reduction layer in front of one
 * decoder attention layer; Eq. 1: u = Attn(h) + h) are plain linear layers on few rows around
 * jk_tree_verify_attention:  out = x . w^T (+ residual), bf16 operands, fp32 accumulation, on
 * the same weight-streaming MFMA kernel as the heads and the experts.
 *   m 1..256 rows;  k a multiple of 128;  n >= 1
 *   x        device bf16 [m][k];  w device bf16 [n][k];  both 16-byte aligned
 *   residual device bf16 [m][n], added in fp32; may be NULL
 *   out_bf16 device bf16 [m][n] (one rounding) and/or out_f32 device fp32 [m][n]; at least one
 *   workspace jk_linear_workspace(m, n, k) bytes, 256-byte aligned */
size_t jk_linear_workspace(int32_t m, int32_t n, int32_t k);

jk_status jk_linear(int32_t m, int32_t n, int32_t k, const void* x, const void* w, const void* residual,
                    void* out_bf16, float* out_f32, void* workspace, size_t workspace_bytes, void* hip_stream);

/* Zero-fills a workspace with a small kernel on `hip_stream` (safe under HIP-graph
 * capture).  Needed once per workspace before its first jk_accept_path or
 * jk_tree_verify_attention(_paged) call: the cooperative sampling walk synchronises
 * its workgroups through tagged words in the workspace and relies on tags only ever
 * growing, the attention kernel counts the arrivals of a row tile's key splits in
 * words that every call returns to zero, and the error word is sticky.  Returns
 * JK_ERR_WORKSPACE for a null or misaligned pointer. */
jk_status jk_workspace_init(void* workspace, size_t workspace_bytes, void* hip_stream);

/* Device-side findings of the calls that used `workspace` (an attention or acceptance
 * workspace) since it was last zero-filled: the OR of the JK_DEVERR_* bits below, or -1 if
 * the word cannot be read.  Synchronous: copies one word from the device (hipMemcpy), so call
 * it after the work of interest has been synchronised, never under stream capture.  The word
 * is sticky; jk_workspace_init clears it.  (The tree of Section 3.1.2 and the token ids live in
 * device memory, so the host-side checks of the entry points cannot see them: a kernel that
 * meets a bad entry repairs it - parent -1, token or page id clamped - and records the fact.) */
#define JK_DEVERR_BAD_TREE 1    /* a parent[] entry outside [-1, i-1] was treated as -1 */
#define JK_DEVERR_BAD_TOKEN 2   /* a token id outside [0, vocab) was clamped (sampling walk) */
#define JK_DEVERR_BAD_PAGE 4    /* a block-table entry outside [0, n_pages) was clamped */
#define JK_DEVERR_MERGE_WAIT 8  /* attention: a workgroup stopped waiting for its key splits' partners; the
                                   result is still complete once every workgroup has run (the last one to
                                   arrive merges what the others left), but the call was slow */
#define JK_DEVERR_WALK_WAIT 16  /* sampling walk: a tree's workgroups did not meet; accept_len = -1 for it */
int32_t jk_last_device_error(const void* workspace);

/* How the next jk_tree_verify_attention(_paged) call with this descriptor and bound would be cut
 * into workgroups on the current device (for reports and tests; the plan is the library's own
 * business and may change): plan_out[0..5] = waves along the query rows, waves along the keys,
 * 32-key tiles per wave and round, row tiles, key splits, 1 if the splits are merged inside the
 * attention kernel (0: by a second kernel; always 0 for the fp32 path and for one split). */
jk_status jk_tree_verify_attention_plan(const jk_attn_desc* desc, int32_t max_prefix_len, int32_t* plan_out);

/* Once per device and process, before the first jk_tree_verify_attention call that should merge
 * its key splits inside the attention kernel: launches a small probe on `hip_stream` that records
 * on which XCD consecutive workgroups run, WAITS for it (the only call besides
 * jk_last_device_error that synchronises), and remembers the answer for the current device.  The
 * merge inside the kernel lets the workgroups of one row tile meet in one XCD's L2 and is only
 * used on a device where workgroups n and n + 8 were seen to share an XCD; without jk_init (or
 * where the probe says otherwise) attention uses a second, merging kernel launch instead - same
 * results, bit for bit.  Must not be called under stream capture.  Returns JK_ERR_HIP on failure. */
jk_status jk_init(void* hip_stream);

/* Overrides for experiments and tests; nothing in normal use needs them.  The library's launch
 * plans are functions of the descriptors and the device; these knobs force parts of them.
 * Process-wide, not thread-safe against concurrent calls.  Names: "attn_wm", "attn_wn" (wave
 * arrangement of the bf16 attention kernel: 4x1 or 2x2; 0 = automatic), "attn_splits" (key
 * splits, 0 = automatic), "attn_fused" (-1 automatic, 0 never merge inside the kernel, 1 whenever
 * the grid allows it), "attn_deep" (-1 automatic, 0 never use the deeper K/V ring of the 2x2
 * arrangement, 1 whenever one workgroup per CU is planned), "accept_single" (1: one-workgroup sampling walk), "spin_limit" (polls of
 * the bounded waits; -1 default, 0 = give up at once: the give-up paths run with every kernel
 * ending normally), "verbose" (1: print attention plans to stderr).  The same knobs are seeded
 * once, when the library is loaded, from the environment variables JK_ATTN_WM, JK_ATTN_WN,
 * JK_ATTN_SPLITS, JK_ATTN_FUSED, JK_ATTN_DEEP, JK_ACCEPT_SINGLE, JK_SPIN_LIMIT, JK_ATTN_VERBOSE.  With an
 * override in force jk_tree_verify_attention_workspace answers for the forced plan.
 * Returns JK_ERR_INVALID_ARG for an unknown name. */
jk_status jk_set_tuning(const char* name, int32_t value);

/* Measurement aid, not part of the method: enqueues a kernel that only streams `bytes`
 * bytes (device, 16-byte aligned) with 128-bit loads.  Timing it gives the ceiling that an
 * HBM-bound call of the same size (for instance one attention layer's K/V) can be compared
 * with on the machine at hand.  `sink` is a device word that is written only if the data
 * hash to one particular value. */
jk_status jk_stream_read_probe(const void* src, size_t bytes, void* sink, void* hip_stream);

/* Host-side check of a tree held in host memory: JK_OK, JK_ERR_BAD_TREE
 * (some parent[i] outside [-1, i-1]) or JK_ERR_INVALID_ARG (null, n outside
 * [1, JK_MAX_TREE]). */
jk_status jk_validate_tree(const int32_t* parent_host, int32_t n_tree);

/* Static, NUL-terminated description of a status code. */
const char* jk_status_string(int32_t status);

/* Library version, "major.minor". */
const char* jk_version(void);

#ifdef __cplusplus
}
#endif
#endif /* JAKIRO_VERIFY_H */
