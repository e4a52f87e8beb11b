/*
 * omnisparse.h -- C ABI of the MI355X (gfx950) OmniSparse hot-path library.
 *
 * One transformer layer's sparse attention as defined by arxiv 2511.12201
 * ("OmniSparse"): lazy/active query classification, KV selection under one
 * token budget set by the flattest head, sparse prefill attention (forward and
 * backward) and a decode step that fetches visual KV only for heads whose
 * decoding query is active.
 *
 * General rules (all entry points)
 *   - Every tensor pointer is a DEVICE pointer owned by the caller unless the
 *     comment says "host".  The library allocates and frees no device memory:
 *     scratch comes from the caller's workspace `ws` of `ws_bytes` bytes, whose
 *     required size is returned by omni_workspace_bytes().  The workspace
 *     content is unspecified between calls.  `ws` must be 256-byte aligned.
 *   - `stream` is a hipStream_t passed as void*.  Calls only enqueue work on
 *     that stream and return; results are valid once the stream has been
 *     synchronised.  Nothing else orders the work.
 *   - Data-dependent scalars (kept-query counts, the budget b) live in device
 *     memory and are consumed from there by later calls, so the pipeline needs
 *     no host synchronisation.
 *   - Layout: Q, O, dO, dQ are [batch, n_q_heads, n_tokens, head_dim]; K, V,
 *     dK, dV are [batch, n_kv_heads, n_tokens, head_dim]; head_dim is
 *     contiguous, the other strides are given in elements in the descriptor.
 *     Outputs O, dQ, dK, dV use the same strides as Q resp. K.  Query head i
 *     reads KV head i / (n_q_heads / n_kv_heads).
 *   - Heads and tokens are 0-based; the paper's "first attention head" is
 *     head 0 and its "first token" (attention sink) is `sink_index`.
 *   - Return value: OMNI_OK, or a negative omni_status.  On error nothing has
 *     been enqueued; omni_last_error() gives a message (thread local).
 *     Arguments are validated on the host before any launch: null pointers,
 *     n_q_heads % n_kv_heads, head_dim in {64, 128}, 0 <= vis_begin < vis_end
 *     <= n_tokens, 0 <= sink_index < n_tokens, strides at least the natural
 *     ones and multiples of 8 elements, workspace size and alignment.
 *   - Deterministic: equal inputs give bit-equal outputs (no floating-point
 *     atomics anywhere).
 */
#ifndef OMNISPARSE_H
#define OMNISPARSE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { OMNI_F32 = 0, OMNI_BF16 = 1 } omni_dtype;

typedef enum {
  OMNI_OK = 0,
  OMNI_ERR_INVALID = -1,      /* bad argument value or null pointer            */
  OMNI_ERR_UNSUPPORTED = -2,  /* shape / dtype outside what the kernels handle */
  OMNI_ERR_WORKSPACE = -3,    /* workspace too small or misaligned             */
  OMNI_ERR_HIP = -4           /* a HIP runtime call failed                     */
} omni_status;

/* Identifiers for omni_workspace_bytes(). */
typedef enum {
  OMNI_CALL_SCORE_QUERIES = 0,
  OMNI_CALL_SELECT_QUERIES = 1,
  OMNI_CALL_KV_BUDGET = 2,
  OMNI_CALL_SELECT_KV = 3,
  OMNI_CALL_SPARSE_ATTN_FWD = 4,
  OMNI_CALL_SPARSE_ATTN_BWD = 5,
  OMNI_CALL_SLIM_DECODE = 6,
  OMNI_CALL_DENSE_ATTN_FWD = 7,
  OMNI_CALL_DENSE_DECODE = 8,
  OMNI_CALL_GROUP_SUBSET = 9,
  OMNI_CALL_BLOCK_SCORES = 10,
  OMNI_CALL_PREFILL_SELECT = 11,
  OMNI_CALL_BLOCK_ATTN_FWD = 12,
  OMNI_CALL_BLOCK_ATTN_BWD = 13
} omni_call_id;

/* One attention layer during prefill / training.
 * Visual tokens are [vis_begin, vis_end) (paper Sec. "Overview": X = [X_v, X_t]);
 * every other token is text. */
typedef struct {
  int32_t batch, n_q_heads, n_kv_heads, head_dim, n_tokens;
  int32_t vis_begin, vis_end, sink_index;
  int32_t causal;              /* 1: token n attends tokens <= n (Sec. "Preliminary") */
  int32_t dtype;               /* omni_dtype of Q, K, V, O, dO, dQ, dK, dV */
  float softmax_scale;         /* 1 / sqrt(head_dim) in the paper's attention equation */
  int64_t q_stride[3];         /* batch, head, token strides of Q-shaped tensors, in elements */
  int64_t kv_stride[3];        /* same for K/V-shaped tensors */
} omni_layer_desc;

/* KV cache during decode: rows [0, ctx_len[b]) of each sequence are valid;
 * [vis_begin, vis_end) is the visual segment K^v, the rest text K^t and
 * decoded answer K^a (Sec. "KV Cache Slimming"). */
typedef struct {
  int32_t batch, n_q_heads, n_kv_heads, head_dim, cache_capacity;
  int32_t vis_begin, vis_end;
  int32_t dtype;               /* omni_dtype of q, Kcache, Vcache, O */
  float softmax_scale;
  float tau;                   /* lazy/active threshold of the query-mask equation */
  int64_t kv_stride[3];        /* batch, head, token strides of the caches, in elements */
  int32_t static_lists;        /* omni_slim_decode / omni_slim_decode_prepare only.  1: the lists are fixed after
                                  prefill (Sec. "KV Cache Slimming") and omni_slim_decode_prepare has merged them
                                  per KV group into the workspace that omni_slim_decode is given; the call reads
                                  a stored row once per group, as omni_slim_decode_grouped does, and ignores the
                                  contents of vis_idx / vis_cnt.  Which heads are active is still decided on every
                                  call.  0: the lists are read anew on every call. */
} omni_decode_desc;

/* Paged form of the compacted visual KV store (omni_compact_cache_paged,
 * omni_slim_decode_paged): one pool of fixed-size pages shared by all sequences and
 * KV heads of a layer, and a table that says which page holds which stretch of a
 * (sequence, KV head) pair's group list. */
typedef struct {
  void* K;                     /* device, [n_pages, page_rows, head_dim] dtype of the decode descriptor */
  void* V;                     /* same shape */
  const int32_t* page_table;   /* device, [batch, n_kv_heads, pages_cap]: page of the pool that holds list
                                  positions [j * page_rows, (j + 1) * page_rows) of the pair's group list;
                                  an entry outside [0, n_pages) marks a page that is not there */
  int32_t n_pages;             /* pages in the pool; n_pages * page_rows < 2^31 */
  int32_t page_rows;           /* rows per page, a power of two */
  int32_t pages_cap;           /* table entries per pair; pages_cap * page_rows >= u_cap of the call */
} omni_page_pool;

/*
 * omni_score_queries -- Sec. "Query Selection as Binary Lazy-Active
 * Classification", probe-softmax equation.
 * For every KV head: probe_keys[.,.,0,:] = K[sink_index] (lazy reference),
 * probe_keys[.,.,1,:] = mean of the visual keys (active reference).
 * For every query head and token: scores = second column of the two-way
 * softmax of (q . k_lazy, q . k_act) * softmax_scale, i.e. the probability of
 * the active class.  Accumulation in fp32.
 *   probe_keys [batch, n_kv_heads, 2, head_dim] f32, out
 *   scores     [batch, n_q_heads, n_tokens] f32, out (all tokens are scored;
 *              only the visual ones are classified later)
 */
int omni_score_queries(const omni_layer_desc* desc, const void* Q, const void* K,
                       float* probe_keys, float* scores,
                       void* ws, size_t ws_bytes, void* stream);

/*
 * omni_select_queries -- same section, query-mask equation.
 * mode 0: a visual query is kept iff scores > param (param = tau, strict).
 * mode 1: the ceil(param * n_visual) visual queries of highest score are kept
 *         per head (equal scores: lower token index first); 0 < param <= 1.
 * Head 0 keeps every query; non-visual queries are always kept.
 *   q_idx [batch, n_q_heads, n_tokens] i32, out: kept token indices, ascending;
 *         entries at and beyond the count are unspecified
 *   q_cnt [batch, n_q_heads] i32, out
 */
int omni_select_queries(const omni_layer_desc* desc, const float* scores,
                        int mode, float param, int32_t* q_idx, int32_t* q_cnt,
                        void* ws, size_t ws_bytes, void* stream);

/*
 * omni_kv_budget -- Sec. "KV Selection with Head-level Dynamic Budget
 * Allocation" (accumulated key score, kurtosis, budget equation) with the
 * block-wise probe of the paragraph "Block-wise probing and sparse flash
 * attention kernel".
 * key_scores[i,k] = sum over pooled query blocks j (probe_block consecutive
 * tokens, all queries) of w_j * softmax_k(mean_q(j) . K[k] * scale), w_j = rows
 * in block j; under the causal mask block j sees keys up to its last token.
 * kurtosis[i] = m4 / m2^2 - 3 of key_scores[i,:] (fp64; -2 when m2 == 0).
 * flattest = arg min kurtosis (lowest index on ties).
 * budget = min { b : sum of the b largest key_scores[flattest] >= recall_p * n_tokens }
 * (budget_mode 0, the paper's rule) or the maximum over heads of each head's own
 * such b (budget_mode 1).  recall[i] = mass of head i's b largest scores / n_tokens.
 * budget_mode 2 gives every head the budget of its own scores (b_i = the same
 * minimum taken on key_scores[i]): the per-head alternative that the paper's
 * introduction and this section set aside as too slow.  budget and budget_host
 * then hold [batch, n_q_heads] entries, recall[i] is the mass of head i's b_i
 * largest scores, and the *_per_head entry points below consume the result.
 *   key_scores [batch, n_q_heads, n_tokens] f32, out
 *   kurtosis   [batch, n_q_heads] f64, out
 *   flattest   [batch] i32, out
 *   budget     [batch] i32, out (device); [batch, n_q_heads] in budget_mode 2
 *   recall     [batch, n_q_heads] f32, out
 *   budget_host: optional pinned HOST pointer, same shape as budget; if not null
 *                the budget is also copied there (valid after the stream is
 *                synchronised).
 * 0 < recall_p <= 1, probe_block >= 1.
 */
int omni_kv_budget(const omni_layer_desc* desc, const void* Q, const void* K,
                   float recall_p, int probe_block, int budget_mode,
                   float* key_scores, double* kurtosis, int32_t* flattest,
                   int32_t* budget, float* recall, int32_t* budget_host,
                   void* ws, size_t ws_bytes, void* stream);

/*
 * omni_budget_from_scores -- the second half of omni_kv_budget on key scores
 * the caller already holds (same section: kurtosis, flattest head, budget
 * equation, per-head recall).  Arguments as in omni_kv_budget; key_scores is an
 * input here.
 */
int omni_budget_from_scores(const omni_layer_desc* desc, const float* key_scores,
                            float recall_p, int budget_mode,
                            double* kurtosis, int32_t* flattest, int32_t* budget, float* recall,
                            void* ws, size_t ws_bytes, void* stream);

/*
 * omni_prefill_select -- the four selection calls of a prefill step in one:
 * omni_score_queries, omni_select_queries, omni_kv_budget and omni_select_kv
 * (omni_select_kv_per_head when budget_mode is 2), i.e. Sec. "Query Selection"
 * (probe-softmax and query-mask equations) followed by Sec. "KV Selection"
 * (accumulated key score, kurtosis, budget and key-mask equations).  Every
 * output is bit-identical to what the separate calls write on the same inputs;
 * the fused call reads Q once for both the query scores and the pooled queries,
 * and compacts the key lists from the per-head cut that the recall computation
 * already finds, instead of searching it again.
 * Arguments and outputs as in the separate calls (q_mode, q_param: mode and
 * param of omni_select_queries), with one difference: recall[i] is the mass of
 * the min(budget, b_cap) keys that are actually selected, which is the recall
 * of omni_kv_budget whenever b_cap >= budget.
 * Workspace: OMNI_CALL_PREFILL_SELECT with param = probe_block.
 */
int omni_prefill_select(const omni_layer_desc* desc, const void* Q, const void* K,
                        int q_mode, float q_param,
                        float recall_p, int probe_block, int budget_mode,
                        float* probe_keys, float* scores, int32_t* q_idx, int32_t* q_cnt,
                        float* key_scores, double* kurtosis, int32_t* flattest,
                        int32_t* budget, float* recall,
                        int32_t* kv_idx, int32_t b_cap,
                        void* ws, size_t ws_bytes, void* stream);

/*
 * omni_sparse_prefill -- a whole prefill step in one call: omni_prefill_select
 * followed by omni_sparse_attn_fwd (the _per_head forms when budget_mode is 2),
 * i.e. Sec. "Query Selection", Sec. "KV Selection" and the sparse attention of
 * Sec. "Preliminary" under the two masks.  Every output (the selection's arrays,
 * O and lse) is bit-identical to what the two calls write.  What the fusion
 * changes is the hand-over between them: the kernel that gathers each head's
 * selected K and V rows into the attention's tile layout forms the key lists
 * itself, from the accumulated key scores and the head's cut (key-mask
 * equation), and writes kv_idx on the way; the list is neither written by a
 * pass of its own nor read back.
 * Arguments: as in omni_prefill_select, then V, O and lse as in
 * omni_sparse_attn_fwd.
 * Workspace: omni_sparse_prefill_workspace_bytes(desc, probe_block, b_cap)
 * (the two calls' workspaces one after the other); 0 with a message in
 * omni_last_error on invalid arguments.
 */
size_t omni_sparse_prefill_workspace_bytes(const omni_layer_desc* desc, int32_t probe_block,
                                           int32_t b_cap);
int omni_sparse_prefill(const omni_layer_desc* desc, const void* Q, const void* K, const void* V,
                        int q_mode, float q_param,
                        float recall_p, int probe_block, int budget_mode,
                        float* probe_keys, float* scores, int32_t* q_idx, int32_t* q_cnt,
                        float* key_scores, double* kurtosis, int32_t* flattest,
                        int32_t* budget, float* recall,
                        int32_t* kv_idx, int32_t b_cap,
                        void* O, float* lse,
                        void* ws, size_t ws_bytes, void* stream);

/*
 * omni_prefill_select_varlen -- omni_prefill_select for sequences of different
 * lengths in one padded batch: sequence b occupies rows [0, seq_tokens[b]) of its
 * slab of Q and K, its visual tokens are [seq_vis_begin[b], seq_vis_end[b]), and
 * everything the selection computes for it (probe keys, scores, kept queries,
 * accumulated key scores, kurtosis, flattest head, budget, recall, key lists) is
 * what omni_prefill_select gives on that sequence alone, bit for bit.  desc
 * describes the padded batch (n_tokens = the padded length; its vis_begin / vis_end
 * are not used; sink_index is common and must lie inside every sequence).
 *   seq_tokens, seq_vis_begin, seq_vis_end: [batch] i32, HOST pointers, read
 *   before the call returns.
 * Outputs have the padded batch's shapes ([batch, n_q_heads, n_tokens] for scores,
 * q_idx and key_scores, as omni_sparse_attn_fwd / _bwd take them); rows and list
 * entries beyond a sequence's length / counts are unspecified.  The kernels of a
 * sequence are sized to that sequence and are launched sequence after sequence on
 * the caller's stream.  Padding rows of Q and K are never read.
 * Workspace: OMNI_CALL_PREFILL_SELECT with param = probe_block (as for the padded
 * length; one sequence uses it at a time).
 */
int omni_prefill_select_varlen(const omni_layer_desc* desc, const void* Q, const void* K,
                               const int32_t* seq_tokens, const int32_t* seq_vis_begin,
                               const int32_t* seq_vis_end,
                               int q_mode, float q_param, float recall_p, int probe_block,
                               int budget_mode,
                               float* probe_keys, float* scores, int32_t* q_idx, int32_t* q_cnt,
                               float* key_scores, double* kurtosis, int32_t* flattest,
                               int32_t* budget, float* recall, int32_t* kv_idx, int32_t b_cap,
                               void* ws, size_t ws_bytes, void* stream);

/*
 * omni_select_kv -- same section, key-mask equation (value mask = key mask).
 * Per head the min(budget, b_cap) keys of largest key_scores; when several keys
 * share the cut value those of lower token index are taken.
 *   kv_idx [batch, n_q_heads, b_cap] i32, out: ascending; entries beyond the
 *          budget are unspecified
 */
int omni_select_kv(const omni_layer_desc* desc, const float* key_scores, const int32_t* budget,
                   int32_t b_cap, int32_t* kv_idx,
                   void* ws, size_t ws_bytes, void* stream);

/*
 * omni_select_kv_per_head, omni_sparse_attn_fwd_per_head,
 * omni_sparse_attn_bwd_per_head, omni_visual_subset_per_head,
 * omni_group_subset_per_head -- the calls of the
 * same names without the suffix, with one budget per head instead of one per
 * batch item (same section: the key-mask equation holds per head for any b; the
 * paper shares one b between the heads to save the per-head search, the
 * budget_mode 2 of omni_kv_budget does that search).
 *   budget [batch, n_q_heads] i32 (device): head i keeps, attends and stores
 *   min(budget[batch, i], b_cap) keys; kv_idx keeps its [batch, n_q_heads, b_cap]
 *   layout, so b_cap bounds the largest head.
 * Everything else (arguments, outputs, workspace sizes by the same call ids,
 * errors) is as in the unsuffixed call.
 */
int omni_select_kv_per_head(const omni_layer_desc* desc, const float* key_scores, const int32_t* budget,
                            int32_t b_cap, int32_t* kv_idx,
                            void* ws, size_t ws_bytes, void* stream);
int omni_sparse_attn_fwd_per_head(const omni_layer_desc* desc, const void* Q, const void* K, const void* V,
                                  const int32_t* q_idx, const int32_t* q_cnt,
                                  const int32_t* kv_idx, const int32_t* budget, int32_t b_cap,
                                  void* O, float* lse,
                                  void* ws, size_t ws_bytes, void* stream);
int omni_sparse_attn_bwd_per_head(const omni_layer_desc* desc, const void* Q, const void* K, const void* V,
                                  const void* O, const void* dO, const float* lse,
                                  const int32_t* q_idx, const int32_t* q_cnt,
                                  const int32_t* kv_idx, const int32_t* budget, int32_t b_cap,
                                  void* dQ, void* dK, void* dV,
                                  void* ws, size_t ws_bytes, void* stream);
int omni_visual_subset_per_head(const omni_layer_desc* desc, const int32_t* kv_idx, const int32_t* budget,
                                int32_t b_cap, int32_t* vis_idx, int32_t* vis_cnt, void* stream);
int omni_group_subset_per_head(const omni_layer_desc* desc, const int32_t* kv_idx, const int32_t* budget,
                               int32_t b_cap, int32_t* grp_idx, uint32_t* grp_mask, int32_t* grp_cnt,
                               int32_t u_cap, void* ws, size_t ws_bytes, void* stream);

/*
 * omni_sparse_attn_fwd -- Sec. "Preliminary" (attention equation restricted by
 * the masks M^Q, M^K, M^V) for the kept queries and selected keys.
 * For head i and kept query n: softmax over {k in kv_idx[i] : k <= n} (all of
 * kv_idx[i] when not causal) of q_n . k_k * scale, times V.  Queries that are
 * not kept, and kept queries with no admissible key, get an all-zero output row
 * and lse = -inf.  bf16 inputs: Q K^T on the bf16 matrix cores, softmax in fp32,
 * the weights rounded to f16 and multiplied with V on the f16 matrix cores (fp32
 * accumulation); V is converted to f16 on the way, which is exact for magnitudes
 * in [2^-14, 65504]; larger magnitudes saturate at 65504, smaller ones keep an
 * absolute accuracy of 3e-8.  The dense baseline and the block-list calls share
 * the kernel and the limit.
 *   q_idx/q_cnt as written by omni_select_queries, kv_idx/budget as written by
 *   omni_select_kv / omni_kv_budget (both index lists ascending); the effective
 *   number of keys per head is min(budget[batch], b_cap).
 *   O   [batch, n_q_heads, n_tokens, head_dim] dtype, out (fully written)
 *   lse [batch, n_q_heads, n_tokens] f32, out: natural-log sum of exp of the
 *       scaled logits over the admissible keys
 */
int omni_sparse_attn_fwd(const omni_layer_desc* desc, const void* Q, const void* K, const void* V,
                         const int32_t* q_idx, const int32_t* q_cnt,
                         const int32_t* kv_idx, const int32_t* budget, int32_t b_cap,
                         void* O, float* lse,
                         void* ws, size_t ws_bytes, void* stream);

/*
 * omni_sparse_attn_bwd -- gradient of omni_sparse_attn_fwd with the index sets
 * held constant (the paper trains with the same sparse attention and defines no
 * gradient through the selection): dV = P^T dO, dP = dO V^T,
 * dS = P (dP - rowsum(dO O)), dQ = dS K scale, dK = dS^T Q scale, with dK, dV
 * summed over the query heads of a KV group.
 *   O, lse: outputs of the forward call on the same inputs
 *   dQ [like Q], dK, dV [like K], out, fully written (zero rows where nothing
 *   was kept / selected)
 */
int omni_sparse_attn_bwd(const omni_layer_desc* desc, const void* Q, const void* K, const void* V,
                         const void* O, const void* dO, const float* lse,
                         const int32_t* q_idx, const int32_t* q_cnt,
                         const int32_t* kv_idx, const int32_t* budget, int32_t b_cap,
                         void* dQ, void* dK, void* dV,
                         void* ws, size_t ws_bytes, void* stream);

/*
 * omni_slim_decode -- Sec. "KV Cache Slimming", decoding-attention equation.
 * Per head the decoding query is scored against probe_keys as in
 * omni_score_queries; the head is active iff score > tau or it is head 0.  An
 * active head attends its stored visual rows vis_idx[i, 0:vis_cnt[i]) (those
 * below ctx_len), a lazy head none of the visual rows; every head attends all
 * non-visual rows below ctx_len.
 *   q       [batch, n_q_heads, head_dim] dtype, contiguous
 *   Kcache, Vcache [batch, n_kv_heads, cache_capacity, head_dim] dtype (strides in desc)
 *   ctx_len [batch] i32
 *   probe_keys [batch, n_kv_heads, 2, head_dim] f32 (from prefill)
 *   vis_idx [batch, n_q_heads, b_cap] i32, vis_cnt [batch, n_q_heads] i32
 *   O       [batch, n_q_heads, head_dim] dtype, out
 *   active  [batch, n_q_heads] u8, out
 */
int omni_slim_decode(const omni_decode_desc* desc, const void* q,
                     const void* Kcache, const void* Vcache, const int32_t* ctx_len,
                     const float* probe_keys,
                     const int32_t* vis_idx, const int32_t* vis_cnt, int32_t b_cap,
                     void* O, uint8_t* active,
                     void* ws, size_t ws_bytes, void* stream);

/*
 * omni_slim_decode_prepare -- once after prefill, and again whenever the lists
 * change: merges the per-head lists of every KV group (ascending union with a
 * membership bit per head, as omni_group_subset builds it from kv_idx) into the
 * workspace, behind the partial states of the decode call.  The omni_slim_decode
 * calls that follow with static_lists = 1, the same shapes and this workspace then
 * read every stored row once per group.  The merged lists live in the caller's
 * memory and nowhere else: between this call and the decode calls that rely on it
 * no other call may be given the workspace (the stateless omni_slim_decode and the
 * other decode calls write their partial states over it), and a workspace that was
 * freed and allocated again has to be prepared again.  desc must have
 * static_lists = 1.  Groups wider than 32 heads have no membership word: the call
 * does nothing and omni_slim_decode reads the per-head lists.
 * Workspace: OMNI_CALL_SLIM_DECODE for this descriptor (it includes the lists).
 */
int omni_slim_decode_prepare(const omni_decode_desc* desc,
                             const int32_t* vis_idx, const int32_t* vis_cnt, int32_t b_cap,
                             void* ws, size_t ws_bytes, void* stream);

/*
 * omni_visual_subset -- helper for the hand-over from prefill to decode
 * (Sec. "KV Cache Slimming": the selected KV pairs are stored at token level).
 * Copies, per head, the entries of kv_idx that are visual tokens to vis_idx and
 * writes their number to vis_cnt.
 *   vis_idx [batch, n_q_heads, b_cap] i32, out; vis_cnt [batch, n_q_heads] i32, out
 */
int omni_visual_subset(const omni_layer_desc* desc, const int32_t* kv_idx, const int32_t* budget,
                       int32_t b_cap, int32_t* vis_idx, int32_t* vis_cnt, void* stream);

/*
 * omni_group_subset / omni_slim_decode_grouped -- the same decode step (Sec. "KV
 * Cache Slimming", decoding-attention equation) with the stored visual rows kept
 * per KV group instead of per query head.  Under grouped-query attention the heads
 * of a group index one shared cache; the group list is the ascending union of the
 * visual entries of its heads' kv_idx lists, with bit j of grp_mask set iff query
 * head (group * G + j) selected that token (G = n_q_heads / n_kv_heads <= 32).  A
 * decode step loads a listed row once if any ACTIVE head of the group stores it and
 * lets exactly the heads that store it attend it, so the output equals
 * omni_slim_decode on the per-head lists.
 *   grp_idx  [batch, n_kv_heads, u_cap] i32, grp_mask [batch, n_kv_heads, u_cap] u32,
 *   grp_cnt  [batch, n_kv_heads] i32 (the true union size; entries beyond u_cap are
 *   dropped, so pass u_cap >= vis_end - vis_begin to be safe)
 * omni_group_subset needs a workspace (OMNI_CALL_GROUP_SUBSET);
 * omni_slim_decode_grouped the one of OMNI_CALL_SLIM_DECODE.
 */
int omni_group_subset(const omni_layer_desc* desc, const int32_t* kv_idx, const int32_t* budget,
                      int32_t b_cap, int32_t* grp_idx, uint32_t* grp_mask, int32_t* grp_cnt,
                      int32_t u_cap, void* ws, size_t ws_bytes, void* stream);
int omni_slim_decode_grouped(const omni_decode_desc* desc, const void* q,
                             const void* Kcache, const void* Vcache, const int32_t* ctx_len,
                             const float* probe_keys,
                             const int32_t* grp_idx, const uint32_t* grp_mask, const int32_t* grp_cnt,
                             int32_t u_cap, void* O, uint8_t* active,
                             void* ws, size_t ws_bytes, void* stream);

/*
 * omni_slim_decode_grouped_static -- omni_slim_decode_grouped for callers that
 * cannot allocate or carry a workspace: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments without ws / ws_bytes,
 * same kernels, same output bits.  The partial softmax states go to a buffer the
 * library holds in device memory (a file-scope __device__ array of
 * omni_static_scratch_bytes() = 16 MiB, one copy on every GPU the library runs on,
 * kept until the process ends).  The call allocates and frees nothing; the first
 * call on a device looks the buffer's address up once.
 * Errors: OMNI_ERR_WORKSPACE if the shape needs more scratch than the buffer holds
 * (omni_workspace_bytes(OMNI_CALL_SLIM_DECODE, desc, 0) > omni_static_scratch_bytes());
 * use omni_slim_decode_grouped then.  All calls on one GPU share the buffer: two
 * calls that overlap in time on the same GPU (different streams or threads) race.
 * Nothing of an earlier call's contents is relied on or needs clearing.
 */
int omni_slim_decode_grouped_static(const omni_decode_desc* desc, const void* q,
                                    const void* Kcache, const void* Vcache, const int32_t* ctx_len,
                                    const float* probe_keys,
                                    const int32_t* grp_idx, const uint32_t* grp_mask,
                                    const int32_t* grp_cnt, int32_t u_cap, void* O, uint8_t* active,
                                    void* stream);
size_t omni_static_scratch_bytes(void);

/*
 * Block-granular variant of the KV selection -- Sec. "Block-wise probing and sparse
 * flash attention kernel" as the paper runs it: queries AND keys are mean-pooled in
 * blocks of `block` tokens, the pooled map gives one accumulated score per key block
 * (a key block of c tokens enters a row's softmax with weight c; under the causal
 * mask query block j sees key blocks 0..j; row j counts for its number of queries).
 *
 * omni_block_scores writes block_scores [batch, n_q_heads, n_blocks] f32,
 * n_blocks = ceil(n_tokens / block) <= 2048, normalised to sum to n_blocks per head,
 * so that omni_budget_from_scores and omni_select_kv run on them unchanged with a
 * descriptor whose n_tokens is n_blocks (budget and lists are then in blocks).
 * Workspace: OMNI_CALL_BLOCK_SCORES with param = block.
 *
 * omni_expand_blocks turns ascending block lists blk_idx [batch, n_q_heads, blk_cap]
 * (blk_budget [batch] entries used) into ascending token lists kv_idx [batch,
 * n_q_heads, b_cap] and writes budget [batch] = min(blk_budget, blk_cap) * block; the
 * tokens a partial last block lacks become pad entries that no query ever sees under
 * the causal mask (without it n_tokens must be a multiple of block).
 * b_cap must be >= blk_cap * block to hold every list.
 */
int omni_block_scores(const omni_layer_desc* desc, const void* Q, const void* K, int32_t block,
                      float* block_scores, void* ws, size_t ws_bytes, void* stream);
int omni_expand_blocks(const omni_layer_desc* desc, const int32_t* blk_idx, const int32_t* blk_budget,
                       int32_t blk_cap, int32_t block, int32_t* kv_idx, int32_t* budget, int32_t b_cap,
                       void* stream);

/*
 * omni_block_attn_fwd -- the sparse flash attention kernel of Sec. "Block-wise
 * probing and sparse flash attention kernel" on block lists, with no gathered copy
 * of K/V: K and V are laid out once per KV head in token order, and every query
 * head's kernel walks its own list of selected blocks inside that one copy, so the
 * heads of a group share it.  Same result as omni_expand_blocks followed by
 * omni_sparse_attn_fwd (same tile engine, same order of accumulation).
 *
 * bf16 only; block must be a multiple of 64 (the key tile of the kernel) and
 * blk_cap * block <= 131072.  blk_idx [batch, n_q_heads, blk_cap] ascending block
 * ids, blk_budget [batch] entries used (shared by the heads, clamped to blk_cap);
 * q_idx / q_cnt, O and lse as in omni_sparse_attn_fwd.  Without the causal mask
 * n_tokens must be a multiple of block (pad tokens of a partial last block are
 * hidden by the mask only).
 * Workspace: OMNI_CALL_BLOCK_ATTN_FWD with param = blk_cap * block.
 */
int omni_block_attn_fwd(const omni_layer_desc* desc, const void* Q, const void* K, const void* V,
                        const int32_t* q_idx, const int32_t* q_cnt,
                        const int32_t* blk_idx, const int32_t* blk_budget, int32_t blk_cap,
                        int32_t block, void* O, float* lse, void* ws, size_t ws_bytes, void* stream);

/*
 * omni_block_attn_bwd -- gradients of omni_block_attn_fwd (the chain rule on the
 * attention equation of Sec. "Preliminary" with the block lists constant, as in
 * omni_sparse_attn_bwd; the paper trains with the same block-sparse attention, Sec.
 * "Implementation Details"), again without a gathered copy: K and V (natural and
 * k-packed K) are laid out once per KV head in token order and the kernels of
 * omni_sparse_attn_bwd find tile t of a head's list through the same tile map.
 * Same tiles in the same order, so dQ, dK, dV are bit for bit what
 * omni_expand_blocks + omni_sparse_attn_bwd give.
 * Arguments as in omni_block_attn_fwd and omni_sparse_attn_bwd (O, dO, lse in; dQ
 * [batch, n_q_heads, n_tokens, head_dim], dK, dV [batch, n_kv_heads, n_tokens,
 * head_dim] out, fully written); same limits as omni_block_attn_fwd.
 * Workspace: OMNI_CALL_BLOCK_ATTN_BWD with param = blk_cap * block.
 */
int omni_block_attn_bwd(const omni_layer_desc* desc, const void* Q, const void* K, const void* V,
                        const void* O, const void* dO, const float* lse,
                        const int32_t* q_idx, const int32_t* q_cnt,
                        const int32_t* blk_idx, const int32_t* blk_budget, int32_t blk_cap,
                        int32_t block, void* dQ, void* dK, void* dV,
                        void* ws, size_t ws_bytes, void* stream);

/*
 * Baselines used by the reported metric (not part of the method): plain causal
 * / non-causal attention of the attention equation in Sec. "Preliminary" built
 * on the same tile engine, and plain decode attention over rows [0, ctx_len).
 */
/*
 * omni_compact_cache / omni_slim_decode_compact -- Sec. "KV Cache Slimming": what
 * the decode stage keeps of the visual KV cache is the selected rows only.  Under
 * grouped-query attention a cache row belongs to a KV head, so the rows that can
 * be dropped are those no query head of the group selected: omni_compact_cache
 * copies the rows of the group lists (omni_group_subset) side by side,
 *   Kcomp, Vcomp [batch, n_kv_heads, u_cap, head_dim] dtype, out:
 *   row u of group (b, g) = cache row grp_idx[b, g, u], for u < min(grp_cnt, u_cap)
 *   (rows beyond that are left untouched),
 * and omni_slim_decode_compact is omni_slim_decode_grouped reading the listed rows
 * from Kcomp / Vcomp (sequentially, no gather) instead of the cache.  It reads
 * Kcache / Vcache at non-visual rows only ([0, vis_begin) and [vis_end, ctx_len)),
 * so a caller may release the visual part of the cache after compaction; the
 * store it then holds is Kcomp, Vcomp, grp_idx, grp_mask and the non-visual rows.
 * Output and `active` equal omni_slim_decode_grouped's (same rows, same order).
 * Workspace of the decode call: OMNI_CALL_SLIM_DECODE.
 */
/*
 * Paged variants: the same store cut into pages of a pool (omni_page_pool), the
 * layout a serving engine's block allocator hands out.  The caller owns pool and
 * table and assigns the pages (ceil(grp_cnt / page_rows) per pair; two pairs never
 * share a page).  omni_compact_cache_paged writes row u of pair (b, g) to row
 * u % page_rows of page page_table[b, g, u / page_rows]; omni_slim_decode_paged is
 * omni_slim_decode_compact reading the rows from there.  Rows whose table entry is
 * outside [0, n_pages) are neither stored nor attended (no error).  With every
 * page present the output equals omni_slim_decode_compact's bit for bit.
 */
int omni_compact_cache_paged(const omni_decode_desc* desc, const void* Kcache, const void* Vcache,
                             const int32_t* grp_idx, const int32_t* grp_cnt, int32_t u_cap,
                             const omni_page_pool* pool, void* stream);
int omni_slim_decode_paged(const omni_decode_desc* desc, const void* q,
                           const void* Kcache, const void* Vcache, const int32_t* ctx_len,
                           const float* probe_keys, const omni_page_pool* pool,
                           const int32_t* grp_idx, const uint32_t* grp_mask, const int32_t* grp_cnt,
                           int32_t u_cap, void* O, uint8_t* active,
                           void* ws, size_t ws_bytes, void* stream);
int omni_compact_cache(const omni_decode_desc* desc, const void* Kcache, const void* Vcache,
                       const int32_t* grp_idx, const int32_t* grp_cnt, int32_t u_cap,
                       void* Kcomp, void* Vcomp, void* stream);
int omni_slim_decode_compact(const omni_decode_desc* desc, const void* q,
                             const void* Kcache, const void* Vcache, const int32_t* ctx_len,
                             const float* probe_keys,
                             const void* Kcomp, const void* Vcomp,
                             const int32_t* grp_idx, const uint32_t* grp_mask, const int32_t* grp_cnt,
                             int32_t u_cap,
                             void* O, uint8_t* active,
                             void* ws, size_t ws_bytes, void* stream);

int omni_dense_attn_fwd(const omni_layer_desc* desc, const void* Q, const void* K, const void* V,
                        void* O, float* lse, void* ws, size_t ws_bytes, void* stream);
int omni_dense_decode(const omni_decode_desc* desc, const void* q,
                      const void* Kcache, const void* Vcache, const int32_t* ctx_len,
                      void* O, void* ws, size_t ws_bytes, void* stream);

/* Workspace bytes needed by call `call_id` (omni_call_id) for the given
 * descriptor (omni_layer_desc* for prefill calls, omni_decode_desc* for the two
 * decode calls).  `param` is the index capacity b_cap for the calls that take
 * one, the probe block for OMNI_CALL_KV_BUDGET and OMNI_CALL_PREFILL_SELECT,
 * blk_cap * block for OMNI_CALL_BLOCK_ATTN_FWD and OMNI_CALL_BLOCK_ATTN_BWD, and ignored otherwise.
 * Returns 0 on invalid input (a valid call never needs 0 bytes). */
size_t omni_workspace_bytes(int call_id, const void* desc, int32_t param);

/*
 * Kernel timing for benchmarks (not part of the method).  While enabled, the
 * library records a HIP event pair on the call's stream around each launch of
 * the kernels listed below (at most 64 launches per kernel; later ones are not
 * recorded).  omni_profile_enable(mask): 0 switches the timing off, a negative
 * value times every listed kernel, otherwise bit k of mask switches kernel_id k
 * on (an event pair costs a few microseconds on the stream: time one kernel
 * inside a region whose wall clock matters).  It also resets the records; omni_profile_read()
 * waits for the recorded launches and returns their summed duration in
 * milliseconds and their number.  Not thread safe.  kernel_id: 0 attention
 * forward main kernel, 1 K/V pack (gather), 2 output clear, 3 query pooling,
 * 4 probe pass 1 (row log-sum-exp), 5 probe pass 2 (column sums), 6 query
 * scoring, 7 backward dK/dV kernel, 8 backward dQ kernel, 9 backward
 * scatter-reduce, 10 decode partial kernel, 11 selection kernels.
 */
int omni_profile_enable(int mask);
int omni_profile_read(int kernel_id, float* total_ms /* host */, int* launches /* host */);

/*
 * Diagnostic, host only: the work list the query-tile kernels (attention forward,
 * backward dQ) build on the device, computed by the same rule on the host.  Work item
 * = one tile of tile_rows (128 or 256) kept queries of a head, its cost the number of
 * 64-key tiles it streams (estimated here from the position of the tile; the device
 * uses exact counts where it has them).  queues = 1: one list, longest item first,
 * handed out from one atomic counter.  queues = 8 (the sparse bf16 forward): one list
 * per XCD -- whole heads are placed on queues, largest head first onto the least loaded
 * queue; inside a queue head follows head, each longest item first; a workgroup takes
 * from its XCD's queue and, once that is drained, from the queue with the most items left.  All pointers are
 * HOST pointers.  q_cnt [batch * n_q_heads] (null: every head keeps n_tokens rows),
 * budget [batch] (null: n_tokens); item_head / item_tile / item_cost [capacity] out,
 * queue after queue in hand-out order; queue_end [8] out (nullable): queue q is the
 * positions [queue_end[q-1], queue_end[q]); n_items out.  OMNI_ERR_WORKSPACE if
 * capacity is too small (n_items is still written).
 */
int omni_debug_work_list(const omni_layer_desc* desc, const int32_t* q_cnt, const int32_t* budget,
                         int32_t b_cap, int32_t tile_rows, int32_t queues, int32_t* item_head,
                         int32_t* item_tile, int32_t* item_cost, int32_t capacity, int32_t* n_items,
                         int32_t* queue_end);

/*
 * Diagnostic: copy `bytes` (a positive multiple of 16) from src to dst, both DEVICE pointers
 * to 16-byte aligned, non-overlapping buffers, with a plain copy kernel
 * (calibration_copy_kernel) on `stream`.  A launch of known HBM traffic: a profiler's
 * byte counters are scaled by what they report for it.
 */
int omni_debug_copy(const void* src, void* dst, size_t bytes, void* stream);

/*
 * Diagnostic: sustained rate of register-resident bf16 32x32x16 MFMAs on all compute units,
 * with constant operands (random_operands = 0) or pseudo-random ones (1); the second is
 * what power management leaves of the nominal matrix-core peak for operands that toggle
 * like real data.  2: pseudo-random operands with the matrix cores idle a third of the time
 * (all wavefronts sleep together after every 32 MFMAs) -- the clock it reaches tells whether
 * the full-duty rate is set by the power limit.  Runs on the default stream and synchronises; allocates and frees a few
 * MiB.  Outputs are HOST pointers: TFLOP/s and the mean shader clock in MHz.
 */
int omni_debug_mfma_rate(int random_operands, int iters, double* tflops /* host */, double* shader_mhz /* host */);

/*
 * Diagnostic: the backward pass shares a key tile that is seen by very many query tiles (a head
 * that keeps every query, at long context) between several workgroups, from `tiles` 64-query
 * tiles per share on (default 128).  A small value makes short test inputs take that path.
 * tiles <= 0 restores the default.  Process-wide; not for use while a backward call is running.
 */
int omni_debug_key_split_len(int tiles);

/* Message of the last error on this thread ("" if none). */
const char* omni_last_error(void);

/* Library version: major * 10000 + minor * 100 + patch. */
int omni_version(void);

#ifdef __cplusplus
}
#endif
#endif /* OMNISPARSE_H */
