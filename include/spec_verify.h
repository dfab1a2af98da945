/*
 * spec_verify.h - C ABI of the MI355X (gfx950) parallel-verification library.
 *
 * The library implements the verification step of speculative inference as stated
 * in Section 2.1 of the CoSine paper (arXiv 2503.10325) plus the confidence-based
 * token fusion of its Section 4.2:
 *
 *   spec_verify_attn   the attention sub-step of the target model's parallel pass
 *                      over all draft tokens (Section 2.1; tree attention, Sections
 *                      2.1 and 4.2),
 *   spec_fuse_drafts   token fusion across drafters (Algorithm 1, TokenFusion;
 *                      Eq. 4, first line),
 *   spec_accept        acceptance-rejection with residual resampling and the bonus
 *                      token (Section 2.1).
 *
 * Conventions common to every entry point
 *   - Pointers are DEVICE pointers unless the comment says "host".
 *   - The caller owns every buffer (inputs, outputs, workspace).  The library
 *     allocates nothing, frees nothing and keeps no pointer after returning.
 *   - Calls validate their host-visible arguments, enqueue kernels on `stream`
 *     (a hipStream_t passed as void*; NULL = the default stream) and return without
 *     synchronising.  Outputs are valid once the stream has been synchronised.
 *   - The library keeps no state between calls and reads no environment variable; every
 *     launch decision is a function of the call's arguments and of the current device.
 *   - Return value: SPEC_OK (0) or a negative spec_status.  Nothing is enqueued when
 *     validation fails.  Data that lives on the device (parent[], block_table[],
 *     token ids) is NOT validated: out-of-range page or token indices are undefined
 *     behaviour; a parent[i] outside [-1, i) is treated as -1.
 *   - Same inputs give bit-identical outputs from run to run (no floating-point
 *     atomics are used in any reduction).
 *   - bf16 tensors are raw 16-bit patterns; all arithmetic is fp32/fp64 on exact
 *     upcasts (attention feeds bf16 operands to the matrix cores, accumulating in
 *     fp32).
 */
#ifndef SPEC_VERIFY_H
#define SPEC_VERIFY_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  SPEC_OK = 0,
  SPEC_ERR_NULL = -1,        /* a required pointer is NULL                        */
  SPEC_ERR_SHAPE = -2,       /* a size is negative, zero where it may not be, or inconsistent */
  SPEC_ERR_UNSUPPORTED = -3, /* head_dim / page_size / dtype / mode not implemented */
  SPEC_ERR_WORKSPACE = -4,   /* workspace missing or smaller than *_workspace_size */
  SPEC_ERR_LAUNCH = -6       /* the HIP runtime refused a launch                   */
} spec_status;

typedef enum { SPEC_BF16 = 0, SPEC_F32 = 1 } spec_dtype;

/* ------------------------------------------------------------------------------
 * spec_verify_attn
 *
 * For request b (of `batch`), query head h and draft node i (of n[b] =
 * q_offsets[b+1]-q_offsets[b] nodes):
 *
 *   O[i,h,:] = sum_t softmax_t( scale * <Q[i,h,:], K[t,h/G,:]> ) * V[t,h/G,:]
 *
 * where t runs over the ctx_len[b] committed positions and over the draft
 * positions ctx_len[b]+j of node i itself and of its ancestors (a linear draft:
 * j <= i).  G = num_q_heads / num_kv_heads.  Draft node j's key/value are expected
 * in the cache at logical position ctx_len[b]+j before the call.
 * ---------------------------------------------------------------------------- */
typedef struct {
  int32_t batch;             /* B >= 0                                              */
  int32_t num_q_heads;       /* Hq                                                  */
  int32_t num_kv_heads;      /* Hkv, Hq % Hkv == 0                                  */
  int32_t head_dim;          /* D: 64 or 128                                        */
  int32_t page_size;         /* tokens per cache page: 16                           */
  int32_t total_q;           /* sum_b n[b] = q_offsets[B]                           */
  int32_t max_q_per_req;     /* upper bound of n[b]; at most 128 (above 64: two
                                ancestor-mask words per node, row-split kernels)    */
  int32_t max_pages_per_req; /* row stride of block_table; >= ceil((ctx+n)/page)    */
  int64_t total_kv_tokens_hint; /* host's estimate of sum_b (ctx_len[b]+n[b]); 0 = unknown.
                                   Only steers how the context is split into chunks. */
  float scale;               /* softmax scale; 0 selects 1/sqrt(head_dim)           */
  int32_t out_dtype;         /* spec_dtype of `out`: SPEC_BF16 or SPEC_F32          */
} spec_attn_desc;

/* Bytes of workspace spec_verify_attn needs for this descriptor (host call). */
size_t spec_verify_attn_workspace_size(const spec_attn_desc* desc);

int32_t spec_verify_attn(
    const spec_attn_desc* desc,  /* host                                              */
    const void* q,               /* [total_q, Hq, D] bf16                             */
    const void* k_pool,          /* [num_pages, Hkv, page_size, D] bf16               */
    const void* v_pool,          /* [num_pages, Hkv, page_size, D] bf16               */
    const int32_t* block_table,  /* [B, max_pages_per_req] logical page -> pool page  */
    const int32_t* ctx_len,      /* [B]                                               */
    const int32_t* q_offsets,    /* [B+1] prefix sums of n[b]                         */
    const int32_t* parent,       /* [total_q] parent node within the request, -1 = child of
                                    the committed prefix, parent[i] < i; NULL = linear  */
    void* out,                   /* [total_q, Hq, D] of out_dtype                     */
    float* lse,                  /* optional [total_q, Hq]: natural-log sum-exp of the
                                    scaled scores over the allowed set; may be NULL    */
    void* workspace, size_t workspace_bytes, void* stream);
/* q, k_pool, v_pool and out must be 16-byte aligned (SPEC_ERR_SHAPE otherwise). */

/* Writes a one-line description of the kernels and the context split that spec_verify_attn uses
 * for this descriptor into buf (host; for logs and benchmark reports). */
int32_t spec_describe_attn_plan(const spec_attn_desc* desc, char* buf, size_t buf_bytes);

/* ------------------------------------------------------------------------------
 * spec_fuse_drafts
 *
 * Position i of request b holds one candidate token per drafter n with the
 * probability conf[b,i,n] that drafter assigned to it.  ARGMAX (the paper's rule):
 * winner = argmax_n conf (lowest n on ties), fused_token = that drafter's token,
 * q_row = (b*k_max+i)*N + winner, the row of draft_logits the token was drawn from.
 * MIXTURE (weighted averaging of distributions, Section 2.2): additionally
 * fused_probs[b*k_max+i, :] = sum_n w_n softmax(draft_logits[(b,i,n)] / T),
 * w_n = conf_n / sum_n conf_n (1/N when all are zero) and q_row = b*k_max+i.
 * Positions i >= k_len[b] get -1 in the three index outputs (fused_probs rows of
 * such positions are left untouched).
 * ---------------------------------------------------------------------------- */
typedef enum { SPEC_FUSE_ARGMAX = 0, SPEC_FUSE_MIXTURE = 1 } spec_fuse_mode;

size_t spec_fuse_drafts_workspace_size(int32_t B, int32_t k_max, int32_t N, int32_t V, int32_t mode);

int32_t spec_fuse_drafts(
    int32_t B, int32_t k_max, int32_t N, int32_t V,
    const int32_t* k_len,        /* [B] valid positions per request, <= k_max          */
    const float* conf,           /* [B, k_max, N]                                      */
    const int32_t* draft_tokens, /* [B, k_max, N]                                      */
    const void* draft_logits,    /* [B*k_max*N, V]; may be NULL in ARGMAX mode         */
    int32_t logits_dtype,        /* spec_dtype of draft_logits                         */
    float temperature,           /* > 0 (MIXTURE only)                                 */
    int32_t mode,                /* spec_fuse_mode                                     */
    int32_t* fused_token,        /* [B, k_max]                                         */
    int32_t* winner,             /* [B, k_max]                                         */
    int32_t* q_row,              /* [B, k_max]                                         */
    float* fused_probs,          /* MIXTURE: [B*k_max, V] fp32; else may be NULL       */
    void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------------
 * spec_accept
 *
 * Request b owns draft nodes node_offsets[b] .. node_offsets[b+1]) and target rows
 * node_offsets[b]+b ..: local row 0 is the target distribution after the committed
 * prefix, local row 1+j the one after node j.  p = softmax(target row / T);
 * q = softmax(draft row / T) (SPEC_Q_LOGITS) or the row itself (SPEC_Q_PROBS).
 *
 * Walk from the committed prefix: r = p of the current node.  For each child c of
 * the current node in index order, accept when u_accept[c] < r(x_c)/q(x_c) - so
 * q <= r always accepts and otherwise the token is rejected with probability
 * 1 - r/q - and descend; on rejection r <- norm(max(0, r - q)) and the next sibling
 * is tried.  When the current node has no child (everything accepted) or all its
 * children were rejected, one token is drawn from r by inverse CDF in ascending
 * token order with u_resample[b]: the smallest t with sum_{v<=t} r_v > u * sum_v r_v.
 * For a linear draft this is exactly the rule of Section 2.1; the children of one
 * node are i.i.d. draws from one draft row, the row the FIRST child's q_row entry
 * names: it serves q(x_c) and the residual for every child of that node, and the
 * q_row entries of later siblings are not used.  q(x)=0<r(x) accepts,
 * q(x)=r(x)=0 rejects; a residual of zero mass leaves r unchanged.
 * ---------------------------------------------------------------------------- */
typedef enum { SPEC_Q_LOGITS = 0, SPEC_Q_PROBS = 1 } spec_q_kind;

size_t spec_accept_workspace_size(int32_t B, int32_t total_nodes, int32_t n_q_rows, int32_t V);

int32_t spec_accept(
    int32_t B, int32_t V,
    int32_t total_nodes,         /* = node_offsets[B] (host copy)                      */
    int32_t n_q_rows,            /* rows of draft_q                                    */
    int32_t max_nodes_per_req,   /* upper bound of n[b]; at most 128                   */
    const int32_t* node_offsets, /* [B+1]                                              */
    const int32_t* parent,       /* [total_nodes] or NULL = linear chain               */
    const int32_t* draft_tokens, /* [total_nodes] in [0, V)                            */
    const void* target_logits,   /* [total_nodes + B, V]                               */
    int32_t target_dtype,        /* spec_dtype                                         */
    const void* draft_q,         /* [n_q_rows, V]                                      */
    int32_t q_dtype,             /* spec_dtype                                         */
    int32_t q_kind,              /* spec_q_kind                                        */
    const int32_t* q_row,        /* [total_nodes] row of draft_q node j was drawn from */
    float temperature,           /* > 0                                                */
    const float* u_accept,       /* [total_nodes] in [0,1)                             */
    const float* u_resample,     /* [B] in [0,1)                                       */
    int32_t* accept_len,         /* [B] number of accepted draft tokens                */
    int32_t* out_tokens,         /* [B, out_stride]: accepted tokens, then the drawn one;
                                    entries past accept_len[b]+1 are set to -1          */
    int32_t out_stride,          /* >= max_nodes_per_req + 1                           */
    int32_t* stop_node,          /* optional [B]: last accepted node or -1             */
    float* dbg_ratio,            /* optional [total_nodes]: ratio compared at each visited
                                    node, NaN where not visited                         */
    void* workspace, size_t workspace_bytes, void* stream);

/* spec_accept with explicit launch choices, for tests and sweeps (same arguments, same results).
 * The library's choice: linear drafts (parent == NULL) take a statistics pass over all rows and then one
 * kernel that repeats the scalar accept tests in every workgroup and spreads the single vocabulary-wide
 * draw a chain needs over the chip (path 3); large batches use a statistics pass that stops reading a
 * request's rows at its first rejection (path 4).  Trees with bf16 logit rows (16-byte aligned, V a multiple
 * of 8) and a batch of at most one request per compute unit are walked by a cluster of workgroups per
 * request that keep slices of the walked rows in LDS and read no other row (path 2); other inputs take the
 * statistics pass followed by one walking workgroup per request (path 1).  No wait between workgroups is
 * unbounded: `patience` is the number of polls one spends waiting for its peers before it does their share
 * itself (0 = never wait); path 3 has no waits at all.  tuning == NULL is spec_accept. */
typedef struct {
  int32_t path;      /* 0 = library's choice, 1 = statistics pass + walk, 2 = workgroup clusters, 3 = statistics
                        pass + linear-draft kernel, 4 = the same with a statistics pass that stops at each request's
                        first rejection (2, 3, 4 fall back when the inputs do not qualify: 4 to 3, 3 and 2 to 1)   */
  int32_t levels;    /* path 2: rows of the walk looked at in one exchange, 0 = library's choice   */
  int32_t slices;    /* path 2: workgroups one row pair is cut over, 0 = library's choice          */
  int32_t patience;  /* < 0 = library's choice                                                     */
  int32_t helpers;   /* path 1: helper workgroups per request (0..3), < 0 = library's choice       */
} spec_accept_tuning;

int32_t spec_accept_tuned(
    const spec_accept_tuning* tuning, /* host, may be NULL                                 */
    int32_t B, int32_t V, int32_t total_nodes, int32_t n_q_rows, int32_t max_nodes_per_req,
    const int32_t* node_offsets, const int32_t* parent, const int32_t* draft_tokens,
    const void* target_logits, int32_t target_dtype, const void* draft_q, int32_t q_dtype,
    int32_t q_kind, const int32_t* q_row, float temperature, const float* u_accept,
    const float* u_resample, int32_t* accept_len, int32_t* out_tokens, int32_t out_stride,
    int32_t* stop_node, float* dbg_ratio, void* workspace, size_t workspace_bytes, void* stream);

/* spec_accept for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): same arguments without the workspace, same results.
 * The workspace is a fixed array inside the library (spec_accept_noalloc_max_workspace() bytes, 4 MiB,
 * one per GPU, held until the process ends); the call allocates and frees nothing.  Problems whose
 * spec_accept_workspace_size exceeds that are rejected with SPEC_ERR_WORKSPACE and nothing is
 * enqueued; SPEC_ERR_LAUNCH if the array's address cannot be obtained.  Every call on one GPU uses
 * that GPU's one array: calls that may overlap on one GPU (different streams, different threads)
 * race and must be serialised by the caller.  What has to start at zero is cleared by a kernel of
 * the call itself. */
size_t spec_accept_noalloc_max_workspace(void);
int32_t spec_accept_noalloc(
    int32_t B, int32_t V, int32_t total_nodes, int32_t n_q_rows, int32_t max_nodes_per_req,
    const int32_t* node_offsets, const int32_t* parent, const int32_t* draft_tokens,
    const void* target_logits, int32_t target_dtype, const void* draft_q, int32_t q_dtype,
    int32_t q_kind, const int32_t* q_row, float temperature, const float* u_accept,
    const float* u_resample, int32_t* accept_len, int32_t* out_tokens, int32_t out_stride,
    int32_t* stop_node, float* dbg_ratio, void* stream);

/* One-line description of what spec_accept launches for this shape on the current device
 * (host; for logs and benchmark reports).  total_nodes as for spec_accept. */
int32_t spec_describe_accept_plan(const spec_accept_tuning* tuning, int32_t B, int32_t V, int32_t total_nodes,
                                  int32_t max_nodes_per_req, int32_t is_tree, int32_t target_dtype,
                                  int32_t q_dtype, int32_t q_kind, char* buf, size_t buf_bytes);

/* ------------------------------------------------------------------------------
 * spec_accept_greedy
 *
 * The same walk under greedy sampling, the decoding rule of the paper's experiments
 * (Section 6.1, experiment settings: greedy sampling for draft generation and
 * verification).  Target rows are laid out as for spec_accept.  g = index of the
 * largest logit of the current node's target row (ordinary fp32 comparison, -0 equal
 * to +0, NaN never the largest; the lowest index among equal values; a row without
 * any comparable entry gives 0).  The first child c of the current node, in index
 * order, with draft_tokens[c] == g is accepted and the walk descends; when there is
 * none, g is emitted and the walk stops.  No draft distributions, no uniforms, no
 * temperature: the result is exact integer work.  Rows (total_nodes + B) are limited
 * to 65535 per call; bad parent entries (>= own index or < -1) count as -1.
 * ---------------------------------------------------------------------------- */
size_t spec_accept_greedy_workspace_size(int32_t B, int32_t total_nodes, int32_t V);

int32_t spec_accept_greedy(
    int32_t B, int32_t V,
    int32_t total_nodes,         /* = node_offsets[B] (host copy)                      */
    int32_t max_nodes_per_req,   /* upper bound of n[b]; at most 128                   */
    const int32_t* node_offsets, /* [B+1]                                              */
    const int32_t* parent,       /* [total_nodes] or NULL = linear chain               */
    const int32_t* draft_tokens, /* [total_nodes]                                      */
    const void* target_logits,   /* [total_nodes + B, V]                               */
    int32_t target_dtype,        /* spec_dtype                                         */
    int32_t* accept_len,         /* [B] number of accepted draft tokens                */
    int32_t* out_tokens,         /* [B, out_stride]: accepted tokens, then the emitted one;
                                    entries past accept_len[b]+1 are set to -1          */
    int32_t out_stride,          /* >= max_nodes_per_req + 1                           */
    int32_t* stop_node,          /* optional [B]: last accepted node or -1             */
    int32_t* row_argmax,         /* optional [total_nodes + B]: g of every target row  */
    void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------------
 * spec_routing_scores
 *
 * The routing-score update that follows acceptance (Section 4.1, Eq. 1 and Eq. 2).
 * For request b, drafter n and draft position i < k_len[b]:
 *   d = cos(H[out_tokens[b,i]], H[draft_tokens[b,i,n]])  if i < accept_len[b]  (the
 *       positions whose draft was accepted; out_tokens as written by spec_accept),
 *       0 otherwise;
 *   scores[b,n] = (1/k_len[b]) sum_i c d / (c d + (1-c)(1-d)),  c = conf[b,i,n].
 * H = rows of the embedding table.  Where the paper is silent: a negative cosine
 * counts as 0, a zero row gives cosine 0, a term whose denominator is not positive
 * (c=1,d=0 or c=0,d=1) is 0, k_len[b] = 0 gives 0.  Token ids are clamped to [0, V).
 * k_max <= 64, N <= 16.  No workspace.
 * ---------------------------------------------------------------------------- */
int32_t spec_routing_scores(
    int32_t B, int32_t k_max, int32_t N,
    int32_t V, int32_t E,        /* embedding table shape                              */
    const int32_t* k_len,        /* [B] valid positions per request, <= k_max          */
    const float* conf,           /* [B, k_max, N] in [0,1]                             */
    const int32_t* draft_tokens, /* [B, k_max, N]                                      */
    const int32_t* accept_len,   /* [B]                                                */
    const int32_t* out_tokens,   /* [B, out_stride]                                    */
    int32_t out_stride,
    const void* embedding,       /* [V, E]                                             */
    int32_t embedding_dtype,     /* spec_dtype                                         */
    float* scores,               /* [B, N]                                             */
    void* stream);

/* ------------------------------------------------------------------------------
 * spec_adaptive_speculation
 *
 * AdaptiveSpeculation of Algorithm 2 (Section 4.3): the draft lengths gamma_i of the
 * requests of a batch are cut until their sum fits the verification budget: while
 * sum_i gamma_i > gamma_max_total, the request with the largest gamma_i (lowest index
 * on ties) gives up one token.  Every request keeps at least one token (gamma_i >= 1
 * in the batch formulation), so the sum may stay above the budget when all are at 1.
 * Requests with in_batch[i] == 0 are copied unchanged and do not count.  gamma_out must
 * not overlap gamma_in.  The result equals the sequential loop exactly.  Any R; one launch.
 * ---------------------------------------------------------------------------- */
int32_t spec_adaptive_speculation(
    int32_t R,                   /* requests in the pool                               */
    const int32_t* gamma_in,     /* [R] draft tokens asked for                         */
    const int32_t* in_batch,     /* [R] b_i, or NULL = every request is in the batch   */
    int64_t gamma_max_total,     /* Gamma_max                                          */
    int32_t* gamma_out,          /* [R]                                                */
    int64_t* total_out,          /* optional [1]: sum of gamma_out over the batch      */
    void* stream);

/* ------------------------------------------------------------------------------
 * spec_compact_kv
 *
 * After a draft tree has been verified, moves the K/V entries of the accepted path to
 * consecutive cache positions, so that the next step sees an ordinary linear context.
 * The paper only says that verified drafts return to the request pool (Section 4.1);
 * this data movement is what a paged cache with tree drafts needs for that.  Draft
 * node j of request b lives at logical position ctx_len[b] + j; the accepted path is
 * the chain of ancestors root .. stop_node[b] (as written by spec_accept or
 * spec_accept_greedy; -1 = nothing accepted); its d-th node moves to position
 * ctx_len[b] + d, in both pools, for every KV head.  Linear drafts need no move and are
 * left untouched.  Pools and block table as in spec_verify_attn; the pools are modified
 * in place.  new_len[b] = ctx_len[b] + path length.  head_dim 64 or 128, page_size 16,
 * at most 128 nodes per request.
 * ---------------------------------------------------------------------------- */
int32_t spec_compact_kv(
    int32_t B, int32_t num_kv_heads, int32_t head_dim, int32_t page_size, int32_t max_pages_per_req,
    void* k_pool, void* v_pool,  /* [num_pages, Hkv, page_size, D] bf16, modified      */
    const int32_t* block_table,  /* [B, max_pages_per_req]                             */
    const int32_t* ctx_len,      /* [B]                                                */
    const int32_t* q_offsets,    /* [B+1] prefix sums of n[b]                          */
    const int32_t* parent,       /* [total_q] or NULL = linear chains                  */
    const int32_t* stop_node,    /* [B] last accepted node, -1 = none                  */
    int32_t* new_len,            /* optional [B]                                       */
    void* stream);

/* ------------------------------------------------------------------------------
 * spec_lm_head
 *
 * The projection that produces the target logits o_i of Section 2.1, the matrix-matrix
 * product that Section 3.1 identifies as the bulk of verification on the target model,
 * fused with the first pass of the vocab-wide softmax:
 *   logits[r, v] = bf16( sum_k hidden[r, k] * weight[v, k] )      (fp32 accumulation)
 * and, for every row, the statistics (maximum, sum of exp((l - max)/T) per 8192-class
 * segment of the ROUNDED logits) that spec_accept would otherwise compute by reading
 * the logits again.  hidden [rows, d_model] and weight [V, d_model] are bf16, row-major
 * (one weight row per vocabulary entry), 16-byte aligned; d_model a multiple of 128.
 * Rows are the target rows of spec_accept in its order (rows = total_nodes + B).
 * target_stats receives spec_row_stats_size(rows, V) bytes in the library's internal
 * layout: pass the START of the workspace later given to spec_accept_prestats (with
 * the same temperature), or any device buffer of that size.  Any number of rows up to
 * 65535; up to 128 rows the weight matrix is read once.
 * All pointers are device memory owned by the caller; the call only enqueues kernels on
 * `stream` and allocates nothing.  workspace: spec_lm_head_workspace_size(rows,
 * d_model, V) bytes (per-block statistics and, above 128 rows, the hidden states
 * re-laid out in matrix-operand order); its contents need not survive the call.
 * Errors: SPEC_ERR_SHAPE (negative or zero sizes, temperature <= 0, misaligned
 * pointers), SPEC_ERR_UNSUPPORTED (d_model not a multiple of 128 or above 65536, V above
 * 2097152, more than 65535 rows), SPEC_ERR_NULL, SPEC_ERR_WORKSPACE, SPEC_ERR_LAUNCH;
 * rows == 0 is SPEC_OK and touches nothing.
 * ---------------------------------------------------------------------------- */
size_t spec_row_stats_size(int32_t rows, int32_t V);
size_t spec_lm_head_workspace_size(int32_t rows, int32_t d_model, int32_t V);

int32_t spec_lm_head(
    int32_t rows, int32_t d_model, int32_t V,
    const void* hidden,          /* [rows, d_model] bf16                               */
    const void* weight,          /* [V, d_model] bf16                                  */
    float temperature,           /* > 0: the T of the statistics                       */
    void* logits,                /* [rows, V] bf16                                     */
    void* target_stats,          /* spec_row_stats_size(rows, V) bytes                 */
    void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------------
 * spec_accept_prestats
 *
 * spec_accept for target logits that come from spec_lm_head: same arguments, same
 * results, but the first spec_row_stats_size(total_nodes + B, V) bytes of workspace
 * already hold the target rows' statistics (written by spec_lm_head with the same
 * temperature, V and row order), so only the draft rows are read for statistics.
 * (Draft trees for which the library picks the kernel that reads only the walked rows
 * are verified from the logits alone; the supplied statistics are then not read.)
 * target_dtype must be SPEC_BF16.  Workspace size as for spec_accept.
 * ---------------------------------------------------------------------------- */
int32_t spec_accept_prestats(
    int32_t B, int32_t V, int32_t total_nodes, int32_t n_q_rows, int32_t max_nodes_per_req,
    const int32_t* node_offsets, const int32_t* parent, const int32_t* draft_tokens,
    const void* target_logits, int32_t target_dtype, const void* draft_q, int32_t q_dtype,
    int32_t q_kind, const int32_t* q_row, float temperature, const float* u_accept,
    const float* u_resample, int32_t* accept_len, int32_t* out_tokens, int32_t out_stride,
    int32_t* stop_node, float* dbg_ratio, void* workspace, size_t workspace_bytes, void* stream);

const char* spec_strerror(int32_t status);

/* Library/ABI version, bumped when a signature changes. */
int32_t spec_abi_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SPEC_VERIFY_H */
