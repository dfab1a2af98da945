// C ABI of the verification library: argument validation and dispatch only.
#include "../../include/spec_verify.h"

#include <stdio.h>

#include "kernels.h"

using namespace specv;

// Scratch memory of spec_accept_noalloc: one array per GPU, held until the process ends.  In host code
// the array's name is only a stand-in; its device address is asked for once per device and kept.
constexpr size_t kNoallocScratchBytes = 4u << 20;
static __device__ __align__(256) unsigned char scratch[kNoallocScratchBytes];
constexpr int kMaxDevices = 64;
static std::atomic<void*> g_scratch_ptr[kMaxDevices];

static void* noalloc_scratch_ptr() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (p) return p;
  if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return nullptr;
  g_scratch_ptr[dev].store(p, std::memory_order_release);      // racing threads store the same address
  return p;
}

extern "C" {

const char* spec_strerror(int32_t status) {
  switch (status) {
    case SPEC_OK: return "ok";
    case SPEC_ERR_NULL: return "a required pointer is NULL";
    case SPEC_ERR_SHAPE: return "invalid or inconsistent size";
    case SPEC_ERR_UNSUPPORTED: return "unsupported head_dim, page_size, dtype or mode";
    case SPEC_ERR_WORKSPACE: return "workspace missing or too small (or the problem exceeds the built-in scratch)";
    case SPEC_ERR_LAUNCH: return "HIP launch failed";
    default: return "unknown status";
  }
}

int32_t spec_abi_version(void) { return 3; }

static int check_attn_desc(const spec_attn_desc* d) {
  if (!d) return SPEC_ERR_NULL;
  if (d->batch < 0 || d->total_q < 0 || d->num_q_heads <= 0 || d->num_kv_heads <= 0 ||
      d->max_pages_per_req < 0 || d->max_q_per_req < 0)
    return SPEC_ERR_SHAPE;
  if (d->num_q_heads % d->num_kv_heads != 0) return SPEC_ERR_SHAPE;
  if (d->head_dim != 64 && d->head_dim != 128) return SPEC_ERR_UNSUPPORTED;
  if (d->page_size != 16) return SPEC_ERR_UNSUPPORTED;
  if (d->max_q_per_req > 128) return SPEC_ERR_UNSUPPORTED;
  if (d->out_dtype != SPEC_BF16 && d->out_dtype != SPEC_F32) return SPEC_ERR_UNSUPPORTED;
  if (d->batch > 65535 || d->num_kv_heads > 65535) return SPEC_ERR_UNSUPPORTED;
  if (!(d->scale >= 0.f)) return SPEC_ERR_SHAPE;
  if (d->batch > 0 && d->total_q > 0 && (d->max_pages_per_req == 0 || d->max_q_per_req == 0))
    return SPEC_ERR_SHAPE;
  return SPEC_OK;
}

static AttnArgs attn_args_from(const spec_attn_desc* d) {
  AttnArgs a{};
  a.B = d->batch; a.Hq = d->num_q_heads; a.Hkv = d->num_kv_heads; a.D = d->head_dim;
  a.page = d->page_size; a.total_q = d->total_q; a.max_q = d->max_q_per_req;
  a.max_pages = d->max_pages_per_req; a.kv_hint = d->total_kv_tokens_hint;
  a.scale = d->scale; a.out_dtype = d->out_dtype;
  return a;
}

size_t spec_verify_attn_workspace_size(const spec_attn_desc* desc) {
  if (check_attn_desc(desc) != SPEC_OK) return 0;
  const AttnArgs a = attn_args_from(desc);
  return attn_workspace_bytes(a, make_attn_plan(a));
}

int32_t spec_verify_attn(const spec_attn_desc* desc, const void* q, const void* k_pool, const void* v_pool,
                         const int32_t* block_table, const int32_t* ctx_len, const int32_t* q_offsets,
                         const int32_t* parent, void* out, float* lse, void* workspace,
                         size_t workspace_bytes, void* stream) {
  const int rc = check_attn_desc(desc);
  if (rc != SPEC_OK) return rc;
  if (desc->batch == 0 || desc->total_q == 0) return SPEC_OK;
  if (!q || !k_pool || !v_pool || !block_table || !ctx_len || !q_offsets || !out) return SPEC_ERR_NULL;
  // the kernels read q and the pools and write out with 16-byte accesses
  if ((reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(k_pool) | reinterpret_cast<uintptr_t>(v_pool) |
       reinterpret_cast<uintptr_t>(out)) & 15u)
    return SPEC_ERR_SHAPE;
  AttnArgs a = attn_args_from(desc);
  if (a.scale == 0.f) a.scale = 1.0f / sqrtf(static_cast<float>(a.D));
  const AttnPlan plan = make_attn_plan(a);
  const size_t need = attn_workspace_bytes(a, plan);
  if (need > 256 && (!workspace || workspace_bytes < need)) return SPEC_ERR_WORKSPACE;
  a.q = q; a.k_pool = k_pool; a.v_pool = v_pool; a.block_table = block_table; a.ctx_len = ctx_len;
  a.q_offsets = q_offsets; a.parent = parent; a.out = out; a.lse = lse; a.workspace = workspace;
  return launch_attn(a, plan, static_cast<hipStream_t>(stream));
}

int32_t spec_describe_attn_plan(const spec_attn_desc* desc, char* buf, size_t buf_bytes) {
  const int rc = check_attn_desc(desc);
  if (rc != SPEC_OK) return rc;
  if (!buf || buf_bytes == 0) return SPEC_ERR_NULL;
  const AttnArgs a = attn_args_from(desc);
  const AttnPlan p = make_attn_plan(a);
  snprintf(buf, buf_bytes, "%s; head_dim %d; context chunks of %d tokens, at most %d per request", attn_plan_name(p),
           a.D, p.chunk_tokens, p.max_chunks);
  return SPEC_OK;
}

size_t spec_fuse_drafts_workspace_size(int32_t B, int32_t k_max, int32_t N, int32_t V, int32_t mode) {
  if (B < 0 || k_max < 0 || N <= 0 || V < 0) return 0;
  return fuse_workspace_bytes(B, k_max, N, V, mode);
}

int32_t spec_fuse_drafts(int32_t B, int32_t k_max, int32_t N, int32_t V, const int32_t* k_len,
                         const float* conf, const int32_t* draft_tokens, const void* draft_logits,
                         int32_t logits_dtype, float temperature, int32_t mode, int32_t* fused_token,
                         int32_t* winner, int32_t* q_row, float* fused_probs, void* workspace,
                         size_t workspace_bytes, void* stream) {
  if (B < 0 || k_max < 0 || N <= 0) return SPEC_ERR_SHAPE;
  if (mode != SPEC_FUSE_ARGMAX && mode != SPEC_FUSE_MIXTURE) return SPEC_ERR_UNSUPPORTED;
  if (B == 0 || k_max == 0) return SPEC_OK;
  if (!k_len || !conf || !draft_tokens || !fused_token || !winner || !q_row) return SPEC_ERR_NULL;
  if (static_cast<int64_t>(B) * k_max * N > INT32_MAX) return SPEC_ERR_SHAPE;
  if (mode == SPEC_FUSE_MIXTURE) {
    if (V <= 0 || !(temperature > 0.f)) return SPEC_ERR_SHAPE;
    if (logits_dtype != SPEC_BF16 && logits_dtype != SPEC_F32) return SPEC_ERR_UNSUPPORTED;
    if (!draft_logits || !fused_probs) return SPEC_ERR_NULL;
    const size_t need = fuse_workspace_bytes(B, k_max, N, V, mode);
    if (!workspace || workspace_bytes < need) return SPEC_ERR_WORKSPACE;
  }
  FuseArgs a{};
  a.B = B; a.k_max = k_max; a.N = N; a.V = V; a.k_len = k_len; a.conf = conf; a.draft_tokens = draft_tokens;
  a.draft_logits = draft_logits; a.l_dtype = logits_dtype; a.temperature = temperature; a.mode = mode;
  a.fused_token = fused_token; a.winner = winner; a.q_row = q_row; a.fused_probs = fused_probs;
  a.workspace = workspace;
  launch_fuse(a, static_cast<hipStream_t>(stream));
  return hipGetLastError() == hipSuccess ? SPEC_OK : SPEC_ERR_LAUNCH;
}

size_t spec_accept_workspace_size(int32_t B, int32_t total_nodes, int32_t n_q_rows, int32_t V) {
  if (B < 0 || total_nodes < 0 || n_q_rows < 0 || V <= 0) return 0;
  return accept_workspace_bytes(B, total_nodes, n_q_rows, V);
}

static int32_t accept_entry(bool prestats, const spec_accept_tuning* tuning, int32_t B, int32_t V, int32_t total_nodes, int32_t n_q_rows,
                            int32_t max_nodes_per_req, const int32_t* node_offsets, const int32_t* parent,
                            const int32_t* draft_tokens, const void* target_logits, int32_t target_dtype,
                            const void* draft_q, int32_t q_dtype, int32_t q_kind, const int32_t* q_row,
                            float temperature, const float* u_accept, const float* u_resample,
                            int32_t* accept_len, int32_t* out_tokens, int32_t out_stride, int32_t* stop_node,
                            float* dbg_ratio, void* workspace, size_t workspace_bytes, void* stream) {
  if (B < 0 || V <= 0 || total_nodes < 0 || n_q_rows < 0 || max_nodes_per_req < 0) return SPEC_ERR_SHAPE;
  if (!(temperature > 0.f)) return SPEC_ERR_SHAPE;
  if (max_nodes_per_req > 128) return SPEC_ERR_UNSUPPORTED;
  if (V > 2097152) return SPEC_ERR_UNSUPPORTED;        // the walk kernel indexes a row by 16 x 256 blocks of 512
  if (out_stride < max_nodes_per_req + 1) return SPEC_ERR_SHAPE;
  if ((target_dtype != SPEC_BF16 && target_dtype != SPEC_F32) || (q_dtype != SPEC_BF16 && q_dtype != SPEC_F32))
    return SPEC_ERR_UNSUPPORTED;
  if (q_kind != SPEC_Q_LOGITS && q_kind != SPEC_Q_PROBS) return SPEC_ERR_UNSUPPORTED;
  if (total_nodes > 0 && n_q_rows == 0) return SPEC_ERR_SHAPE;
  if (static_cast<int64_t>(total_nodes) + B + n_q_rows > 65535) return SPEC_ERR_UNSUPPORTED;   // rows are the statistics grid's y dimension
  if (B == 0) return SPEC_OK;
  if (!node_offsets || !target_logits || !u_resample || !accept_len || !out_tokens) return SPEC_ERR_NULL;
  if (total_nodes > 0 && (!draft_tokens || !draft_q || !q_row || !u_accept)) return SPEC_ERR_NULL;
  const size_t need = accept_workspace_bytes(B, total_nodes, n_q_rows, V);
  if (!workspace || workspace_bytes < need) return SPEC_ERR_WORKSPACE;
  AcceptArgs a{};
  a.B = B; a.V = V; a.total_nodes = total_nodes; a.n_q_rows = n_q_rows; a.node_offsets = node_offsets;
  a.parent = parent; a.draft_tokens = draft_tokens; a.target = target_logits; a.t_dtype = target_dtype;
  a.draft_q = draft_q; a.q_dtype = q_dtype; a.q_kind = q_kind; a.q_row = q_row; a.temperature = temperature;
  a.u_accept = u_accept; a.u_resample = u_resample; a.accept_len = accept_len; a.out_tokens = out_tokens;
  a.out_stride = out_stride; a.stop_node = stop_node; a.dbg_ratio = dbg_ratio; a.workspace = workspace;
  a.target_stats_ready = prestats;
  a.max_nodes = max_nodes_per_req;
  a.path = 0; a.levels = 0; a.slices = 0; a.patience = -1; a.helpers = -1;
  if (tuning) {
    if (tuning->path < 0 || tuning->path > 4 || tuning->levels < 0 || tuning->slices < 0) return SPEC_ERR_SHAPE;
    a.path = tuning->path; a.levels = tuning->levels; a.slices = tuning->slices;
    a.patience = tuning->patience; a.helpers = tuning->helpers;
  }
  launch_accept(a, static_cast<hipStream_t>(stream));
  return hipGetLastError() == hipSuccess ? SPEC_OK : SPEC_ERR_LAUNCH;
}

int32_t spec_accept(int32_t B, int32_t V, int32_t total_nodes, int32_t n_q_rows, int32_t max_nodes_per_req,
                    const int32_t* node_offsets, const int32_t* parent, const int32_t* draft_tokens,
                    const void* target_logits, int32_t target_dtype, const void* draft_q, int32_t q_dtype,
                    int32_t q_kind, const int32_t* q_row, float temperature, const float* u_accept,
                    const float* u_resample, int32_t* accept_len, int32_t* out_tokens, int32_t out_stride,
                    int32_t* stop_node, float* dbg_ratio, void* workspace, size_t workspace_bytes,
                    void* stream) {
  return accept_entry(false, nullptr, B, V, total_nodes, n_q_rows, max_nodes_per_req, node_offsets, parent, draft_tokens,
                      target_logits, target_dtype, draft_q, q_dtype, q_kind, q_row, temperature, u_accept,
                      u_resample, accept_len, out_tokens, out_stride, stop_node, dbg_ratio, workspace,
                      workspace_bytes, stream);
}

int32_t spec_accept_tuned(const spec_accept_tuning* tuning, int32_t B, int32_t V, int32_t total_nodes,
                          int32_t n_q_rows, int32_t max_nodes_per_req, const int32_t* node_offsets,
                          const int32_t* parent, const int32_t* draft_tokens, const void* target_logits,
                          int32_t target_dtype, const void* draft_q, int32_t q_dtype, int32_t q_kind,
                          const int32_t* q_row, float temperature, const float* u_accept, const float* u_resample,
                          int32_t* accept_len, int32_t* out_tokens, int32_t out_stride, int32_t* stop_node,
                          float* dbg_ratio, void* workspace, size_t workspace_bytes, void* stream) {
  return accept_entry(false, tuning, B, V, total_nodes, n_q_rows, max_nodes_per_req, node_offsets, parent,
                      draft_tokens, target_logits, target_dtype, draft_q, q_dtype, q_kind, q_row, temperature,
                      u_accept, u_resample, accept_len, out_tokens, out_stride, stop_node, dbg_ratio, workspace,
                      workspace_bytes, stream);
}

size_t spec_accept_noalloc_max_workspace(void) { return kNoallocScratchBytes; }

int32_t spec_accept_noalloc(int32_t B, int32_t V, int32_t total_nodes, int32_t n_q_rows, int32_t max_nodes_per_req,
                            const int32_t* node_offsets, const int32_t* parent, const int32_t* draft_tokens,
                            const void* target_logits, int32_t target_dtype, const void* draft_q, int32_t q_dtype,
                            int32_t q_kind, const int32_t* q_row, float temperature, const float* u_accept,
                            const float* u_resample, int32_t* accept_len, int32_t* out_tokens, int32_t out_stride,
                            int32_t* stop_node, float* dbg_ratio, void* stream) {
  if (B < 0 || V <= 0 || total_nodes < 0 || n_q_rows < 0) return SPEC_ERR_SHAPE;
  if (accept_workspace_bytes(B, total_nodes, n_q_rows, V) > kNoallocScratchBytes) return SPEC_ERR_WORKSPACE;
  void* ws = noalloc_scratch_ptr();
  if (!ws) return SPEC_ERR_LAUNCH;
  return accept_entry(false, nullptr, B, V, total_nodes, n_q_rows, max_nodes_per_req, node_offsets, parent,
                      draft_tokens, target_logits, target_dtype, draft_q, q_dtype, q_kind, q_row, temperature,
                      u_accept, u_resample, accept_len, out_tokens, out_stride, stop_node, dbg_ratio, ws,
                      kNoallocScratchBytes, stream);
}

int32_t spec_describe_accept_plan(const spec_accept_tuning* tuning, int32_t B, int32_t V, int32_t total_nodes,
                                  int32_t max_nodes_per_req, int32_t is_tree, int32_t target_dtype, int32_t q_dtype,
                                  int32_t q_kind, char* buf, size_t buf_bytes) {
  if (B < 0 || V <= 0 || max_nodes_per_req < 0 || total_nodes < 0) return SPEC_ERR_SHAPE;
  if (!buf || buf_bytes == 0) return SPEC_ERR_NULL;
  AcceptArgs a{};
  a.B = B; a.V = V; a.total_nodes = total_nodes; a.max_nodes = max_nodes_per_req;
  a.t_dtype = target_dtype; a.q_dtype = q_dtype; a.q_kind = q_kind;
  static const int32_t some_parent = 0;
  a.parent = is_tree ? &some_parent : nullptr;       // only its being NULL or not matters to the plan
  a.patience = -1; a.helpers = -1;
  if (tuning) { a.path = tuning->path; a.levels = tuning->levels; a.slices = tuning->slices; }
  const int n_cu = current_device_cus();
  const char* name = accept_plan_name(a, n_cu);
  const ClusterPlan p = make_cluster_plan(B, V, max_nodes_per_req, is_tree != 0, n_cu, a.levels, a.slices);
  snprintf(buf, buf_bytes, "%s; cluster plan for this shape: %d level(s) x %d slice(s) of %d logits%s", name,
           p.solo ? 1 : p.levels, p.slices, p.upt * 2048, p.solo ? " (one workgroup)" : "");
  return SPEC_OK;
}

int32_t spec_accept_prestats(int32_t B, int32_t V, int32_t total_nodes, int32_t n_q_rows,
                             int32_t max_nodes_per_req, const int32_t* node_offsets, const int32_t* parent,
                             const int32_t* draft_tokens, const void* target_logits, int32_t target_dtype,
                             const void* draft_q, int32_t q_dtype, int32_t q_kind, const int32_t* q_row,
                             float temperature, const float* u_accept, const float* u_resample,
                             int32_t* accept_len, int32_t* out_tokens, int32_t out_stride, int32_t* stop_node,
                             float* dbg_ratio, void* workspace, size_t workspace_bytes, void* stream) {
  if (target_dtype != SPEC_BF16) return SPEC_ERR_UNSUPPORTED;
  return accept_entry(true, nullptr, B, V, total_nodes, n_q_rows, max_nodes_per_req, node_offsets, parent, draft_tokens,
                      target_logits, target_dtype, draft_q, q_dtype, q_kind, q_row, temperature, u_accept,
                      u_resample, accept_len, out_tokens, out_stride, stop_node, dbg_ratio, workspace,
                      workspace_bytes, stream);
}

size_t spec_row_stats_size(int32_t rows, int32_t V) {
  if (rows < 0 || V <= 0) return 0;
  return row_stats_bytes(rows, V);
}

size_t spec_lm_head_workspace_size(int32_t rows, int32_t d_model, int32_t V) {
  if (rows < 0 || d_model <= 0 || V <= 0) return 0;
  return lm_head_workspace_bytes(rows, d_model, V);
}

int32_t spec_lm_head(int32_t rows, int32_t d_model, int32_t V, const void* hidden, const void* weight,
                     float temperature, void* logits, void* target_stats, void* workspace,
                     size_t workspace_bytes, void* stream) {
  if (rows < 0 || d_model <= 0 || V <= 0) return SPEC_ERR_SHAPE;
  if (!(temperature > 0.f)) return SPEC_ERR_SHAPE;
  if (d_model % 128 != 0 || d_model > 65536 || V > 2097152 || rows > 65535) return SPEC_ERR_UNSUPPORTED;
  if (rows == 0) return SPEC_OK;
  if (!hidden || !weight || !logits || !target_stats) return SPEC_ERR_NULL;
  if ((reinterpret_cast<uintptr_t>(hidden) | reinterpret_cast<uintptr_t>(weight)) & 15u) return SPEC_ERR_SHAPE;
  if ((reinterpret_cast<uintptr_t>(logits) & 7u) || (reinterpret_cast<uintptr_t>(target_stats) & 15u))
    return SPEC_ERR_SHAPE;
  if (!workspace || workspace_bytes < lm_head_workspace_bytes(rows, d_model, V)) return SPEC_ERR_WORKSPACE;
  LmHeadArgs a{};
  a.rows = rows; a.d_model = d_model; a.V = V; a.hidden = hidden; a.weight = weight; a.temperature = temperature;
  a.logits = logits; a.stats = target_stats; a.workspace = workspace;
  if (launch_lm_head(a, static_cast<hipStream_t>(stream)) != 0) return SPEC_ERR_LAUNCH;
  return hipGetLastError() == hipSuccess ? SPEC_OK : SPEC_ERR_LAUNCH;
}

size_t spec_accept_greedy_workspace_size(int32_t B, int32_t total_nodes, int32_t V) {
  if (B < 0 || total_nodes < 0 || V <= 0) return 0;
  return greedy_workspace_bytes(B, total_nodes, V);
}

int32_t spec_accept_greedy(int32_t B, int32_t V, int32_t total_nodes, int32_t max_nodes_per_req,
                           const int32_t* node_offsets, const int32_t* parent, const int32_t* draft_tokens,
                           const void* target_logits, int32_t target_dtype, int32_t* accept_len,
                           int32_t* out_tokens, int32_t out_stride, int32_t* stop_node, int32_t* row_argmax,
                           void* workspace, size_t workspace_bytes, void* stream) {
  if (B < 0 || V <= 0 || total_nodes < 0 || max_nodes_per_req < 0) return SPEC_ERR_SHAPE;
  if (max_nodes_per_req > 128) return SPEC_ERR_UNSUPPORTED;
  if (out_stride < max_nodes_per_req + 1) return SPEC_ERR_SHAPE;
  if (target_dtype != SPEC_BF16 && target_dtype != SPEC_F32) return SPEC_ERR_UNSUPPORTED;
  if (static_cast<int64_t>(total_nodes) + B > 65535) return SPEC_ERR_UNSUPPORTED;   // rows are the grid's y dimension
  if (B == 0) return SPEC_OK;
  if (!node_offsets || !target_logits || !accept_len || !out_tokens) return SPEC_ERR_NULL;
  if (total_nodes > 0 && !draft_tokens) return SPEC_ERR_NULL;
  const size_t need = greedy_workspace_bytes(B, total_nodes, V);
  if (!workspace || workspace_bytes < need) return SPEC_ERR_WORKSPACE;
  GreedyArgs a{};
  a.B = B; a.V = V; a.total_nodes = total_nodes; a.node_offsets = node_offsets; a.parent = parent;
  a.draft_tokens = draft_tokens; a.target = target_logits; a.t_dtype = target_dtype; a.accept_len = accept_len;
  a.out_tokens = out_tokens; a.out_stride = out_stride; a.stop_node = stop_node; a.row_argmax = row_argmax;
  a.workspace = workspace;
  launch_accept_greedy(a, static_cast<hipStream_t>(stream));
  return hipGetLastError() == hipSuccess ? SPEC_OK : SPEC_ERR_LAUNCH;
}

int32_t spec_routing_scores(int32_t B, int32_t k_max, int32_t N, int32_t V, int32_t E, const int32_t* k_len,
                            const float* conf, const int32_t* draft_tokens, const int32_t* accept_len,
                            const int32_t* out_tokens, int32_t out_stride, const void* embedding,
                            int32_t embedding_dtype, float* scores, void* stream) {
  if (B < 0 || k_max < 0 || N < 0 || V <= 0 || E <= 0 || out_stride < 0) return SPEC_ERR_SHAPE;
  if (k_max > 64 || N > 16) return SPEC_ERR_UNSUPPORTED;
  if (embedding_dtype != SPEC_BF16 && embedding_dtype != SPEC_F32) return SPEC_ERR_UNSUPPORTED;
  if (B == 0 || N == 0) return SPEC_OK;
  if (!k_len || !accept_len || !scores) return SPEC_ERR_NULL;
  if (k_max > 0 && (!conf || !draft_tokens || !out_tokens || !embedding)) return SPEC_ERR_NULL;
  RoutingArgs a{};
  a.B = B; a.k_max = k_max; a.N = N; a.V = V; a.E = E; a.k_len = k_len; a.conf = conf; a.draft_tokens = draft_tokens;
  a.accept_len = accept_len; a.out_tokens = out_tokens; a.out_stride = out_stride; a.embedding = embedding;
  a.e_dtype = embedding_dtype; a.scores = scores;
  launch_routing_scores(a, static_cast<hipStream_t>(stream));
  return hipGetLastError() == hipSuccess ? SPEC_OK : SPEC_ERR_LAUNCH;
}

int32_t spec_adaptive_speculation(int32_t R, const int32_t* gamma_in, const int32_t* in_batch,
                                  int64_t gamma_max_total, int32_t* gamma_out, int64_t* total_out, void* stream) {
  if (R < 0) return SPEC_ERR_SHAPE;
  if (R == 0) return SPEC_OK;
  if (!gamma_in || !gamma_out) return SPEC_ERR_NULL;
  launch_adaptive_speculation(R, gamma_in, in_batch, static_cast<long long>(gamma_max_total), gamma_out,
                              reinterpret_cast<long long*>(total_out), static_cast<hipStream_t>(stream));
  return hipGetLastError() == hipSuccess ? SPEC_OK : SPEC_ERR_LAUNCH;
}

int32_t spec_compact_kv(int32_t B, int32_t num_kv_heads, int32_t head_dim, int32_t page_size,
                        int32_t max_pages_per_req, void* k_pool, void* v_pool, const int32_t* block_table,
                        const int32_t* ctx_len, const int32_t* q_offsets, const int32_t* parent,
                        const int32_t* stop_node, int32_t* new_len, void* stream) {
  if (B < 0 || num_kv_heads <= 0 || max_pages_per_req < 0) return SPEC_ERR_SHAPE;
  if ((head_dim != 64 && head_dim != 128) || page_size != 16) return SPEC_ERR_UNSUPPORTED;
  if (B > 65535 || num_kv_heads > 65535) return SPEC_ERR_UNSUPPORTED;
  if (B == 0) return SPEC_OK;
  if (!k_pool || !v_pool || !block_table || !ctx_len || !q_offsets || !stop_node) return SPEC_ERR_NULL;
  CompactArgs a{};
  a.B = B; a.Hkv = num_kv_heads; a.D = head_dim; a.max_pages = max_pages_per_req;
  a.k_pool = static_cast<uint16_t*>(k_pool); a.v_pool = static_cast<uint16_t*>(v_pool);
  a.block_table = block_table; a.ctx_len = ctx_len; a.q_offsets = q_offsets; a.parent = parent;
  a.stop_node = stop_node; a.new_len = new_len;
  launch_compact_kv(a, static_cast<hipStream_t>(stream));
  return hipGetLastError() == hipSuccess ? SPEC_OK : SPEC_ERR_LAUNCH;
}

}  // extern "C"
