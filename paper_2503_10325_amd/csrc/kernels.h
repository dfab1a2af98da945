// Host-side launch interfaces between the C-ABI layer and the kernel translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "common.h"

namespace specv {

// ---- accept.hip -------------------------------------------------------------------
struct AcceptParams;
int stats_segments(int V);
void launch_row_stats(const void* t_base, int t_dtype, int n_t_rows, const void* q_base, int q_dtype,
                      int n_q_rows, int V, float c, SegStat* stats, hipStream_t stream,
                      unsigned* zero_words = nullptr, int n_zero = 0, const int32_t* q_row = nullptr,
                      int n_nodes = 0);

struct AcceptArgs {
  int B, V, total_nodes, n_q_rows;
  const int32_t* node_offsets;
  const int32_t* parent;
  const int32_t* draft_tokens;
  const void* target; int t_dtype;
  const void* draft_q; int q_dtype; int q_kind;
  const int32_t* q_row;
  float temperature;
  const float* u_accept;
  const float* u_resample;
  int32_t* accept_len;
  int32_t* out_tokens; int out_stride;
  int32_t* stop_node;
  float* dbg_ratio;
  void* workspace;
  bool target_stats_ready;     // the workspace already starts with the target rows' statistics
};
size_t accept_workspace_bytes(int B, int total_nodes, int n_q_rows, int V);
void launch_accept(const AcceptArgs& a, hipStream_t stream);

// ---- lmhead.hip ------------------------------------------------------------------
struct LmHeadArgs {
  int rows, d_model, V;
  const void* hidden;
  const void* weight;
  float temperature;
  void* logits;
  void* stats;
  void* workspace;
};
size_t lm_head_workspace_bytes(int rows, int d_model, int V);
size_t row_stats_bytes(int rows, int V);
int launch_lm_head(const LmHeadArgs& a, hipStream_t stream);

// ---- greedy.hip -------------------------------------------------------------------
struct GreedyArgs {
  int B, V, total_nodes;
  const int32_t* node_offsets;
  const int32_t* parent;
  const int32_t* draft_tokens;
  const void* target; int t_dtype;
  int32_t* accept_len;
  int32_t* out_tokens; int out_stride;
  int32_t* stop_node;
  int32_t* row_argmax;
  void* workspace;
};
size_t greedy_workspace_bytes(int B, int total_nodes, int V);
void launch_accept_greedy(const GreedyArgs& a, hipStream_t stream);

// ---- routing.hip ------------------------------------------------------------------
struct RoutingArgs {
  int B, k_max, N, V, E;
  const int32_t* k_len;
  const float* conf;
  const int32_t* draft_tokens;
  const int32_t* accept_len;
  const int32_t* out_tokens; int out_stride;
  const void* embedding; int e_dtype;
  float* scores;
};
void launch_routing_scores(const RoutingArgs& a, hipStream_t stream);

// ---- adaptive.hip -----------------------------------------------------------------
void launch_adaptive_speculation(int R, const int32_t* gamma_in, const int32_t* in_batch, long long budget,
                                 int32_t* gamma_out, long long* total_out, hipStream_t stream);

// ---- compact.hip ------------------------------------------------------------------
struct CompactArgs {
  int B, Hkv, D, max_pages;
  uint16_t* k_pool;
  uint16_t* v_pool;
  const int32_t* block_table;
  const int32_t* ctx_len;
  const int32_t* q_offsets;
  const int32_t* parent;
  const int32_t* stop_node;
  int32_t* new_len;
};
void launch_compact_kv(const CompactArgs& a, hipStream_t stream);

// ---- fuse.hip ---------------------------------------------------------------------
struct FuseArgs {
  int B, k_max, N, V;
  const int32_t* k_len;
  const float* conf;
  const int32_t* draft_tokens;
  const void* draft_logits; int l_dtype;
  float temperature;
  int mode;
  int32_t* fused_token;
  int32_t* winner;
  int32_t* q_row;
  float* fused_probs;
  void* workspace;
};
size_t fuse_workspace_bytes(int B, int k_max, int N, int V, int mode);
void launch_fuse(const FuseArgs& a, hipStream_t stream);

// ---- attn.hip ---------------------------------------------------------------------
struct AttnArgs {
  int B, Hq, Hkv, D, page, total_q, max_q, max_pages;
  int64_t kv_hint;
  float scale;
  int out_dtype;
  const void* q;
  const void* k_pool;
  const void* v_pool;
  const int32_t* block_table;
  const int32_t* ctx_len;
  const int32_t* q_offsets;
  const int32_t* parent;
  void* out;
  float* lse;
  void* workspace;
};
size_t attn_workspace_bytes(const AttnArgs& a);
int launch_attn(const AttnArgs& a, hipStream_t stream);   // 0 or a negative spec_status

}  // namespace specv
