// Host-side launch interfaces between the C-ABI layer and the kernel translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>

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
  int B, V, total_nodes, n_q_rows, max_nodes;
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
  // per-call tuning (spec_accept_tuned); zero / negative = the library's choice
  int path;                    // 0: library's choice, 1: statistics kernel + one-workgroup walk, 2: workgroup clusters,
                               // 3 / 4: linear-draft kernel after the statistics of all rows / of the rows up to each first rejection
  int levels, slices;          // cluster path: window levels, vocabulary slices per level
  int patience;                // polls spent waiting for peer workgroups (< 0: default)
  int helpers;                 // statistics + walk path: helper workgroups per request (< 0: default)
};

// ---- accept_cluster.hip -----------------------------------------------------------
struct ClusterPlan {
  int upt;                     // 16-byte loads per thread and row: a slice is upt x 2048 logits
  int levels, slices;          // workgroups per request = levels x slices
  int solo;                    // one workgroup per request computes every part itself
};
constexpr int kClusterMaxV = 32 * 16 * 2048;  // 32 slices of 16 x 2048 logits
ClusterPlan make_cluster_plan(int B, int V, int max_nodes, bool tree, int n_cu, int want_levels, int want_slices);
size_t cluster_msg_bytes(int B);
void launch_accept_cluster(const AcceptArgs& a, const ClusterPlan& plan, int patience, void* msg, hipStream_t stream);
size_t accept_workspace_bytes(int B, int total_nodes, int n_q_rows, int V);
void launch_accept(const AcceptArgs& a, hipStream_t stream);
const char* accept_plan_name(const AcceptArgs& a, int n_cu);

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
// The launch plan is a pure function of the descriptor; the workspace-size query and the launch both
// take the plan object the C-ABI layer computed, so the two can never disagree.
struct AttnPlan {
  int kind;           // 0: token-split kernel, 1: row-split, 4 waves, 2: row-split, 8 waves, 3: row-split, 8 waves, sliced
  int rows_per_wg;
  int row_groups;
  int chunk_tokens;
  int max_chunks;
  int tau;            // > 0: sorted-work-list launch of the token-split kernel, at most tau tiles per wave and item
  int wide;           // more than 64 query nodes per request: kernels with two ancestor-mask words per node
};
AttnPlan make_attn_plan(const AttnArgs& a);
size_t attn_workspace_bytes(const AttnArgs& a, const AttnPlan& plan);
const char* attn_plan_name(const AttnPlan& plan);
int launch_attn(const AttnArgs& a, const AttnPlan& plan, hipStream_t stream);   // 0 or a negative spec_status

// Vector (16-byte) accesses need 16-byte aligned base pointers; the launchers pick the scalar
// variants of their kernels when a caller's pointer is not.
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// The dynamic-LDS limit of a kernel is raised once per device (the attribute belongs to the
// device's copy of the function); the mask is the only state kept, and it is per device.
template <typename K>
inline int set_lds_once(K kernel, size_t lds, std::atomic<uint64_t>& done_mask) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return -6;
  const uint64_t bit = 1ull << (dev & 63);
  if (dev < 64 && (done_mask.load(std::memory_order_acquire) & bit)) return 0;
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                          static_cast<int>(lds)) != hipSuccess)
    return -6;
  if (dev < 64) done_mask.fetch_or(bit, std::memory_order_release);
  return 0;
}

// Compute units of the current device, asked on every call (nothing is cached between calls).
inline int current_device_cus() {
  int dev = 0, n = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
    n = 256;
  return n;
}

}  // namespace specv
