// Greedy verification for gfx950 (Section 6.1 of the paper: draft generation and verification
// both use greedy sampling): a draft token is kept when it equals the target's most likely token
// at its position; the first mismatch is replaced by that token, and a fully accepted draft gets
// the most likely token after its last node as a bonus.
//
// Two kernels:
//   row_argmax_kernel   one workgroup per (row, 8192-token segment): the segment's largest logit
//                       and its lowest index, as one ordered 64-bit key.  Pure streaming, HBM-bound.
//   greedy_walk_kernel  one workgroup per request: merges the segment keys of its rows, then one
//                       wave walks the draft (lane j owns node j; a ballot finds the first child of
//                       the current node that proposes the argmax).
//
// Order of logits: ordinary fp32 comparison, -0 equal to +0, NaN treated as -inf; among equal
// values the lowest token index wins.  All of it is integer work after the bf16/fp32 load, so the
// results are exact.
#include "common.h"
#include "kernels.h"

namespace specv {

constexpr int kArgThreads = 256;
constexpr int kArgPerThread = 32;                              // 4 loads of 8
constexpr int kArgSeg = kArgThreads * kArgPerThread;           // 8192 tokens per workgroup

int argmax_segments(int V) { return (V + kArgSeg - 1) / kArgSeg; }

// Monotone map fp32 -> u32 after canonicalisation (NaN -> -inf, -0 -> +0).
__device__ __forceinline__ uint32_t ordered_bits(float x) {
  x = (x != x) ? -INFINITY : x + 0.f;
  const uint32_t b = __float_as_uint(x);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

// key = (ordered value, ~index): the larger key is the larger value, then the lower index.
__device__ __forceinline__ unsigned long long make_key(float x, int idx) {
  return (static_cast<unsigned long long>(ordered_bits(x)) << 32) | static_cast<uint32_t>(~static_cast<uint32_t>(idx));
}
__device__ __forceinline__ int key_index(unsigned long long k) { return static_cast<int>(~static_cast<uint32_t>(k)); }

__device__ __forceinline__ unsigned long long wave_max_u64(unsigned long long k) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const unsigned long long other = __shfl_xor(k, o, kWave);
    k = other > k ? other : k;
  }
  return k;
}

template <bool VEC>
__global__ __launch_bounds__(kArgThreads) void row_argmax_kernel(const void* __restrict__ base, int dtype, int V,
                                                                 int nseg, unsigned long long* __restrict__ keys) {
  const int seg = blockIdx.x, row = blockIdx.y;
  const int64_t row_off = static_cast<int64_t>(row) * V;
  const int e_seg = seg * kArgSeg;
  float x[kArgPerThread];
#pragma unroll
  for (int j = 0; j < kArgPerThread / 8; ++j) {
    float v8[8];
    load8<VEC>(base, dtype, row_off, e_seg + (j * kArgThreads + threadIdx.x) * 8, V, v8);
#pragma unroll
    for (int i = 0; i < 8; ++i) x[j * 8 + i] = v8[i];
  }
  // within the thread the indices ascend, so "strictly greater" keeps the lowest index
  float best = -INFINITY;
  int best_i = e_seg + threadIdx.x * 8;
#pragma unroll
  for (int j = 0; j < kArgPerThread / 8; ++j)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float v = x[j * 8 + i];              // positions >= V were loaded as -inf
      if (v > best) { best = v; best_i = e_seg + (j * kArgThreads + threadIdx.x) * 8 + i; }
    }
  // a thread whose elements are all -inf / NaN / beyond V proposes its first index; the key order
  // still prefers any lower index with the same value, and index < V holds for the winner because
  // thread 0 of segment 0 proposes index 0
  unsigned long long k = make_key(best, min(best_i, V - 1));
  k = wave_max_u64(k);
  __shared__ unsigned long long sh[kArgThreads / kWave];
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = k;
  __syncthreads();
  if (threadIdx.x == 0) {
    unsigned long long m = sh[0];
#pragma unroll
    for (int w = 1; w < kArgThreads / kWave; ++w) m = sh[w] > m ? sh[w] : m;
    keys[static_cast<int64_t>(row) * nseg + seg] = m;
  }
}

constexpr int kGreedyThreads = 192;
constexpr int kGreedyMaxNodes = 128;
static_assert(kGreedyThreads > kGreedyMaxNodes, "one thread per target row of a request");

__global__ __launch_bounds__(kGreedyThreads) void greedy_walk_kernel(
    int V, int nseg, const int32_t* __restrict__ node_offsets, const int32_t* __restrict__ parent,
    const int32_t* __restrict__ draft_tokens, const unsigned long long* __restrict__ keys,
    int32_t* __restrict__ accept_len, int32_t* __restrict__ out_tokens, int out_stride,
    int32_t* __restrict__ stop_node, int32_t* __restrict__ row_argmax) {
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63;
  const int o = node_offsets[b];
  int n = node_offsets[b + 1] - o;
  n = n < 0 ? 0 : (n > kGreedyMaxNodes ? kGreedyMaxNodes : n);
  const int64_t trow0 = static_cast<int64_t>(o) + b;
  __shared__ int sh_arg[kGreedyMaxNodes + 1];
  // argmax of the request's n+1 target rows: thread i merges the segment keys of local row i
  if (tid <= n) {
    const unsigned long long* kr = keys + (trow0 + tid) * nseg;
    unsigned long long m = kr[0];
    for (int s = 1; s < nseg; ++s) { const unsigned long long k = kr[s]; m = k > m ? k : m; }
    const int g = min(max(key_index(m), 0), V - 1);
    sh_arg[tid] = g;
    if (row_argmax) row_argmax[trow0 + tid] = g;
  }
  __syncthreads();
  if (tid >= kWave) return;
  // lane j owns nodes j and j + 64 (nodes that do not exist hold an impossible parent)
  int my_parent[2] = {-2, -2}, my_tok[2] = {-1, -1};
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int node = lane + kWave * h;
    if (node < n) {
      int par = parent ? parent[o + node] : node - 1;
      if (par < -1 || par >= node) par = -1;                      // same repair as the stochastic walk
      my_parent[h] = par;
      my_tok[h] = draft_tokens[o + node];
    }
  }
  int cur = -1, depth = 0;
  for (int guard = 0; guard <= kGreedyMaxNodes; ++guard) {
    const int g = sh_arg[cur + 1];
    if (lane == 0 && depth < out_stride) out_tokens[static_cast<int64_t>(b) * out_stride + depth] = g;
    // the lowest-numbered child of the current node that proposes the argmax
    const unsigned long long hit = __ballot(my_parent[0] == cur && lane > cur && my_tok[0] == g);
    const unsigned long long hit_hi = __ballot(my_parent[1] == cur && lane + kWave > cur && my_tok[1] == g);
    if (!(hit | hit_hi)) break;
    cur = hit ? __ffsll(static_cast<long long>(hit)) - 1 : kWave + __ffsll(static_cast<long long>(hit_hi)) - 1;
    ++depth;
  }
  if (lane == 0) {
    accept_len[b] = depth;
    if (stop_node) stop_node[b] = cur;
  }
  for (int i = depth + 1 + lane; i < out_stride; i += kWave) out_tokens[static_cast<int64_t>(b) * out_stride + i] = -1;
}

size_t greedy_workspace_bytes(int B, int total_nodes, int V) {
  return (static_cast<size_t>(total_nodes) + B) * argmax_segments(V) * sizeof(unsigned long long) + 256;
}

void launch_accept_greedy(const GreedyArgs& a, hipStream_t stream) {
  if (a.B <= 0) return;
  const int rows = a.total_nodes + a.B;
  const int nseg = argmax_segments(a.V);
  unsigned long long* keys = static_cast<unsigned long long*>(a.workspace);
  const dim3 grid(nseg, rows);
  const bool vec = (a.V % 8 == 0) && aligned16(a.target);
  if (vec)
    hipLaunchKernelGGL(row_argmax_kernel<true>, grid, dim3(kArgThreads), 0, stream, a.target, a.t_dtype, a.V, nseg, keys);
  else
    hipLaunchKernelGGL(row_argmax_kernel<false>, grid, dim3(kArgThreads), 0, stream, a.target, a.t_dtype, a.V, nseg, keys);
  hipLaunchKernelGGL(greedy_walk_kernel, dim3(a.B), dim3(kGreedyThreads), 0, stream, a.V, nseg, a.node_offsets,
                     a.parent, a.draft_tokens, keys, a.accept_len, a.out_tokens, a.out_stride, a.stop_node,
                     a.row_argmax);
}

}  // namespace specv
