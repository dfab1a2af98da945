// Accepted-path compaction of the paged KV cache after a draft tree has been verified.  The paper
// only says that verified drafts go back to the request pool (Section 4.1); for the next step to see
// an ordinary linear context, the K/V entries of the accepted path (root .. stop node, draft node j
// living at logical position ctx + j) move to positions ctx + 0 .. ctx + depth - 1.
//
// One workgroup per (request, KV head): the path is rebuilt from the parent array, every source row
// (K and V, D 16-bit elements) is read into registers, a barrier, then the rows are written to their
// destinations - destinations of one depth can be sources of another, so nothing is written before
// everything is read.  Pure data movement: at most 128 rows of 2*D bytes per tensor, latency-bound.
#include "common.h"
#include "kernels.h"

namespace specv {

constexpr int kCompactThreads = 256;
constexpr int kCompactMaxNodes = 128;

typedef uint32_t cu32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(kCompactThreads) void compact_kv_kernel(
    int Hkv, int D, int max_pages, uint16_t* __restrict__ k_pool, uint16_t* __restrict__ v_pool,
    const int32_t* __restrict__ block_table, const int32_t* __restrict__ ctx_len,
    const int32_t* __restrict__ q_offsets, const int32_t* __restrict__ parent,
    const int32_t* __restrict__ stop_node, int32_t* __restrict__ new_len) {
  constexpr int kPageTokens = 16;
  const int b = blockIdx.x, h = blockIdx.y, tid = threadIdx.x;
  __shared__ int sh_path[kCompactMaxNodes];     // leaf -> root
  __shared__ int sh_depth;
  const int o = q_offsets[b];
  int n = q_offsets[b + 1] - o;
  n = n < 0 ? 0 : (n > kCompactMaxNodes ? kCompactMaxNodes : n);
  const int ctx = ctx_len[b];
  if (tid == 0) {
    int depth = 0;
    int a = stop_node[b];
    while (a >= 0 && a < n && depth < kCompactMaxNodes) {
      sh_path[depth++] = a;
      const int p = parent ? parent[o + a] : a - 1;
      a = (p < a) ? p : -1;                     // a malformed parent entry ends the path
    }
    sh_depth = depth;
    if (h == 0 && new_len) new_len[b] = ctx + depth;
  }
  __syncthreads();
  const int depth = sh_depth;
  if (depth == 0) return;
  const int chunks = D / 8;                      // 16-byte chunks per row
  const int items = depth * 2 * chunks;          // (position on the path, K or V, chunk)
  const int32_t* bt = block_table + static_cast<int64_t>(b) * max_pages;
  const int64_t page_elems = static_cast<int64_t>(Hkv) * kPageTokens * D;
  constexpr int kPerThread = (kCompactMaxNodes * 2 * 16 + kCompactThreads - 1) / kCompactThreads;   // D <= 128
  cu32x4 held[kPerThread];
#pragma unroll
  for (int r = 0; r < kPerThread; ++r) {
    const int it = r * kCompactThreads + tid;
    if (it < items) {
      const int d = it / (2 * chunks), rem = it % (2 * chunks), which = rem / chunks, c = rem % chunks;
      const int pos = ctx + sh_path[depth - 1 - d];
      const int64_t src = bt[pos / kPageTokens] * page_elems + (static_cast<int64_t>(h) * kPageTokens + pos % kPageTokens) * D + c * 8;
      held[r] = *reinterpret_cast<const cu32x4*>((which ? v_pool : k_pool) + src);
    }
  }
  __syncthreads();                               // every source row is in registers
#pragma unroll
  for (int r = 0; r < kPerThread; ++r) {
    const int it = r * kCompactThreads + tid;
    if (it < items) {
      const int d = it / (2 * chunks), rem = it % (2 * chunks), which = rem / chunks, c = rem % chunks;
      const int pos = ctx + d;
      const int64_t dst = bt[pos / kPageTokens] * page_elems + (static_cast<int64_t>(h) * kPageTokens + pos % kPageTokens) * D + c * 8;
      *reinterpret_cast<cu32x4*>((which ? v_pool : k_pool) + dst) = held[r];
    }
  }
}

void launch_compact_kv(const CompactArgs& a, hipStream_t stream) {
  if (a.B <= 0 || a.Hkv <= 0) return;
  hipLaunchKernelGGL(compact_kv_kernel, dim3(a.B, a.Hkv), dim3(kCompactThreads), 0, stream, a.Hkv, a.D, a.max_pages,
                     a.k_pool, a.v_pool, a.block_table, a.ctx_len, a.q_offsets, a.parent, a.stop_node, a.new_len);
}

}  // namespace specv
