// Confidence-based token fusion (Algorithm 1, TokenFusion; Eq. 4 first line of the paper):
// at every draft position keep the token whose own drafter gave it the highest
// probability.  The optional MIXTURE mode forms the confidence-weighted average of the
// drafters' distributions (the "weighted averaging" ensemble of Section 2.2).
#include "common.h"
#include "kernels.h"

namespace specv {

__global__ void fuse_argmax_kernel(int B, int k_max, int N, const int32_t* __restrict__ k_len,
                                   const float* __restrict__ conf, const int32_t* __restrict__ toks,
                                   int mixture, int32_t* __restrict__ fused, int32_t* __restrict__ winner,
                                   int32_t* __restrict__ q_row) {
  const int pos = blockIdx.x * blockDim.x + threadIdx.x;
  if (pos >= B * k_max) return;
  const int b = pos / k_max, i = pos % k_max;
  if (i >= k_len[b]) {
    fused[pos] = -1; winner[pos] = -1; q_row[pos] = -1;
    return;
  }
  const float* c = conf + static_cast<int64_t>(pos) * N;
  int best = 0;
  float bv = c[0];
  for (int n = 1; n < N; ++n) {
    const float v = c[n];
    if (v > bv) { bv = v; best = n; }
  }
  winner[pos] = best;
  fused[pos] = toks[static_cast<int64_t>(pos) * N + best];
  q_row[pos] = mixture ? pos : pos * N + best;
}

// MIXTURE: fused_probs[pos, v] = sum_n w_n 2^((l_nv - m_n) c) / Z_n
constexpr int kMixThreads = 256;
constexpr int kMixSeg = kMixThreads * 8;
constexpr int kMixMaxN = 16;

template <bool VEC>
__global__ __launch_bounds__(kMixThreads) void fuse_mixture_kernel(
    int k_max, int N, int V, const int32_t* __restrict__ k_len, const float* __restrict__ conf,
    const void* __restrict__ logits, int l_dtype, float c, int nseg, const SegStat* __restrict__ stats,
    float* __restrict__ out) {
  const int pos = blockIdx.y;
  const int b = pos / k_max, i = pos % k_max;
  if (i >= k_len[b]) return;
  const int e0 = (blockIdx.x * kMixThreads + threadIdx.x) * 8;
  if (e0 >= V) return;
  double csum = 0.0;
  for (int n = 0; n < N; ++n) csum += static_cast<double>(conf[static_cast<int64_t>(pos) * N + n]);
  double acc[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) acc[j] = 0.0;
  for (int n = 0; n < N; ++n) {
    const int64_t row = static_cast<int64_t>(pos) * N + n;
    float M = -INFINITY;
    for (int s = 0; s < nseg; ++s) M = fmaxf(M, stats[row * nseg + s].m);
    double Z = 0.0;
    for (int s = 0; s < nseg; ++s) {
      const SegStat st = stats[row * nseg + s];
      if (st.m != -INFINITY) Z += st.z * exp2(static_cast<double>(st.m - M) * static_cast<double>(c));
    }
    const double w = (csum > 0.0) ? static_cast<double>(conf[row]) / csum : 1.0 / N;
    const double wz = w / Z;
    float x[8];
    load8<VEC>(logits, l_dtype, row * V, e0, V, x);
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] += wz * static_cast<double>(fast_exp2((x[j] - M) * c));
  }
  float* o = out + static_cast<int64_t>(pos) * V + e0;
  if (VEC && e0 + 8 <= V) {
    float4 a, d;
    a.x = acc[0]; a.y = acc[1]; a.z = acc[2]; a.w = acc[3];
    d.x = acc[4]; d.y = acc[5]; d.z = acc[6]; d.w = acc[7];
    *reinterpret_cast<float4*>(o) = a;
    *reinterpret_cast<float4*>(o + 4) = d;
  } else {
#pragma unroll
    for (int j = 0; j < 8; ++j) if (e0 + j < V) o[j] = static_cast<float>(acc[j]);
  }
}

size_t fuse_workspace_bytes(int B, int k_max, int N, int V, int mode) {
  if (mode != 1) return 0;
  return static_cast<size_t>(B) * k_max * N * stats_segments(V) * sizeof(SegStat) + 256;
}

void launch_fuse(const FuseArgs& a, hipStream_t stream) {
  const int positions = a.B * a.k_max;
  if (positions <= 0) return;
  hipLaunchKernelGGL(fuse_argmax_kernel, dim3((positions + 255) / 256), dim3(256), 0, stream, a.B, a.k_max,
                     a.N, a.k_len, a.conf, a.draft_tokens, a.mode == 1, a.fused_token, a.winner, a.q_row);
  if (a.mode != 1) return;
  const float c = kLog2e / a.temperature;
  SegStat* stats = static_cast<SegStat*>(a.workspace);
  // statistics of every drafter row (rows of unused positions are computed but never read)
  launch_row_stats(a.draft_logits, a.l_dtype, positions * a.N, nullptr, kBF16, 0, a.V, c, stats, stream);
  const int nseg = stats_segments(a.V);
  dim3 grid((a.V + kMixSeg - 1) / kMixSeg, positions);
  if (a.V % 8 == 0 && aligned16(a.draft_logits) && aligned16(a.fused_probs))
    hipLaunchKernelGGL(fuse_mixture_kernel<true>, grid, dim3(kMixThreads), 0, stream, a.k_max, a.N, a.V,
                       a.k_len, a.conf, a.draft_logits, a.l_dtype, c, nseg, stats, a.fused_probs);
  else
    hipLaunchKernelGGL(fuse_mixture_kernel<false>, grid, dim3(kMixThreads), 0, stream, a.k_max, a.N, a.V,
                       a.k_len, a.conf, a.draft_logits, a.l_dtype, c, nseg, stats, a.fused_probs);
}

}  // namespace specv
