// Routing-score update that follows acceptance (Section 4.1 of the paper, Eq. 1 and Eq. 2):
//   d[b,i,n] = cos(H(accepted token i), H(draft token of drafter n at i))   for i < accept_len[b], else 0
//   score[b,n] = (1/K) sum_i c d / (c d + (1-c)(1-d)),  K = k_len[b]
// H = rows of an embedding table.  Where the paper is silent: a negative cosine counts as 0, a zero
// row gives cosine 0, a term whose denominator is not positive is 0, K = 0 gives 0.
//
// One 1024-thread workgroup per (request, drafter); each wave takes draft positions, streams the two
// embedding rows with 16-byte loads, four per row in flight (a gather of a few rows of 2E bytes:
// latency-bound), reduces dot product and norms (fp32 per lane, fp64 across lanes) and leaves the
// term in LDS; one thread then adds the terms in position order, so the result does not depend on
// scheduling.
#include "common.h"
#include "kernels.h"

namespace specv {

constexpr int kRouteThreads = 1024;
constexpr int kRouteWaves = kRouteThreads / kWave;
constexpr int kRouteMaxPos = 64;
constexpr int kRouteDepth = 4;                 // 512-element blocks of a row in flight per wave

template <bool VEC>
__global__ __launch_bounds__(kRouteThreads) void routing_scores_kernel(
    int k_max, int N, int V, int E, const int32_t* __restrict__ k_len, const float* __restrict__ conf,
    const int32_t* __restrict__ toks, const int32_t* __restrict__ accept_len, const int32_t* __restrict__ out_tokens,
    int out_stride, const void* __restrict__ emb, int e_dtype, float* __restrict__ scores) {
  const int b = blockIdx.x, n = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  __shared__ double sh_term[kRouteMaxPos];
  const int K = min(max(k_len[b], 0), k_max);
  const int Lacc = min(max(accept_len[b], 0), min(K, out_stride));
  if (tid < kRouteMaxPos) sh_term[tid] = 0.0;          // positions past Lacc keep d = 0: term 0
  __syncthreads();
  for (int i = wave; i < Lacc; i += kRouteWaves) {
    const int ta = min(max(out_tokens[static_cast<int64_t>(b) * out_stride + i], 0), V - 1);
    const int tx = min(max(toks[(static_cast<int64_t>(b) * k_max + i) * N + n], 0), V - 1);
    const int64_t ra = static_cast<int64_t>(ta) * E, rx = static_cast<int64_t>(tx) * E;
    float dot = 0.f, na = 0.f, nx = 0.f;
    for (int base = 0; base < E; base += kRouteDepth * kWave * 8) {
      float a[kRouteDepth][8], x[kRouteDepth][8];
#pragma unroll
      for (int u = 0; u < kRouteDepth; ++u) {          // all loads first; blocks past the row end re-read its start
        const int e0 = base + (u * kWave + lane) * 8;
        const int es = e0 < E ? e0 : 0;
        load8<VEC>(emb, e_dtype, ra, es, E, a[u]);
        load8<VEC>(emb, e_dtype, rx, es, E, x[u]);
      }
#pragma unroll
      for (int u = 0; u < kRouteDepth; ++u) {
        const int e0 = base + (u * kWave + lane) * 8;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const bool in = e0 + j < E;                  // also masks the -inf padding of a ragged row end
          const float av = in ? a[u][j] : 0.f, xv = in ? x[u][j] : 0.f;
          dot = fmaf(av, xv, dot); na = fmaf(av, av, na); nx = fmaf(xv, xv, nx);
        }
      }
    }
    const double sd = wave_sum(static_cast<double>(dot));
    const double sa = wave_sum(static_cast<double>(na));
    const double sx = wave_sum(static_cast<double>(nx));
    if (lane == 0) {
      double d = 0.0;
      if (sa > 0.0 && sx > 0.0) d = sd / (sqrt(sa) * sqrt(sx));
      d = d < 0.0 ? 0.0 : (d > 1.0 ? 1.0 : d);
      const double c = static_cast<double>(conf[(static_cast<int64_t>(b) * k_max + i) * N + n]);
      const double den = c * d + (1.0 - c) * (1.0 - d);
      sh_term[i] = den > 0.0 ? c * d / den : 0.0;
    }
  }
  __syncthreads();
  if (tid == 0) {
    double sum = 0.0;
    for (int i = 0; i < K; ++i) sum += sh_term[i];
    scores[static_cast<int64_t>(b) * N + n] = K > 0 ? static_cast<float>(sum / static_cast<double>(K)) : 0.f;
  }
}

void launch_routing_scores(const RoutingArgs& a, hipStream_t stream) {
  if (a.B <= 0 || a.N <= 0) return;
  const bool vec = (a.E % 8 == 0) && aligned16(a.embedding);
  if (vec)
    hipLaunchKernelGGL(routing_scores_kernel<true>, dim3(a.B, a.N), dim3(kRouteThreads), 0, stream, a.k_max, a.N, a.V, a.E,
                       a.k_len, a.conf, a.draft_tokens, a.accept_len, a.out_tokens, a.out_stride, a.embedding,
                       a.e_dtype, a.scores);
  else
    hipLaunchKernelGGL(routing_scores_kernel<false>, dim3(a.B, a.N), dim3(kRouteThreads), 0, stream, a.k_max, a.N, a.V, a.E,
                       a.k_len, a.conf, a.draft_tokens, a.accept_len, a.out_tokens, a.out_stride, a.embedding,
                       a.e_dtype, a.scores);
}

}  // namespace specv
