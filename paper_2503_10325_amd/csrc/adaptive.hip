// AdaptiveSpeculation of Algorithm 2 of the paper: while the draft tokens of the batch exceed the
// verification budget Gamma_max, the request with the most draft tokens (lowest index on ties) gives
// one up; every request keeps at least one (the batch formulation's gamma_i >= 1, Section 4.3).
//
// The loop's result has a closed form, which is what the kernel computes: with D = sum - Gamma_max
// decrements to spend (at most sum (gamma_i - 1)), find the lowest level t >= 1 such that cutting
// every request down to t costs no more than D; the D - cost(t) decrements left over take the
// requests standing at t one token further down, lowest index first.  One workgroup; sums in 64 bits;
// integer work, so parity with the sequential loop is exact.
#include "common.h"
#include "kernels.h"

namespace specv {

constexpr int kAdaptThreads = 1024;

__device__ __forceinline__ long long block_sum_ll(long long v, long long* sh) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  __syncthreads();                                  // previous users of sh are done
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  long long t = 0;
  for (int w = 0; w < kAdaptThreads / kWave; ++w) t += sh[w];
  return t;
}

__global__ __launch_bounds__(kAdaptThreads) void adaptive_speculation_kernel(
    int R, const int32_t* __restrict__ gamma_in, const int32_t* __restrict__ in_batch, long long budget,
    int32_t* __restrict__ gamma_out, long long* __restrict__ total_out) {
  __shared__ long long sh[kAdaptThreads / kWave];
  __shared__ int sh_max[kAdaptThreads / kWave];
  const int tid = threadIdx.x;
  auto member = [&](int i) { return !in_batch || in_batch[i] != 0; };
  // totals over the batch
  long long s = 0, room = 0;
  int mx = 1;
  for (int i = tid; i < R; i += kAdaptThreads) {
    if (!member(i)) continue;
    const int g = gamma_in[i];
    s += g;
    room += g > 1 ? g - 1 : 0;
    mx = max(mx, g);
  }
  const long long sum = block_sum_ll(s, sh);
  const long long max_cut = block_sum_ll(room, sh);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) mx = max(mx, __shfl_xor(mx, o, kWave));
  if ((tid & 63) == 0) sh_max[tid >> 6] = mx;
  __syncthreads();
  for (int w = 0; w < kAdaptThreads / kWave; ++w) mx = max(mx, sh_max[w]);
  long long D = sum - budget;
  if (D > max_cut) D = max_cut;
  if (D <= 0) {                                      // within budget: nothing changes
    for (int i = tid; i < R; i += kAdaptThreads) gamma_out[i] = gamma_in[i];
    if (total_out && tid == 0) *total_out = sum;
    return;
  }
  // lowest level t in [1, mx] with cost(t) = sum max(gamma - t, 0) <= D (cost is non-increasing in t)
  int lo = 1, hi = mx;                               // cost(mx) = 0 <= D
  long long cost_hi = 0;
  while (lo < hi) {
    const int mid = lo + (hi - lo) / 2;
    long long c = 0;
    for (int i = tid; i < R; i += kAdaptThreads)
      if (member(i)) { const int g = gamma_in[i]; c += g > mid ? g - mid : 0; }
    c = block_sum_ll(c, sh);
    if (c <= D) { hi = mid; cost_hi = c; } else lo = mid + 1;
  }
  const int t = hi;
  long long rest = D - cost_hi;                      // requests at level t that go down to t - 1, lowest index first
  // index-ordered assignment: running count of requests with gamma >= t
  __shared__ int sh_cnt[kAdaptThreads / kWave];
  long long seen = 0;                                // such requests in earlier chunks
  for (int base = 0; base < R; base += kAdaptThreads) {
    const int i = base + tid;
    int g = 0;
    bool mem = false;
    if (i < R) { g = gamma_in[i]; mem = member(i); }
    const bool tall = mem && g >= t && t > 1;
    const unsigned long long bal = __ballot(tall);
    const int before_in_wave = __popcll(bal & ((1ull << (tid & 63)) - 1ull));
    __syncthreads();
    if ((tid & 63) == 0) sh_cnt[tid >> 6] = __popcll(bal);
    __syncthreads();
    int before = 0, chunk_total = 0;
    for (int w = 0; w < kAdaptThreads / kWave; ++w) {
      if (w < (tid >> 6)) before += sh_cnt[w];
      chunk_total += sh_cnt[w];
    }
    if (i < R) {
      int out = g;
      if (mem && g > t) out = t;
      if (tall && seen + before + before_in_wave < rest) out = t - 1;
      gamma_out[i] = out;
    }
    seen += chunk_total;
  }
  if (total_out && tid == 0) *total_out = sum - D;
}

void launch_adaptive_speculation(int R, const int32_t* gamma_in, const int32_t* in_batch, long long budget,
                                 int32_t* gamma_out, long long* total_out, hipStream_t stream) {
  if (R <= 0) return;
  hipLaunchKernelGGL(adaptive_speculation_kernel, dim3(1), dim3(kAdaptThreads), 0, stream, R, gamma_in, in_batch,
                     budget, gamma_out, total_out);
}

}  // namespace specv
