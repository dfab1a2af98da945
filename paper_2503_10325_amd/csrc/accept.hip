// Vocab-wide softmax statistics and the acceptance-rejection walk (Section 2.1 of the
// paper: accept x_i when q_i(x_i) <= o_i(x_i), else reject with probability
// 1 - o_i(x_i)/q_i(x_i); replacement from norm(max(0, o_i - q_i)); bonus token when
// nothing is rejected), extended to sibling drafts of a tree by recursive rejection.
//
// Two kernels:
//   row_stats_kernel    one workgroup per (row, vocab segment): segment maximum and
//                       sum of 2^((l-m)c).  Pure streaming, HBM-bound.
//   accept_walk_kernel  one workgroup per request: the sequential walk; every full
//                       pass over a row pair (residual mass, inverse-CDF search) is
//                       spread over the workgroup's 16 waves.
#include "common.h"
#include "kernels.h"

namespace specv {

// ----------------------------------------------------------------------------------
// row statistics
// ----------------------------------------------------------------------------------
constexpr int kStatThreads = 256;
constexpr int kStatPerThread = 32;                              // 4 x 8 elements
constexpr int kStatSeg = kStatThreads * kStatPerThread;         // 8192 logits per workgroup

int stats_segments(int V) { return (V + kStatSeg - 1) / kStatSeg; }

template <bool VEC>
__global__ __launch_bounds__(kStatThreads) void row_stats_kernel(
    const void* __restrict__ t_base, int t_dtype, int n_t_rows,
    const void* __restrict__ q_base, int q_dtype, int n_q_rows,
    int V, float c, int nseg, SegStat* __restrict__ stats) {
  const int seg = blockIdx.x;
  const int row = blockIdx.y;
  const void* base = t_base;
  int dtype = t_dtype;
  int64_t r = row;
  if (row >= n_t_rows) { base = q_base; dtype = q_dtype; r = row - n_t_rows; }
  const int64_t row_off = r * static_cast<int64_t>(V);
  const int e_seg = seg * kStatSeg;

  float x[kStatPerThread];
#pragma unroll
  for (int j = 0; j < kStatPerThread / 8; ++j) {
    float v8[8];
    load8<VEC>(base, dtype, row_off, e_seg + (j * kStatThreads + threadIdx.x) * 8, V, v8);
#pragma unroll
    for (int i = 0; i < 8; ++i) x[j * 8 + i] = v8[i];
  }
  float m = x[0];
#pragma unroll
  for (int i = 1; i < kStatPerThread; ++i) m = fmaxf(m, x[i]);
  const float mm = (m == -INFINITY) ? 0.f : m;
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < kStatPerThread; ++i) s += fast_exp2((x[i] - mm) * c);

  // workgroup combine: maximum first, then rescaled sums in fp64
  __shared__ float sh_m[kStatThreads / kWave];
  __shared__ double sh_z[kStatThreads / kWave];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const float wm = wave_max(m);
  if (lane == 0) sh_m[wave] = wm;
  __syncthreads();
  float M = sh_m[0];
#pragma unroll
  for (int w = 1; w < kStatThreads / kWave; ++w) M = fmaxf(M, sh_m[w]);
  const float MM = (M == -INFINITY) ? 0.f : M;
  double z = static_cast<double>(s) * static_cast<double>(fast_exp2((mm - MM) * c));
  if (m == -INFINITY) z = 0.0;
  z = wave_sum(z);
  if (lane == 0) sh_z[wave] = z;
  __syncthreads();
  if (threadIdx.x == 0) {
    double Z = 0.0;
#pragma unroll
    for (int w = 0; w < kStatThreads / kWave; ++w) Z += sh_z[w];
    SegStat st;
    st.m = M; st.pad = 0.f; st.z = Z;
    stats[static_cast<int64_t>(row) * nseg + seg] = st;
  }
}

void launch_row_stats(const void* t_base, int t_dtype, int n_t_rows, const void* q_base, int q_dtype,
                      int n_q_rows, int V, float c, SegStat* stats, hipStream_t stream) {
  const int rows = n_t_rows + n_q_rows;
  if (rows <= 0 || V <= 0) return;
  const int nseg = stats_segments(V);
  dim3 grid(nseg, rows);
  const bool vec = (V % 8 == 0);
  if (vec)
    hipLaunchKernelGGL(row_stats_kernel<true>, grid, dim3(kStatThreads), 0, stream, t_base, t_dtype,
                       n_t_rows, q_base, q_dtype, n_q_rows, V, c, nseg, stats);
  else
    hipLaunchKernelGGL(row_stats_kernel<false>, grid, dim3(kStatThreads), 0, stream, t_base, t_dtype,
                       n_t_rows, q_base, q_dtype, n_q_rows, V, c, nseg, stats);
}

// ----------------------------------------------------------------------------------
// walk
// ----------------------------------------------------------------------------------
constexpr int kWalkThreads = 1024;
constexpr int kWalkWaves = kWalkThreads / kWave;
constexpr int kMaxNodes = 64;

struct RowStat {
  float m;    // largest logit of the row
  double z;   // sum_v 2^((l_v - m) c)
};

__device__ __forceinline__ RowStat merge_stats(const SegStat* __restrict__ stats, int64_t row, int nseg, float c) {
  float M = -INFINITY;
  for (int s = 0; s < nseg; ++s) M = fmaxf(M, stats[row * nseg + s].m);
  double Z = 0.0;
  for (int s = 0; s < nseg; ++s) {
    const SegStat st = stats[row * nseg + s];
    if (st.m != -INFINITY)
      Z += st.z * exp2(static_cast<double>(st.m - M) * static_cast<double>(c));
  }
  RowStat r;
  r.m = M; r.z = Z;
  return r;
}

struct WalkRows {
  const void* t_base; int t_dtype; int64_t t_off; float t_m; double t_invz;   // target row
  const void* q_base; int q_dtype; int64_t q_off; float q_m; double q_invz;   // draft row
  int q_is_probs;
  int have_q;       // level 0 needs no draft row
};

// Weight of token class v at residual level L (L rejections so far at this node):
//   level 0: p_v;  level k>=1: max(0, w_{k-1}(v)/R_{k-1} - q_v)  with R_{-1} := 1... written
//   out: r_0 = p; w_k = max(0, r_{k-1} - q); r_k = w_k / R_k.
__device__ __forceinline__ double level_weight(double p, double q, int L, const double* __restrict__ inv_R) {
  double r = p;
  for (int k = 0; k < L; ++k) {
    double w = r - q;
    w = w > 0.0 ? w : 0.0;
    r = (k + 1 < L) ? w * inv_R[k] : w;      // the last level stays unnormalised
  }
  return r;
}

template <bool VEC>
__device__ __forceinline__ void weights8(const WalkRows& R, int e0, int V, float c, int L,
                                         const double* __restrict__ inv_R, double (&w)[8]) {
  float lp[8], lq[8];
  load8<VEC>(R.t_base, R.t_dtype, R.t_off, e0, V, lp);
  if (L > 0) load8<VEC>(R.q_base, R.q_dtype, R.q_off, e0, V, lq);
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const double p = static_cast<double>(fast_exp2((lp[j] - R.t_m) * c)) * R.t_invz;
    double q = 0.0;
    if (L > 0) {
      if (R.q_is_probs) q = (e0 + j < V) ? static_cast<double>(lq[j]) : 0.0;
      else q = static_cast<double>(fast_exp2((lq[j] - R.q_m) * c)) * R.q_invz;
    }
    w[j] = level_weight(p, q, L, inv_R);
  }
}

struct AcceptParams {
  int B, V, n_t_rows, nseg;
  const int32_t* node_offsets;
  const int32_t* parent;
  const int32_t* draft_tokens;
  const void* target; int t_dtype;
  const void* draft_q; int q_dtype; int q_kind;
  const int32_t* q_row;
  float c;                  // log2(e)/T
  const float* u_accept;
  const float* u_resample;
  int32_t* accept_len;
  int32_t* out_tokens; int out_stride;
  int32_t* stop_node;
  float* dbg_ratio;
  const SegStat* stats;
};

template <bool VEC>
__global__ __launch_bounds__(kWalkThreads) void accept_walk_kernel(AcceptParams P) {
  const int b = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int o = P.node_offsets[b];
  int n = P.node_offsets[b + 1] - o;
  n = n < 0 ? 0 : (n > kMaxNodes ? kMaxNodes : n);
  const int64_t trow0 = static_cast<int64_t>(o) + b;
  const int V = P.V;
  const float c = P.c;
  // contiguous vocab segment of each wave, a multiple of 512 tokens
  const int seg_w = (((V + kWalkWaves - 1) / kWalkWaves) + 511) / 512 * 512;

  __shared__ double sh_wave_sum[kWalkWaves];
  __shared__ double sh_inv_R[kMaxNodes];
  __shared__ int sh_token;
  // per-request tables filled once, in parallel, so that the walk itself touches no global memory
  __shared__ float sh_tm[kMaxNodes + 1];       // target local row i: max logit
  __shared__ double sh_tinvz[kMaxNodes + 1];   //                     1 / sum 2^((l-m)c)
  __shared__ float sh_qm[kMaxNodes];           // draft row of node j
  __shared__ double sh_qinvz[kMaxNodes];
  __shared__ int sh_par[kMaxNodes], sh_tok[kMaxNodes], sh_qrow[kMaxNodes];
  __shared__ double sh_px[kMaxNodes], sh_qx[kMaxNodes];   // p_parent(x_j), q(x_j)
  __shared__ float sh_u[kMaxNodes];

  const bool q_is_probs = (P.q_kind == 1);
  if (wave == 0) {
    if (lane <= n) {
      const RowStat ps = merge_stats(P.stats, trow0 + lane, P.nseg, c);
      sh_tm[lane] = ps.m;
      sh_tinvz[lane] = 1.0 / ps.z;
    }
  } else if (wave == 1) {
    if (lane < n) {
      int par = P.parent ? P.parent[o + lane] : lane - 1;
      if (par < -1 || par >= lane) par = -1;
      const int qr = P.q_row[o + lane];
      sh_par[lane] = par;
      sh_tok[lane] = P.draft_tokens[o + lane];
      sh_qrow[lane] = qr;
      sh_u[lane] = P.u_accept[o + lane];
      if (!q_is_probs) {
        const RowStat qs = merge_stats(P.stats, static_cast<int64_t>(P.n_t_rows) + qr, P.nseg, c);
        sh_qm[lane] = qs.m;
        sh_qinvz[lane] = 1.0 / qs.z;
      }
      if (P.dbg_ratio) P.dbg_ratio[o + lane] = __builtin_nanf("");
    }
  }
  __syncthreads();
  if (tid < n) {
    const int x = sh_tok[tid], par = sh_par[tid];
    const int64_t prow = trow0 + 1 + par;
    const double lp = static_cast<double>(load_logit(P.target, P.t_dtype, prow * V + x));
    sh_px[tid] = exp2((lp - static_cast<double>(sh_tm[par + 1])) * static_cast<double>(c)) * sh_tinvz[par + 1];
    const int64_t qoff = static_cast<int64_t>(sh_qrow[tid]) * V + x;
    if (q_is_probs) sh_qx[tid] = static_cast<double>(load_logit(P.draft_q, P.q_dtype, qoff));
    else {
      const double lq = static_cast<double>(load_logit(P.draft_q, P.q_dtype, qoff));
      sh_qx[tid] = exp2((lq - static_cast<double>(sh_qm[tid])) * static_cast<double>(c)) * sh_qinvz[tid];
    }
  }
  __syncthreads();

  const int my_parent = (lane < n) ? sh_par[lane] : -2;   // lanes >= n hold an impossible parent

  int cur = -1, depth = 0;
  WalkRows R;
  R.t_base = P.target; R.t_dtype = P.t_dtype;
  R.q_base = P.draft_q; R.q_dtype = P.q_dtype; R.q_is_probs = q_is_probs;
  R.q_off = 0; R.q_m = 0.f; R.q_invz = 0.0; R.have_q = 0;

  // one full pass at residual level L: per-wave sums to LDS, returns the total
  auto full_pass = [&](int L) -> double {
    double acc = 0.0;
    const int e_begin = wave * seg_w;
    const int e_end = min(V, e_begin + seg_w);
    for (int e0 = e_begin + lane * 8; e0 < e_end; e0 += 512) {
      double w[8];
      weights8<VEC>(R, e0, V, c, L, sh_inv_R, w);
#pragma unroll
      for (int j = 0; j < 8; ++j) acc += w[j];
    }
    acc = wave_sum(acc);
    __syncthreads();                 // previous readers of sh_wave_sum are done
    if (lane == 0) sh_wave_sum[wave] = acc;
    __syncthreads();
    double tot = 0.0;
    for (int w = 0; w < kWalkWaves; ++w) tot += sh_wave_sum[w];
    return tot;
  };

  int level = 0;          // rejections so far at the current node
  int sums_level = -1;    // level whose per-wave sums sit in sh_wave_sum (-1: none)
  double total = 0.0;     // total of those sums

  for (int guard = 0; guard <= kMaxNodes; ++guard) {
    // target row of the current node
    R.t_off = (trow0 + 1 + cur) * static_cast<int64_t>(V);
    R.t_m = sh_tm[cur + 1];
    R.t_invz = sh_tinvz[cur + 1];
    level = 0;
    sums_level = -1;
    R.have_q = 0;

    unsigned long long kids = __ballot(my_parent == cur && lane > cur);
    int accepted = -1;
    while (kids) {
      const int ch = __ffsll(static_cast<long long>(kids)) - 1;
      kids &= kids - 1;
      if (!R.have_q) {
        R.q_off = static_cast<int64_t>(sh_qrow[ch]) * V;
        R.q_m = sh_qm[ch];
        R.q_invz = sh_qinvz[ch];
        R.have_q = 1;
      }
      const double qx = sh_qx[ch];
      double rx = sh_px[ch];
      for (int k = 0; k < level; ++k) {
        double w = rx - qx;
        w = w > 0.0 ? w : 0.0;
        rx = w * sh_inv_R[k];
      }
      double ratio;
      if (qx > 0.0) ratio = rx / qx;
      else ratio = (rx > 0.0) ? INFINITY : 0.0;
      if (P.dbg_ratio && tid == 0) P.dbg_ratio[o + ch] = static_cast<float>(ratio);
      const double u = static_cast<double>(sh_u[ch]);
      if (u < ratio) { accepted = ch; break; }
      // rejected: mass of max(0, r - q)
      const double mass = full_pass(level + 1);
      if (mass > 0.0) {
        __syncthreads();
        if (tid == 0) sh_inv_R[level] = 1.0 / mass;
        __syncthreads();
        ++level;
        sums_level = level;
        total = mass;
      } else {
        sums_level = -1;           // residual has no mass: r stays as it was
      }
    }
    if (accepted >= 0) {
      if (tid == 0 && depth < P.out_stride) P.out_tokens[static_cast<int64_t>(b) * P.out_stride + depth] = sh_tok[accepted];
      ++depth;
      cur = accepted;
      continue;
    }
    // no child, or every child rejected: draw from the level's weights by inverse CDF
    if (sums_level != level) { total = full_pass(level); sums_level = level; }
    const double target = static_cast<double>(P.u_resample[b]) * total;
    int ws = -1;
    double before = 0.0;
    for (int w = 0; w < kWalkWaves; ++w) {
      const double s = sh_wave_sum[w];
      if (before + s > target) { ws = w; break; }
      before += s;
    }
    if (ws < 0) {                    // rounding left no crossing: last wave with positive mass
      for (int w = kWalkWaves - 1; w >= 0; --w) if (sh_wave_sum[w] > 0.0) { ws = w; break; }
      if (ws < 0) ws = 0;
      before = 0.0;
      for (int w = 0; w < ws; ++w) before += sh_wave_sum[w];
    }
    if (tid == 0) sh_token = -1;
    __syncthreads();
    if (wave == ws) {
      const int e_begin = ws * seg_w;
      const int e_end = min(V, e_begin + seg_w);
      double run = before;
      int found = -1, last_pos = -1;
      for (int e_it = e_begin; e_it < e_end && found < 0; e_it += 512) {
        const int e0 = e_it + lane * 8;
        double w[8];
        if (e0 < e_end) weights8<VEC>(R, e0, V, c, level, sh_inv_R, w);
        else {
#pragma unroll
          for (int j = 0; j < 8; ++j) w[j] = 0.0;
        }
        double ls = 0.0;
        int my_last = -1;
#pragma unroll
        for (int j = 0; j < 8; ++j) { ls += w[j]; if (w[j] > 0.0) my_last = e0 + j; }
        // inclusive scan of lane sums
        double inc = ls;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
          const double t = __shfl_up(inc, d, kWave);
          if (lane >= d) inc += t;
        }
        const double it_total = __shfl(inc, 63, kWave);
        const unsigned long long cross = __ballot(run + inc > target);
        if (cross) {
          const int fl = __ffsll(static_cast<long long>(cross)) - 1;
          int tok = -1;
          if (lane == fl) {
            double acc = run + inc - ls;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
              acc += w[j];
              if (tok < 0 && acc > target && w[j] > 0.0) tok = e0 + j;
            }
            if (tok < 0) tok = my_last;      // rounding inside the lane: its last positive class
          }
          found = __shfl(tok, fl, kWave);
        }
        // remember the last class with positive weight seen so far
        int ml = my_last;
#pragma unroll
        for (int d = 32; d > 0; d >>= 1) ml = max(ml, __shfl_xor(ml, d, kWave));
        last_pos = max(last_pos, ml);
        run += it_total;
      }
      if (found < 0) found = last_pos >= 0 ? last_pos : min(V - 1, e_begin);
      if (lane == 0) sh_token = found;
    }
    __syncthreads();
    if (tid == 0 && depth < P.out_stride) P.out_tokens[static_cast<int64_t>(b) * P.out_stride + depth] = sh_token;
    break;
  }
  if (tid == 0) {
    P.accept_len[b] = depth;
    if (P.stop_node) P.stop_node[b] = cur;
  }
  for (int i = depth + 1 + tid; i < P.out_stride; i += kWalkThreads) P.out_tokens[static_cast<int64_t>(b) * P.out_stride + i] = -1;
}

size_t accept_workspace_bytes(int B, int total_nodes, int n_q_rows, int V) {
  const size_t rows = static_cast<size_t>(total_nodes) + B + n_q_rows;
  return rows * stats_segments(V) * sizeof(SegStat) + 256;
}

void launch_accept(const AcceptArgs& a, hipStream_t stream) {
  if (a.B <= 0) return;
  const float c = kLog2e / a.temperature;
  const int n_t_rows = a.total_nodes + a.B;
  const int n_q_stat_rows = (a.q_kind == 0) ? a.n_q_rows : 0;
  SegStat* stats = static_cast<SegStat*>(a.workspace);
  launch_row_stats(a.target, a.t_dtype, n_t_rows, a.draft_q, a.q_dtype, n_q_stat_rows, a.V, c, stats, stream);
  AcceptParams P;
  P.B = a.B; P.V = a.V; P.n_t_rows = n_t_rows; P.nseg = stats_segments(a.V);
  P.node_offsets = a.node_offsets; P.parent = a.parent; P.draft_tokens = a.draft_tokens;
  P.target = a.target; P.t_dtype = a.t_dtype;
  P.draft_q = a.draft_q; P.q_dtype = a.q_dtype; P.q_kind = a.q_kind;
  P.q_row = a.q_row; P.c = c; P.u_accept = a.u_accept; P.u_resample = a.u_resample;
  P.accept_len = a.accept_len; P.out_tokens = a.out_tokens; P.out_stride = a.out_stride;
  P.stop_node = a.stop_node; P.dbg_ratio = a.dbg_ratio; P.stats = stats;
  const bool vec = (a.V % 8 == 0);
  if (vec) hipLaunchKernelGGL(accept_walk_kernel<true>, dim3(a.B), dim3(kWalkThreads), 0, stream, P);
  else hipLaunchKernelGGL(accept_walk_kernel<false>, dim3(a.B), dim3(kWalkThreads), 0, stream, P);
}

}  // namespace specv
